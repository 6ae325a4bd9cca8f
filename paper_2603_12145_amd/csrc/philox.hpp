// Philox4x32-10 for gfx950, one counter block per lane, everything in registers.
// Definition: Salmon et al., "Parallel random numbers: as easy as 1, 2, 3" (SC'11).  The fused
// rollout (paper App. B.1 item 5) needs a generator without per-environment state so that the
// draw for (seed, env, step) is the same however the rollout is split into launches.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace envk {

struct Draw4 { uint32_t w0, w1, w2, w3; };

// The 32x32 -> 64 product is written as one 64-bit multiply so that the compiler can use a single
// v_mad_u64_u32 for both halves.
__device__ __forceinline__ void philox_round(uint32_t& c0, uint32_t& c1, uint32_t& c2, uint32_t& c3,
                                             uint32_t k0, uint32_t k1) {
  const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
  const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
  // a ^ b ^ c in one instruction (v_bitop3_b32 with the truth table of a three-way xor)
  const uint32_t t0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
  const uint32_t t2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
  c1 = (uint32_t)p1;
  c3 = (uint32_t)p0;
  c0 = t0;
  c2 = t2;
}

// counter = (env, step lo, step hi, stream), key = (seed lo, seed hi)
__device__ __forceinline__ Draw4 philox_draw(uint64_t seed, uint32_t env, uint64_t step,
                                             uint32_t stream) {
  uint32_t c0 = env, c1 = (uint32_t)step, c2 = (uint32_t)(step >> 32), c3 = stream;
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
  for (uint32_t r = 0; r < 10; ++r)
    philox_round(c0, c1, c2, c3, k0 + r * 0x9E3779B9u, k1 + r * 0xBB67AE85u);
  return Draw4{c0, c1, c2, c3};
}

// top 24 bits -> [0,1) on the 2^-24 grid (exact)
__device__ __forceinline__ float unit_float(uint32_t w) {
  return (float)(w >> 8) * 5.9604644775390625e-8f;
}
// top 24 bits -> (0,1]
__device__ __forceinline__ float unit_float_nonzero(uint32_t w) {
  return ((float)(w >> 8) + 1.0f) * 5.9604644775390625e-8f;
}

}  // namespace envk
