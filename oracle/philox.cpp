// TEST INFRASTRUCTURE — CPU oracle. Not part of the product path; shares no code with the HIP library.
//
// Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
// easy as 1, 2, 3", SC'11, section 3.3 / the Random123 definition) and the word -> draw mappings the
// environments use.  The paper's fused rollout relies on a stateless generator keyed by
// (seed, env, step) so that an environment's trajectory does not depend on batch size or on how the
// rollout is cut into launches (App. B.1 items 3 and 5: a pure single-instance step, vmapped, scanned).
//
// Keying used throughout this repo:
//   key     = (seed & 0xffffffff, seed >> 32)
//   counter = (env index, step & 0xffffffff, step >> 32, stream)
//   step    = number of env steps taken since creation (never rewound by episode ends)
//   stream  = 0 per-step block, 1 second per-step block, 16+b reset block b.
#include <cstdint>
#include <cmath>

namespace {

const uint32_t kMulA = 0xD2511F53u;   // multiplier applied to counter word 0
const uint32_t kMulB = 0xCD9E8D57u;   // multiplier applied to counter word 2
const uint32_t kWeylA = 0x9E3779B9u;  // key word 0 increment (golden ratio)
const uint32_t kWeylB = 0xBB67AE85u;  // key word 1 increment (sqrt(3)-1)

}  // namespace

extern "C" {

// out = Philox4x32-10(counter, key).
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {  // the key is bumped before every round but the first
      k0 += kWeylA;
      k1 += kWeylB;
    }
    const uint64_t pa = (uint64_t)kMulA * (uint64_t)c0;
    const uint64_t pb = (uint64_t)kMulB * (uint64_t)c2;
    const uint32_t hi_a = (uint32_t)(pa >> 32), lo_a = (uint32_t)pa;
    const uint32_t hi_b = (uint32_t)(pb >> 32), lo_b = (uint32_t)pb;
    const uint32_t n0 = hi_b ^ c1 ^ k0;
    const uint32_t n1 = lo_b;
    const uint32_t n2 = hi_a ^ c3 ^ k1;
    const uint32_t n3 = lo_a;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The block of four words an environment draws: (seed; env, step, stream).
void oracle_draw_block(uint64_t seed, uint32_t env, uint64_t step, uint32_t stream, uint32_t out[4]) {
  const uint32_t ctr[4] = {env, (uint32_t)(step & 0xffffffffu), (uint32_t)(step >> 32), stream};
  const uint32_t key[2] = {(uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32)};
  oracle_philox4x32_10(ctr, key, out);
}

// Uniform in [0,1): the top 24 bits scaled by 2^-24 (exact in float32).
float oracle_u01(uint32_t w) { return (float)(w >> 8) * 5.9604644775390625e-8f; }

// Uniform in (0,1]: used under the logarithm of the Box-Muller transform.
float oracle_u01_open0(uint32_t w) { return ((float)(w >> 8) + 1.0f) * 5.9604644775390625e-8f; }

// Pong action in {0,1,2}: multiply-high range reduction, floor(3 w / 2^32).
int32_t oracle_pong_action(uint32_t w) { return (int32_t)(((uint64_t)w * 3u) >> 32); }

// Pong serve x velocity: top bit set -> +3, else -3.
float oracle_pong_serve_vx(uint32_t w) { return (w >> 31) ? 3.0f : -3.0f; }

// Pong serve y velocity: uniform in [-2,2) on a 2^-22 grid (exact in float32).
float oracle_pong_serve_vy(uint32_t w) { return -2.0f + 4.0f * oracle_u01(w); }

// Uniform in [lo, hi): lo + (hi-lo)*u, float32, one multiply then one add.
float oracle_uniform(uint32_t w, float lo, float hi) { return lo + (hi - lo) * oracle_u01(w); }

// Box-Muller pair from two words (float32 library log/sqrt/cos/sin).
void oracle_normal_pair(uint32_t wa, uint32_t wb, float out[2]) {
  const float u1 = oracle_u01_open0(wa);
  const float u2 = oracle_u01(wb);
  const float radius = sqrtf(-2.0f * logf(u1));
  const float angle = 6.283185307179586f * u2;
  out[0] = radius * cosf(angle);
  out[1] = radius * sinf(angle);
}

}  // extern "C"
