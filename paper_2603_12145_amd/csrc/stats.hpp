// Per-batch episode statistics: per-lane accumulators are combined with a wave64 butterfly and one
// lane per wavefront issues the atomics, so the number of atomics is (waves that saw an episode
// end), not (episodes).  Integer sums make the Pong statistics independent of the order in which
// wavefronts retire.  The block is kept STATS_STRIPES times, one 128-byte line each, and a
// wavefront adds to the copy its index picks: atomics on one address go through one after the
// other (about 45 ns each), which for a per-step launch whose every wavefront sees an episode end
// (cart-pole with random actions, N = 65536: 1024 wavefronts x 5 atomics) was 55 of the step's
// 60 us.  Whoever reads the statistics adds the copies up.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace envk {

constexpr int STATS_STRIPES = 256;

struct alignas(128) DeviceStats {
  unsigned long long episodes;
  unsigned long long length_sum;
  long long return_sum_i;   // Pong: returns are integers
  double return_sum_f;      // body: float returns
  int return_min_key;       // Pong: the integer return; body: order-preserving key of the float
  int return_max_key;
  unsigned long long nonfinite;
};

template <class T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = min(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ int wave_max(int v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, 64));
  return v;
}

// monotone map float -> int (total order of finite floats)
__device__ __forceinline__ int float_order_key(float x) {
  const int b = __float_as_int(x);
  return b ^ ((b >> 31) & 0x7fffffff);
}

struct LaneEpisodes {
  int count = 0;
  int length_sum = 0;
  int ret_sum_i = 0;
  float ret_sum_f = 0.0f;
  int min_key = INT32_MAX;
  int max_key = INT32_MIN;
  int nonfinite = 0;
};

// Must be called by all 64 lanes of the wavefront (inactive environments pass empty accumulators).
// WAVES_PER_GROUP: the workgroup's size in wavefronts where the kernel knows it (a kernel launched
// without arguments must not ask for blockDim); 0 = ask.
template <bool FLOAT_RETURNS, int WAVES_PER_GROUP = 0>
__device__ __forceinline__ void flush_wave_stats(DeviceStats* __restrict__ stripes, const LaneEpisodes& le) {
  if (__ballot(le.count > 0 || le.nonfinite > 0) == 0ull) return;   // wave-uniform
  const unsigned waves = WAVES_PER_GROUP ? (unsigned)WAVES_PER_GROUP : (blockDim.x >> 6);
  DeviceStats* st = stripes + ((blockIdx.x * waves + (threadIdx.x >> 6)) & (STATS_STRIPES - 1));
  const long long cnt = wave_sum((long long)le.count);
  const long long len = wave_sum((long long)le.length_sum);
  const long long bad = wave_sum((long long)le.nonfinite);
  const int mn = wave_min(le.min_key);
  const int mx = wave_max(le.max_key);
  long long ri = 0;
  double rf = 0.0;
  if (FLOAT_RETURNS) rf = wave_sum((double)le.ret_sum_f);
  else ri = wave_sum((long long)le.ret_sum_i);
  if ((threadIdx.x & 63) == 0) {
    if (cnt) {
      atomicAdd(&st->episodes, (unsigned long long)cnt);
      atomicAdd(&st->length_sum, (unsigned long long)len);
      if (FLOAT_RETURNS) atomicAdd(&st->return_sum_f, rf);
      else atomicAdd((unsigned long long*)&st->return_sum_i, (unsigned long long)ri);
      atomicMin(&st->return_min_key, mn);
      atomicMax(&st->return_max_key, mx);
    }
    if (bad) atomicAdd(&st->nonfinite, (unsigned long long)bad);
  }
}

}  // namespace envk
