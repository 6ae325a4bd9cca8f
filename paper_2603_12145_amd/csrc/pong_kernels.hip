// Pong with vector observations: reset and the fused T-step rollout (T = 1 is env_step).
//
// One lane per environment, one wavefront per 64 consecutive environments.  The state is read from
// the SoA arrays once, lives in VGPRs for all T steps (paper App. B.1 item 5: the rollout loop is
// fused into the kernel, no per-step dispatch), and is written back once.  Per step a wavefront
// emits: two 16-byte stores per lane for obs[t, i, 0:8], one dword per lane for reward[t, i], and
// the 64 done flags of the wavefront packed into 16 dwords (ballot -> byte spread), 37 bytes per
// environment step in total.  The kernel is a pure write stream; nothing is re-read.
#include "kernels.hpp"
#include "pong_device.hpp"

namespace envk {

namespace {

constexpr int WAVE = 64;
#ifndef MI355ENV_ROLLOUT_BLOCK
#define MI355ENV_ROLLOUT_BLOCK 64
#endif
constexpr int ROLLOUT_BLOCK = MI355ENV_ROLLOUT_BLOCK;   // threads per workgroup of the rollout kernel

__global__ __launch_bounds__(256) void pong_reset_kernel(uint32_t* __restrict__ state, int64_t n,
                                                         uint64_t seed, uint64_t step,
                                                         float* __restrict__ obs) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const PongLane s = pong_initial(seed, (uint32_t)i, step);
  pong_store(state, n, i, s);
  if (obs) {
    float4* o = reinterpret_cast<float4*>(obs + i * PONG_OBS);
    o[0] = make_float4(s.bx, s.by, s.vx, s.vy);
    o[1] = make_float4(s.pa, s.po, 0.0f, 0.0f);
  }
}

// bit k of `nibble` -> byte k of the result (0 or 1)
__device__ __forceinline__ uint32_t spread_nibble(uint32_t nibble) {
  return (nibble & 1u) | ((nibble & 2u) << 7) | ((nibble & 4u) << 14) | ((nibble & 8u) << 21);
}

template <bool PACK_DONE>
__global__ __launch_bounds__(ROLLOUT_BLOCK) void pong_rollout_kernel(PongLaunch a) {
  const int lane = threadIdx.x & (WAVE - 1);
  const int64_t i = (int64_t)blockIdx.x * ROLLOUT_BLOCK + threadIdx.x;
  const int64_t wave_base = i - lane;
  const bool live = i < a.n;
  const int64_t n = a.n;

  PongLane s = live ? pong_load(a.state, n, i) : pong_idle_lane();
  LaneEpisodes le;

  for (int32_t t = 0; t < a.T; ++t) {
    const uint64_t step = a.step0 + (uint64_t)t;
    const Draw4 d = philox_draw(a.seed, (uint32_t)i, step, 0u);
    const int64_t row = (int64_t)t * n;
    int action = pong_action_from_word(d.w0);
    if (a.actions) action = live ? (int)a.actions[row + i] : 0;

    const PongEvent ev = pong_transition(s, action, d.w1, d.w2, a.max_score);
    const bool done = live && ev.done;
    if (done) {
      le.count += 1;
      le.length_sum += ev.fin_len;
      le.ret_sum_i += ev.fin_ret;
      le.min_key = min(le.min_key, ev.fin_ret);
      le.max_key = max(le.max_key, ev.fin_ret);
    }

#ifdef MI355ENV_EXPERIMENT_NO_STORES
    if (live && a.T < 0) {
#else
    if (live) {
#endif
      float4* o = reinterpret_cast<float4*>(a.obs + (row + i) * PONG_OBS);
      o[0] = make_float4(s.bx, s.by, s.vx, s.vy);
      o[1] = make_float4(s.pa, s.po, (float)s.sa, (float)s.so);
      a.reward[row + i] = ev.reward;
    }
    if (PACK_DONE) {
      // n % 4 == 0 and done 4-byte aligned: every dword is entirely inside or outside the row
      const unsigned long long mask = __ballot(done);
      const int64_t first = wave_base + 4 * lane;
      if (lane < 16 && first < n) {
        const uint32_t nibble = (uint32_t)(mask >> (4 * lane)) & 0xFu;
        *reinterpret_cast<uint32_t*>(a.done + row + first) = spread_nibble(nibble);
      }
    } else if (live) {
      a.done[row + i] = done ? 1 : 0;
    }
  }

  if (live) pong_store(a.state, n, i, s);
  flush_wave_stats<false>(a.stats, le);
}

}  // namespace

hipError_t launch_pong_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step, float* obs,
                             hipStream_t stream) {
  const unsigned blocks = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(pong_reset_kernel, dim3(blocks), dim3(256), 0, stream, state, n, seed, step, obs);
  return hipGetLastError();
}

hipError_t launch_pong_rollout(const PongLaunch& a, hipStream_t stream) {
  const unsigned blocks = (unsigned)((a.n + ROLLOUT_BLOCK - 1) / ROLLOUT_BLOCK);
  const bool pack = (a.n % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.done) & 3u) == 0);
  if (pack)
    hipLaunchKernelGGL(pong_rollout_kernel<true>, dim3(blocks), dim3(ROLLOUT_BLOCK), 0, stream, a);
  else
    hipLaunchKernelGGL(pong_rollout_kernel<false>, dim3(blocks), dim3(ROLLOUT_BLOCK), 0, stream, a);
  return hipGetLastError();
}

}  // namespace envk
