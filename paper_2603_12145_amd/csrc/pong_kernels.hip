// Pong with vector observations: reset and the fused T-step rollout (T = 1 is env_step).
//
// One lane per environment, one wavefront per 64 consecutive environments.  The state is read from
// the SoA arrays once, lives in VGPRs for all T steps (paper App. B.1 item 5: the rollout loop is
// fused into the kernel, no per-step dispatch), and is written back once.  Per step a wavefront
// emits: two 16-byte stores per lane for obs[t, i, 0:8], one dword per lane for reward[t, i] and
// one byte per lane for done[t, i], 37 bytes per environment step in total.  The kernel is a pure
// write stream; nothing is re-read.
#include "kernels.hpp"
#include "pong_device.hpp"

namespace envk {

namespace {

constexpr int WAVE = 64;
constexpr int ROLLOUT_BLOCK = 256;   // default threads per workgroup of the rollout kernel

__global__ __launch_bounds__(256) void pong_reset_kernel(uint32_t* __restrict__ state, int64_t n,
                                                         uint64_t seed, uint64_t host_step,
                                                         const StepCounter* __restrict__ counter,
                                                         float* __restrict__ obs, bool normalize) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint64_t step = read_step(counter, host_step);
  const PongLane s = pong_initial(seed, (uint32_t)i, step);
  pong_store(state, n, i, s);
  if (obs) {
    float4* o = reinterpret_cast<float4*>(obs + i * PONG_OBS);
    float4 lo, hi;
    if (normalize) pong_observe<true>(s, 0.0f, lo, hi);     // scores are 0 at a reset
    else pong_observe<false>(s, 0.0f, lo, hi);
    o[0] = lo;
    o[1] = hi;
  }
}

// One wavefront's T-step loop.  FULL: all 64 lanes own an environment (no per-lane predication in
// the loop).  Row pointers are wave-uniform and advance by one row per step.  The done flags go
// out as one byte per lane: the 64 bytes of a wavefront are contiguous, so the memory pipeline
// sees a single 64-byte write either way, and packing them by hand (ballot, shift, spread) only
// added ~25 instructions per step.
template <bool FULL, bool EXTERNAL_ACTIONS, bool NORMALIZE>
__device__ __forceinline__ void rollout_wave(const PongLaunch& a, PongLane& s, LaneEpisodes& le,
                                             const int lane, const int64_t wave_base) {
  const int64_t n = a.n;
  const uint32_t env = (uint32_t)(wave_base + lane);
  const bool live = FULL || (wave_base + lane < n);
  float* obs_row = a.obs + wave_base * PONG_OBS;
  float* rew_row = a.reward + wave_base;
  uint8_t* done_row = a.done + wave_base;
  const uint8_t* act_row = EXTERNAL_ACTIONS ? a.actions + wave_base : nullptr;

  Draw4 d = philox_draw(a.seed, env, a.step0, 0u);
  for (int32_t t = 0; t < a.T; ++t) {
    // draw of the next step first: it does not depend on the state, so its multiply chain
    // overlaps the compare/select chain of this step's transition
    const Draw4 d_next = philox_draw(a.seed, env, a.step0 + (uint64_t)t + 1u, 0u);
    int action;
    if (EXTERNAL_ACTIONS) action = live ? (int)act_row[lane] : 0;
    else action = pong_action_from_word(d.w0);

    const PongEvent ev = pong_transition(s, action, d.w1, d.w2, a.max_score);
    const bool done = live && ev.done;
    // selects, not a branch: the loop body stays one basic block, which lets the scheduler
    // interleave the next step's Philox rounds with this step's transition
    le.count += done ? 1 : 0;
    le.length_sum += done ? ev.fin_len : 0;
    le.ret_sum_i += done ? ev.fin_ret : 0;
    le.min_key = done ? min(le.min_key, ev.fin_ret) : le.min_key;
    le.max_key = done ? max(le.max_key, ev.fin_ret) : le.max_key;

    if (live) {
      float4* o = reinterpret_cast<float4*>(obs_row + lane * PONG_OBS);
      float4 lo, hi;
      pong_observe<NORMALIZE>(s, a.inv_score, lo, hi);
      o[0] = lo;
      o[1] = hi;
      rew_row[lane] = ev.reward;
      done_row[lane] = done ? 1 : 0;
    }
    obs_row += n * PONG_OBS;
    rew_row += n;
    done_row += n;
    if (EXTERNAL_ACTIONS) act_row += n;
    d = d_next;
  }
}

template <bool XCD_REMAP>
__global__ __launch_bounds__(256) void pong_rollout_kernel(PongLaunch a) {
  a.step0 = launch_first_step(a.counter, a.step0, a.T);
  const int lane = threadIdx.x & (WAVE - 1);
  // wave-uniform by construction; readfirstlane tells the compiler so (scalar address math)
  const int wave_in_block = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  // Workgroups are handed to the 8 XCDs round-robin by blockIdx.  Give XCD x the x-th contiguous
  // eighth of the environments (gridDim.x is a multiple of 8), so that every row of obs / reward /
  // done is written as 8 contiguous slices, each through a single L2, instead of being
  // interleaved across all eight at workgroup granularity.
  const unsigned per_xcd = gridDim.x >> 3;
  const unsigned logical_block = XCD_REMAP ? (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3) : blockIdx.x;
  const int64_t wave_base = ((int64_t)logical_block * (blockDim.x >> 6) + wave_in_block) * WAVE;
  const int64_t n = a.n;
  if (wave_base >= n) return;
  const int64_t i = wave_base + lane;
  const bool live = i < n;
  const bool full = wave_base + WAVE <= n;

  PongLane s = live ? pong_load(a.state, n, i) : pong_idle_lane();
  LaneEpisodes le;
  if (a.normalize) {                    // the optional form takes the general (predicated) loop
    if (a.actions) rollout_wave<false, true, true>(a, s, le, lane, wave_base);
    else rollout_wave<false, false, true>(a, s, le, lane, wave_base);
  } else if (a.actions) {
    if (full) rollout_wave<true, true, false>(a, s, le, lane, wave_base);
    else rollout_wave<false, true, false>(a, s, le, lane, wave_base);
  } else {
    if (full) rollout_wave<true, false, false>(a, s, le, lane, wave_base);
    else rollout_wave<false, false, false>(a, s, le, lane, wave_base);
  }
  if (live) pong_store(a.state, n, i, s);
  flush_wave_stats<false>(a.stats, le);
}

int g_rollout_block = 0;   // 0 = choose from N
int g_xcd_remap = 1;

}  // namespace

hipError_t launch_pong_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                             const StepCounter* counter, float* obs, bool normalize, hipStream_t stream) {
  const unsigned blocks = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(pong_reset_kernel, dim3(blocks), dim3(256), 0, stream, state, n, seed, step, counter,
                     obs, normalize);
  return hipGetLastError();
}

// Measurement knob: threads per workgroup of the rollout kernel (64, 128, 256; 0 = automatic).
bool set_rollout_block(int threads, int xcd_remap) {
  if (threads != 0 && threads != 64 && threads != 128 && threads != 256) return false;
  g_rollout_block = threads;
  g_xcd_remap = xcd_remap;
  return true;
}

hipError_t launch_pong_rollout(const PongLaunch& a, hipStream_t stream) {
  const int block = g_rollout_block ? g_rollout_block : ROLLOUT_BLOCK;
  unsigned blocks = (unsigned)((a.n + block - 1) / block);
  blocks = (blocks + 7u) & ~7u;   // multiple of the XCD count; surplus workgroups exit at once
  const dim3 g(blocks), b(block);
  if (g_xcd_remap) hipLaunchKernelGGL(pong_rollout_kernel<true>, g, b, 0, stream, a);
  else hipLaunchKernelGGL(pong_rollout_kernel<false>, g, b, 0, stream, a);
  return hipGetLastError();
}

}  // namespace envk
