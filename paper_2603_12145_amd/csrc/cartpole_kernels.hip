// CartPole: reset and the fused T-step rollout (T = 1 is env_step), one lane per environment.
// Third workload of the fused-rollout path (paper Table 8 and App. B.1 item 5 use a CartPole scan).
// Dynamics: the classic cart-pole (Barto, Sutton, Anderson 1983) in the usual parametrisation:
// cart 1.0 kg, pole 0.1 kg, half-length 0.5 m, g 9.8, force +-10 N, Euler step 0.02 s, failure at
// |x| > 2.4 or |theta| > 12 degrees, reward 1 per step, truncation at max_episode_steps.
// float32, -ffp-contract=off, every operation in the order written; sin / cos are the fixed
// degree-7 / degree-8 polynomials below (theta stays within +-0.21 rad during an episode), so a
// scalar CPU implementation of the same polynomials reproduces the trajectories bit for bit.
// Per step a lane writes one 16-byte obs, one reward dword and one done byte: 21 B per env-step.
#include "kernels.hpp"
#include "philox.hpp"

namespace envk {

namespace {

constexpr int WAVE = 64;

struct CartLane { float x, xd, th, thd; int ep_len; };

__device__ __forceinline__ float poly_sin(float x) {
  const float x2 = x * x;
  float p = -(1.0f / 5040.0f);
  p = p * x2; p = p + (1.0f / 120.0f);
  p = p * x2; p = p - (1.0f / 6.0f);
  p = p * x2; p = p + 1.0f;
  return x * p;
}
__device__ __forceinline__ float poly_cos(float x) {
  const float x2 = x * x;
  float p = 1.0f / 40320.0f;
  p = p * x2; p = p - (1.0f / 720.0f);
  p = p * x2; p = p + (1.0f / 24.0f);
  p = p * x2; p = p - 0.5f;
  p = p * x2; p = p + 1.0f;
  return p;
}

__device__ __forceinline__ CartLane cart_initial(uint64_t seed, uint32_t env, uint64_t step) {
  const Draw4 d = philox_draw(seed, env, step, 16u);
  CartLane s;
  s.x = -0.05f + 0.1f * unit_float(d.w0);
  s.xd = -0.05f + 0.1f * unit_float(d.w1);
  s.th = -0.05f + 0.1f * unit_float(d.w2);
  s.thd = -0.05f + 0.1f * unit_float(d.w3);
  s.ep_len = 0;
  return s;
}

// One Euler step of the dynamics in place; returns true if the episode ended (fin_len = its length).
__device__ __forceinline__ bool cart_advance(CartLane& s, int action, int max_steps, int& fin_len) {
  const float force = (action == 1) ? 10.0f : -10.0f;
  const float sn = poly_sin(s.th), cs = poly_cos(s.th);
  const float temp = (force + ((0.05f * s.thd) * s.thd) * sn) / 1.1f;
  const float denom = 0.5f * ((4.0f / 3.0f) - ((0.1f * cs) * cs) / 1.1f);
  const float thacc = (9.8f * sn - cs * temp) / denom;
  const float xacc = temp - ((0.05f * thacc) * cs) / 1.1f;
  s.x = s.x + 0.02f * s.xd;
  s.xd = s.xd + 0.02f * xacc;
  s.th = s.th + 0.02f * s.thd;
  s.thd = s.thd + 0.02f * thacc;
  s.ep_len += 1;
  const bool failed = (s.x < -2.4f) | (s.x > 2.4f) | (s.th < -0.20943951f) | (s.th > 0.20943951f);
  fin_len = s.ep_len;
  return failed | (s.ep_len >= max_steps);
}

// returns true if the episode ended (fin_len = its length); s is then the next episode's start
__device__ __forceinline__ bool cart_transition(CartLane& s, int action, int max_steps, uint64_t seed,
                                                uint32_t env, uint64_t step, int& fin_len) {
  const bool ended = cart_advance(s, action, max_steps, fin_len);
  // The reset draw is skipped only when no lane of the wavefront needs it (a wave-uniform branch:
  // under a random policy some lane ends an episode on almost every step, under a good policy
  // almost none does); within the branch every lane computes it and selects.
  if (__ballot(ended) != 0ull) {
    const CartLane fresh = cart_initial(seed, env, step + 1);
    s.x = ended ? fresh.x : s.x; s.xd = ended ? fresh.xd : s.xd;
    s.th = ended ? fresh.th : s.th; s.thd = ended ? fresh.thd : s.thd;
    s.ep_len = ended ? 0 : s.ep_len;
  }
  return ended;
}

__device__ __forceinline__ CartLane cart_load(const uint32_t* __restrict__ st, int64_t n, int64_t i) {
  CartLane s;
  s.x = __uint_as_float(st[0 * n + i]); s.xd = __uint_as_float(st[1 * n + i]);
  s.th = __uint_as_float(st[2 * n + i]); s.thd = __uint_as_float(st[3 * n + i]);
  s.ep_len = (int)st[5 * n + i];
  return s;
}
__device__ __forceinline__ void cart_store(uint32_t* __restrict__ st, int64_t n, int64_t i, const CartLane& s) {
  st[0 * n + i] = __float_as_uint(s.x); st[1 * n + i] = __float_as_uint(s.xd);
  st[2 * n + i] = __float_as_uint(s.th); st[3 * n + i] = __float_as_uint(s.thd);
  st[4 * n + i] = __float_as_uint((float)s.ep_len);      // return so far = steps so far
  st[5 * n + i] = (uint32_t)s.ep_len;
}

__global__ __launch_bounds__(256) void cartpole_reset_kernel(uint32_t* __restrict__ state, int64_t n,
                                                             uint64_t seed, uint64_t host_step,
                                                             const StepCounter* __restrict__ counter,
                                                             float* __restrict__ obs) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint64_t step = read_step(counter, host_step);
  const CartLane s = cart_initial(seed, (uint32_t)i, step);
  cart_store(state, n, i, s);
  if (obs) reinterpret_cast<float4*>(obs)[i] = make_float4(s.x, s.xd, s.th, s.thd);
}

// EXTERNAL_ACTIONS: one kernel per loop, so that each gets a register allocation and an instruction
// order of its own.
template <bool EXTERNAL_ACTIONS>
__global__ __launch_bounds__(256) void cartpole_rollout_kernel(PongLaunch a) {
  a.step0 = launch_first_step(a.counter, a.step0, a.T, a.ticket != 0);
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave_in_block = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  // XCD-aware mapping as in the Pong rollout: each XCD owns a contiguous eighth of the batch
  const unsigned per_xcd = gridDim.x >> 3;
  const unsigned logical_block = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  const int64_t wave_base = ((int64_t)logical_block * (blockDim.x >> 6) + wave_in_block) * WAVE;
  const int64_t n = a.n;
  if (wave_base >= n) return;
  const int64_t i = wave_base + lane;
  const bool live = i < n;
  const int64_t ic = live ? i : n - 1;
  CartLane s = cart_load(a.state, n, ic);
  LaneEpisodes le;
  float4* obs_row = reinterpret_cast<float4*>(a.obs) + wave_base;
  float* rew_row = a.reward + wave_base;
  uint8_t* done_row = a.done + wave_base;
  const uint8_t* act_row = EXTERNAL_ACTIONS ? a.actions + wave_base : nullptr;
  auto one_step = [&](const int32_t t, const int action) {
    const uint64_t step = a.step0 + (uint64_t)t;
    int fin_len;
    const bool ended = cart_transition(s, action, a.max_score, a.seed, (uint32_t)ic, step, fin_len);
    const bool done = live && ended;
    le.count += done ? 1 : 0;
    le.length_sum += done ? fin_len : 0;
    le.ret_sum_i += done ? fin_len : 0;
    le.min_key = done ? min(le.min_key, fin_len) : le.min_key;
    le.max_key = done ? max(le.max_key, fin_len) : le.max_key;
    if (live) {
      obs_row[lane] = make_float4(s.x, s.xd, s.th, s.thd);
      rew_row[lane] = 1.0f;
      done_row[lane] = done ? 1 : 0;
    }
    obs_row += n; rew_row += n; done_row += n;
  };
  if (!EXTERNAL_ACTIONS) {
    for (int32_t t = 0; t < a.T; ++t)
      one_step(t, (int)(philox_draw(a.seed, (uint32_t)ic, a.step0 + (uint64_t)t, 0u).w0 >> 31));
  } else {
    // External actions are fetched AHEAD steps before their use: a load issued in the step that
    // needs it leaves its whole latency exposed (0.95 against 0.53 ms at N = 65536 x T = 1000).
    // Every lane loads from a valid address (an idle lane its wavefront's first environment, a row
    // past the end the last row), so the loads stay unconditional.
    constexpr int AHEAD = 8;
    const int64_t act_lane = live ? lane : 0;
    auto fetch_action = [&](int32_t row) -> int {
      return (int)act_row[(int64_t)(row < a.T ? row : a.T - 1) * n + act_lane];
    };
    int pending[AHEAD];
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) pending[k] = fetch_action(k);
    // These first loads are waited for here, once.  Otherwise the compiler's wait-count
    // bookkeeping carries "just issued, nothing behind them" into the loop header, where it is
    // merged with the loop's own state, and every trip then waits for everything in flight,
    // stores included.  For the same reason the main loop has no branch inside a trip.
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) asm volatile("" : : "v"(pending[k]));
    asm volatile("" : : "v"(s.x), "v"(s.xd), "v"(s.th), "v"(s.thd), "v"(s.ep_len));   // the state's loads too
    int32_t t = 0;
    for (; t + AHEAD <= a.T; t += AHEAD) {
#pragma unroll
      for (int k = 0; k < AHEAD; ++k) {
        const int action = live ? pending[k] : 0;
        pending[k] = fetch_action(t + k + AHEAD);
        one_step(t + k, action);
      }
    }
    // fewer than AHEAD steps are left and their actions have been fetched
#pragma unroll
    for (int k = 0; k < AHEAD; ++k)
      if (t + k < a.T) one_step(t + k, live ? pending[k] : 0);     // wave-uniform
  }
  if (live) cart_store(a.state, n, i, s);
  flush_wave_stats<false>(a.stats, le);
}

// env_step (T = 1) as a kernel of its own, launched with its descriptor as a kernel argument or,
// in a steady loop, without any argument (see kernels.hpp).  Same arithmetic on the same words as
// the rollout loops.
template <bool EXTERNAL_ACTIONS>
__device__ __forceinline__ void cart_single_step(const PongLaunch& a, const uint64_t step) {
  const int64_t n = a.n;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const bool live = i < n;
  const int64_t ic = live ? i : n - 1;                          // idle lanes shadow the last environment
  const uint32_t word = EXTERNAL_ACTIONS ? 0u : philox_draw(a.seed, (uint32_t)ic, step, 0u).w0;
  CartLane s = cart_load(a.state, n, ic);
  const int action = EXTERNAL_ACTIONS ? (live ? (int)a.actions[ic] : 0) : (int)(word >> 31);
  int fin_len;
  const bool ended = cart_transition(s, action, a.max_score, a.seed, (uint32_t)ic, step, fin_len);
  const bool done = live && ended;
  LaneEpisodes le;
  if (done) { le.count = 1; le.length_sum = fin_len; le.ret_sum_i = fin_len; le.min_key = fin_len; le.max_key = fin_len; }
  if (live) {
    reinterpret_cast<float4*>(a.obs)[i] = make_float4(s.x, s.xd, s.th, s.thd);
    a.reward[i] = 1.0f;
    a.done[i] = done ? 1 : 0;
    cart_store(a.state, n, i, s);
  }
  flush_wave_stats<false, 4>(a.stats, le);
}

template <bool EXTERNAL_ACTIONS>
__global__ __launch_bounds__(256) void cartpole_step_kernel(PongLaunch a) {
  const uint64_t step = first_step_of_launch(a.counter, a.step0);
  cart_single_step<EXTERNAL_ACTIONS>(a, step);
  if (a.counter && a.ticket) finish_launch_steps(a.counter, step, 1, gridDim.x);
}

__device__ PongLaunch g_cart_step_records[STEP_RECORD_SLOTS];
__device__ unsigned long long g_cart_step_record_steps[STEP_RECORD_SLOTS][STEP_RECORD_MAX_GROUPS * 4];

template <int SLOT>
__global__ __launch_bounds__(256) void cartpole_step_resident_kernel() {
  PongLaunch a = g_cart_step_records[SLOT];
  a.state = known_global(a.state);
  a.actions = known_global(a.actions);
  a.obs = known_global(a.obs);
  a.reward = known_global(a.reward);
  a.done = known_global(a.done);
  a.stats = known_global(a.stats);
  unsigned long long* const mine = &g_cart_step_record_steps[SLOT][blockIdx.x * 4u + (threadIdx.x >> 6)];
  const unsigned long long s = *mine;
  const uint64_t step = ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(s >> 32)) << 32) |
                        __builtin_amdgcn_readfirstlane((uint32_t)s);
  if (a.actions) cart_single_step<true>(a, step);
  else cart_single_step<false>(a, step);
  if ((threadIdx.x & 63u) == 0u) *mine = step + 1;
}

// One workgroup of 256 threads: the record, and every wavefront's copy of the step index.
__global__ __launch_bounds__(256) void cart_step_record_write_kernel(int slot, PongLaunch a, unsigned long long step) {
  if (threadIdx.x == 0) g_cart_step_records[slot] = a;
  g_cart_step_record_steps[slot][threadIdx.x] = step;
}
static_assert(STEP_RECORD_MAX_GROUPS * 4 == 256, "cart_step_record_write_kernel writes one copy per thread");

template <int SLOT>
void launch_cart_resident(unsigned groups, hipStream_t stream) {
  hipLaunchKernelGGL(cartpole_step_resident_kernel<SLOT>, dim3(groups), dim3(256), 0, stream);
}

// Batches of at most one wavefront per SIMD (N <= 65536) with in-kernel actions: two wavefronts per
// 64 environments.  A lone wavefront on a SIMD issues an instruction every 5.4 cycles, two of them
// share the SIMD's issue slots at close to one every 4 (the same loop takes 0.438 ms per 1000
// steps at N = 65536 and 0.350 ms per 65536 environments at N = 131072).  Neither the action draw
// nor the reset draw depends on the state, so a second wavefront of the workgroup draws both
// Philox blocks of every step, CART_SPLIT_STEPS steps at a time, and hands five words per step
// over through LDS (the action bit and the four start values of the next episode, already scaled),
// two buffers taking turns, one workgroup barrier per hand-over; the first wavefront keeps the
// dynamics, the selects and the stores.  Both pass the same number of barriers.  Same arithmetic
// on the same words as the single-wavefront loop: identical results.
constexpr int CART_SPLIT_STEPS = 8;

template <bool FULL>
__global__ __launch_bounds__(128) void cartpole_split_rollout_kernel(PongLaunch a) {
  a.step0 = launch_first_step(a.counter, a.step0, a.T, a.ticket != 0);
  __shared__ uint32_t words[2][CART_SPLIT_STEPS][5][WAVE];   // 20 KiB
  const int lane = threadIdx.x & (WAVE - 1);
  const int producer = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform: 0 = the consumer
  const unsigned per_xcd = gridDim.x >> 3;
  const unsigned logical_block = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  const int64_t wave_base = (int64_t)logical_block * WAVE;
  const int64_t n = a.n;
  if (wave_base >= n) return;                                // the whole workgroup
  const int32_t rounds = (a.T + CART_SPLIT_STEPS - 1) / CART_SPLIT_STEPS;
  const int64_t i = wave_base + lane;
  const bool live = FULL || i < n;
  const int64_t ic = live ? i : n - 1;

  if (producer) {
    auto fill = [&](const int32_t round) {
#pragma unroll
      for (int k = 0; k < CART_SPLIT_STEPS; ++k) {
        const uint64_t step = a.step0 + (uint64_t)(round * CART_SPLIT_STEPS + k);
        const CartLane fresh = cart_initial(a.seed, (uint32_t)ic, step + 1);
        words[round & 1][k][0][lane] = philox_draw(a.seed, (uint32_t)ic, step, 0u).w0 >> 31;
        words[round & 1][k][1][lane] = __float_as_uint(fresh.x);
        words[round & 1][k][2][lane] = __float_as_uint(fresh.xd);
        words[round & 1][k][3][lane] = __float_as_uint(fresh.th);
        words[round & 1][k][4][lane] = __float_as_uint(fresh.thd);
      }
    };
    fill(0);
    __syncthreads();
    for (int32_t r = 0; r < rounds; ++r) {
      if (r + 1 < rounds) fill(r + 1);
      __syncthreads();
    }
    return;
  }

  CartLane s = cart_load(a.state, n, ic);
  LaneEpisodes le;
  float4* obs_row = reinterpret_cast<float4*>(a.obs) + wave_base;
  float* rew_row = a.reward + wave_base;
  uint8_t* done_row = a.done + wave_base;
  auto one_step = [&](const int round, const int k) {
    const int action = (int)words[round & 1][k][0][lane];
    const float fx = __uint_as_float(words[round & 1][k][1][lane]), fxd = __uint_as_float(words[round & 1][k][2][lane]);
    const float fth = __uint_as_float(words[round & 1][k][3][lane]), fthd = __uint_as_float(words[round & 1][k][4][lane]);
    int fin_len;
    const bool ended = cart_advance(s, action, a.max_score, fin_len);
    s.x = ended ? fx : s.x; s.xd = ended ? fxd : s.xd;
    s.th = ended ? fth : s.th; s.thd = ended ? fthd : s.thd;
    s.ep_len = ended ? 0 : s.ep_len;
    const bool done = live && ended;
    le.count += done ? 1 : 0;
    le.length_sum += done ? fin_len : 0;
    le.ret_sum_i += done ? fin_len : 0;
    le.min_key = done ? min(le.min_key, fin_len) : le.min_key;
    le.max_key = done ? max(le.max_key, fin_len) : le.max_key;
    if (live) {
      obs_row[lane] = make_float4(s.x, s.xd, s.th, s.thd);
      rew_row[lane] = 1.0f;
      done_row[lane] = done ? 1 : 0;
    }
    obs_row += n; rew_row += n; done_row += n;
  };
  __syncthreads();
  for (int32_t r = 0; r < rounds; ++r) {
    const int32_t t = r * CART_SPLIT_STEPS;
    if (t + CART_SPLIT_STEPS <= a.T) {                        // wave-uniform
#pragma unroll
      for (int k = 0; k < CART_SPLIT_STEPS; ++k) one_step(r, k);
    } else {
      for (int k = 0; t + k < a.T; ++k) one_step(r, k);
    }
    __syncthreads();
  }
  if (live) cart_store(a.state, n, i, s);
  flush_wave_stats<false>(a.stats, le);
}

int g_cartpole_split = 0;   // 0 = chosen from N and T, 1 = never, 2 = whenever the launch has in-kernel actions

}  // namespace

bool set_cartpole_split(int mode) {
  if (mode < 0 || mode > 2) return false;
  g_cartpole_split = mode;
  return true;
}

hipError_t launch_cartpole_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                                 const StepCounter* counter, float* obs, hipStream_t stream) {
  hipLaunchKernelGGL(cartpole_reset_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, state, n,
                     seed, step, counter, obs);
  return hipGetLastError();
}

// a.max_score carries max_episode_steps
hipError_t launch_cartpole_rollout(const PongLaunch& a, hipStream_t stream, StepResident* resident) {
  unsigned blocks = (unsigned)((a.n + 255) / 256);
  PongLaunch a2 = a;
  if (a.T == 1 && step_kernel_mode() != 0) {
    hipError_t re = hipSuccess;
    if (resident_step_try(
            resident, a, blocks, stream,
            [&](int slot, const PongLaunch& rec, unsigned long long step) {
              hipLaunchKernelGGL(cart_step_record_write_kernel, dim3(1), dim3(256), 0, stream, slot, rec, step);
            },
            [&](int slot, unsigned groups) {
              switch (slot) {
                case 0: launch_cart_resident<0>(groups, stream); break;
                case 1: launch_cart_resident<1>(groups, stream); break;
                case 2: launch_cart_resident<2>(groups, stream); break;
                default: launch_cart_resident<3>(groups, stream); break;
              }
              static_assert(STEP_RECORD_SLOTS == 4, "one case per record");
            },
            &re))
      return re;
    a2.ticket = blocks <= TICKET_MAX_BLOCKS;
    if (a.actions) hipLaunchKernelGGL(cartpole_step_kernel<true>, dim3(blocks), dim3(256), 0, stream, a2);
    else hipLaunchKernelGGL(cartpole_step_kernel<false>, dim3(blocks), dim3(256), 0, stream, a2);
    const hipError_t e = hipGetLastError();
    return e != hipSuccess ? e : advance_step_counter_behind(a.counter, 1, blocks, stream);
  }
  blocks = (blocks + 7u) & ~7u;
  const bool split = !a.actions && (g_cartpole_split == 2 ||
                                    (g_cartpole_split == 0 && a.n <= 65536 && a.T >= 4 * CART_SPLIT_STEPS));
  if (split) {
    unsigned wgs = (unsigned)((a.n + WAVE - 1) / WAVE);
    wgs = (wgs + 7u) & ~7u;
    a2.ticket = wgs <= TICKET_MAX_BLOCKS;
    if (a.n % WAVE == 0) hipLaunchKernelGGL(cartpole_split_rollout_kernel<true>, dim3(wgs), dim3(128), 0, stream, a2);
    else hipLaunchKernelGGL(cartpole_split_rollout_kernel<false>, dim3(wgs), dim3(128), 0, stream, a2);
    const hipError_t e = hipGetLastError();
    return e != hipSuccess ? e : advance_step_counter_behind(a.counter, a.T, wgs, stream);
  }
  a2.ticket = blocks <= TICKET_MAX_BLOCKS;
  if (a.actions) hipLaunchKernelGGL(cartpole_rollout_kernel<true>, dim3(blocks), dim3(256), 0, stream, a2);
  else hipLaunchKernelGGL(cartpole_rollout_kernel<false>, dim3(blocks), dim3(256), 0, stream, a2);
  const hipError_t err = hipGetLastError();
  return err != hipSuccess ? err : advance_step_counter_behind(a.counter, a.T, blocks, stream);
}

}  // namespace envk
