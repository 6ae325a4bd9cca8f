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

#include <atomic>
#include <mutex>
#include <vector>

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
//
// The Philox blocks are drawn CHUNK steps at a time, one chunk ahead: the draws do not depend on
// the state, so the 2 * CHUNK multiply chains of a chunk are independent of each other and of the
// compare/select chains of the transitions they are scheduled between.  With one wavefront per
// SIMD (N = 65536) nothing else hides the latency of a dependent chain.
//
// PAGED (needs a full 256-thread workgroup, see the kernel): the 32-byte observation of a lane is
// handed through LDS so that each of the two store instructions of a step covers 1 KiB of
// contiguous memory per wavefront and the four wavefronts of a workgroup write one 4 KiB page after
// the other, instead of two half-dense instructions per wavefront over its own 2 KiB.
//
// PACED: a chunk starts no sooner than a.pace after the previous one, by the constant 100 MHz
// clock.  Left alone, the wavefronts of a launch of 61440 environments or more issue their stores
// faster than the memory system drains them; the stores queue, the wavefronts drift apart over
// many rows of the trajectory arrays, and the write stream settles at 5.4 TB/s instead of 6.4.
// LEAN: see PongBooks.
template <bool FULL, bool EXTERNAL_ACTIONS, bool NORMALIZE, bool PAGED, int CHUNK = 4, bool LEAN = false, bool PACED = false>
__device__ __forceinline__ void rollout_wave(const PongLaunch& a, PongLane& s, LaneEpisodes& le,
                                             const int lane, const int64_t wave_base,
                                             float4* __restrict__ stage, const int64_t block_base) {
  const int64_t n = a.n;
  const uint32_t env = (uint32_t)(wave_base + lane);
  const bool live = FULL || (wave_base + lane < n);
  float* obs_row = a.obs + (PAGED ? block_base : wave_base) * PONG_OBS;
  float* rew_row = a.reward + wave_base;
  uint8_t* done_row = a.done + wave_base;
  const uint8_t* act_row = EXTERNAL_ACTIONS ? a.actions + wave_base : nullptr;
  int parity = 0;
  const uint32_t obs_off = (uint32_t)lane * (PONG_OBS * 4u), rew_off = (uint32_t)lane * 4u, done_off = (uint32_t)lane;

  // External actions are fetched two chunks ahead of their use (as the Philox blocks are drawn one
  // chunk ahead): a load issued in the step that needs it leaves its whole latency exposed, which
  // doubled the launch (0.95 against 0.44 ms at N = 65536 x T = 1000; fetched ahead: 0.46).
  // Every lane loads from a valid address -- an idle lane its wavefront's first environment, a row
  // past the end the last row -- so that the loads stay unconditional.
  const int64_t act_lane = live ? lane : 0;
  auto fetch_action = [&](int32_t row) -> int {
    return EXTERNAL_ACTIONS ? (int)act_row[(int64_t)(row < a.T ? row : a.T - 1) * n + act_lane] : 0;
  };

  // Episode bookkeeping.  Plain: every step adds to the lane's statistics with selects (no branch:
  // the steps of a chunk stay one basic block).  LEAN: an episode's end only leaves a mark in a
  // step and is added to the statistics at the next flush, once per chunk; eight vector
  // instructions fewer per step, which pays where the launch is bound by instruction issue.
  PongBooks books = pong_books_open(s);

  auto one_step = [&](const Draw4& d, const int action, const uint32_t steps_taken) {
    float move;
    if (EXTERNAL_ACTIONS) move = pong_move_of_action(live ? action : 0);
    else move = pong_move_of_word(d.w0);
    float reward;
    bool done;
    if constexpr (LEAN) {
      bool ended;
      reward = pong_transition_booked(s, books, move, d.w1, d.w2, a.max_score, steps_taken, ended).reward;
      done = live && ended;
    } else {
      const PongEvent ev = pong_transition_move(s, move, d.w1, d.w2, a.max_score);
      reward = ev.reward;
      done = live && ev.done;
      le.count += done ? 1 : 0;
      le.length_sum += done ? ev.fin_len : 0;
      le.ret_sum_i += done ? ev.fin_ret : 0;
      le.min_key = done ? min(le.min_key, ev.fin_ret) : le.min_key;
      le.max_key = done ? max(le.max_key, ev.fin_ret) : le.max_key;
    }
    float4 lo, hi;
    pong_observe<NORMALIZE>(s, a.inv_score, lo, hi);
    if (PAGED) {
      // two buffers, one barrier per step: a thread reaches the barrier of step t+1 only after
      // its reads of step t have landed (the global stores below need them), so the buffer of
      // step t is free again when step t+2 writes it
      float4* st = stage + parity * 512;
      st[2 * threadIdx.x] = lo;
      st[2 * threadIdx.x + 1] = hi;
      __syncthreads();
      const float4 p0 = st[threadIdx.x], p1 = st[256 + threadIdx.x];
      float4* o = reinterpret_cast<float4*>(obs_row);
      o[threadIdx.x] = p0;
      o[256 + threadIdx.x] = p1;
      parity ^= 1;
      rew_row[lane] = reward;
      done_row[lane] = done ? 1 : 0;
    } else if (live) {
      float4* o = reinterpret_cast<float4*>(reinterpret_cast<char*>(obs_row) + obs_off);
      o[0] = lo;
      o[1] = hi;
      *reinterpret_cast<float*>(reinterpret_cast<char*>(rew_row) + rew_off) = reward;
      done_row[done_off] = done ? 1 : 0;
    }
    obs_row += n * PONG_OBS;
    rew_row += n;
    done_row += n;
  };

  // PACED: the chunks of a wavefront start no closer together than a.pace (in 1/256 of a tick of
  // the 100 MHz constant clock)
  const uint32_t period = PACED ? (uint32_t)a.pace : 0u;
  uint32_t slot = PACED ? ((uint32_t)__builtin_amdgcn_s_memrealtime() << 8) : 0u;
  int32_t t = 0;
  static_assert(!LEAN || CHUNK <= 8, "a lane may end at most one episode between two flushes");
  if (a.T >= CHUNK) {
    Draw4 cur[CHUNK];
#pragma unroll
    for (int c = 0; c < CHUNK; ++c) cur[c] = philox_draw(a.seed, env, a.step0 + (uint64_t)c, 0u);
    // one chunk: draw the next chunk's Philox blocks, take this chunk's steps with the actions in
    // `use`, and (external actions) start the loads of the chunk after next into `fill`
    auto chunk = [&](const int (&use)[CHUNK], int (&fill)[CHUNK]) {
      // the previous chunk's episode ends, here rather than behind its steps: the branch then sits
      // where the loop's own branch already ends the basic block, and draws and steps stay together
      if constexpr (LEAN) pong_books_flush(books, le, live);
      if constexpr (PACED) {
        // wave-uniform and scalar throughout (32-bit clock arithmetic: the differences are small,
        // so wrap-around is harmless); ends: the clock advances, and the looks at it are capped
        uint32_t now = (uint32_t)__builtin_amdgcn_s_memrealtime() << 8;
        for (int look = 0; look < 64 && (int32_t)(now - slot) < 0; ++look) {
          __builtin_amdgcn_s_sleep(1);
          now = (uint32_t)__builtin_amdgcn_s_memrealtime() << 8;
        }
        // a late wavefront does not catch up in a burst
        slot = ((int32_t)(now - slot) > (int32_t)period ? now : slot) + period;
      }
      Draw4 nxt[CHUNK];
#pragma unroll
      for (int c = 0; c < CHUNK; ++c) {
        nxt[c] = philox_draw(a.seed, env, a.step0 + (uint64_t)(t + CHUNK + c), 0u);
        fill[c] = fetch_action(t + 2 * CHUNK + c);
      }
#pragma unroll
      for (int c = 0; c < CHUNK; ++c) one_step(cur[c], use[c], (uint32_t)(t + c + 1));
#pragma unroll
      for (int c = 0; c < CHUNK; ++c) cur[c] = nxt[c];
      t += CHUNK;
    };
    if (EXTERNAL_ACTIONS) {
      // Three sets of action registers take turns (in use, loaded, being loaded), three chunks per
      // trip, so that no set is ever copied into another: a copy would make the wavefront wait for
      // a load it has only just issued, and with it (memory operations complete in order) for
      // every store before that.
      int s0[CHUNK], s1[CHUNK], s2[CHUNK];
#pragma unroll
      for (int c = 0; c < CHUNK; ++c) {
        s0[c] = fetch_action(c);
        s1[c] = fetch_action(CHUNK + c);
      }
      // These first loads are waited for here, once, before the loop.  Otherwise the compiler's
      // wait-count bookkeeping carries "just issued, nothing behind them" into the loop header,
      // where it is merged with the loop's own state, and every trip then begins by waiting for
      // everything in flight, stores included (0.63 ms at N = 65536 x T = 1000).
#pragma unroll
      for (int c = 0; c < CHUNK; ++c) asm volatile("" : : "v"(s0[c]), "v"(s1[c]));
      while (t + 3 * CHUNK <= a.T) {
        chunk(s0, s2);
        chunk(s1, s0);
        chunk(s2, s1);
      }
      // at most two whole chunks are left; s0 and s1 hold their actions
      if (t + CHUNK <= a.T) chunk(s0, s2);
      if (t + CHUNK <= a.T) chunk(s1, s0);
    } else {
      int none[CHUNK] = {}, sink[CHUNK];
      while (t + CHUNK <= a.T) chunk(none, sink);
    }
  }
  if constexpr (LEAN) pong_books_flush(books, le, live);
  for (; t < a.T; ++t) {
    one_step(philox_draw(a.seed, env, a.step0 + (uint64_t)t, 0u), fetch_action(t), (uint32_t)(t + 1));
    if constexpr (LEAN) pong_books_flush(books, le, live);
  }
  if constexpr (LEAN) pong_books_close(s, books, le, (uint32_t)a.T, live);
}

// Every variant of the main loop is a kernel of its own: inlined into one kernel they share a
// register allocation and a scheduling budget, and the order the compiler picks for one loop then
// depends on which other loops exist (the same source ran between 0.40 and 0.44 ms at N = 65536).
// A kernel holds its loop for full wavefronts and the general loop for a ragged last wavefront.
enum RolloutVariant {
  V_RAW_2, V_RAW_4, V_RAW_8,   // in-kernel actions, raw observations, direct stores; steps per chunk
  V_PACED,                     // ... two steps per chunk, lean bookkeeping, chunks keep to a clock
  V_PAGED,                     // ... with observation stores paged through LDS
  V_EXTERNAL,                  // external actions, raw observations
  V_EXTERNAL_PACED,            // ... lean bookkeeping, chunks keep to a clock
  V_NORMALIZED, V_NORMALIZED_EXTERNAL,
  V_NORMALIZED_PACED           // normalised observations in the paced loop
};

// TRIAL changes nothing but the kernel's name: the launches with which the launcher measures, once
// per device and batch size, whether pacing pays (see launch_pong_rollout) show up on their own
// line in a kernel trace instead of being mixed with the launches a caller asked for.
template <int VARIANT, bool TRIAL = false>
__global__ __launch_bounds__(256) void pong_rollout_kernel(PongLaunch a) {
  a.step0 = launch_first_step(a.counter, a.step0, a.T, a.ticket != 0);
  const int lane = threadIdx.x & (WAVE - 1);
  // wave-uniform by construction; readfirstlane tells the compiler so (scalar address math)
  const int wave_in_block = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  // Workgroups are handed to the 8 XCDs round-robin by blockIdx.  Give XCD x the x-th contiguous
  // eighth of the environments (gridDim.x is a multiple of 8), so that every row of obs / reward /
  // done is written as 8 contiguous slices, each through a single L2, instead of being
  // interleaved across all eight at workgroup granularity.
  const unsigned per_xcd = gridDim.x >> 3;
  const unsigned logical_block = a.xcd_remap ? (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3) : blockIdx.x;
  const int64_t wave_base = ((int64_t)logical_block * (blockDim.x >> 6) + wave_in_block) * WAVE;
  const int64_t n = a.n;
  if (wave_base >= n) return;
  const int64_t i = wave_base + lane;
  const bool live = i < n;
  const bool full = wave_base + WAVE <= n;

  PongLane s = live ? pong_load(a.state, n, i) : pong_idle_lane();
  LaneEpisodes le;
  // paged stores need every thread of a 256-thread workgroup at the barrier of every step
  __shared__ float4 stage[VARIANT == V_PAGED ? 2 * 512 : 1];
  const int64_t block_base = (int64_t)logical_block * blockDim.x;
  constexpr bool EXTERNAL = VARIANT == V_EXTERNAL || VARIANT == V_EXTERNAL_PACED || VARIANT == V_NORMALIZED_EXTERNAL;
  constexpr bool NORMALIZE = VARIANT == V_NORMALIZED || VARIANT == V_NORMALIZED_EXTERNAL || VARIANT == V_NORMALIZED_PACED;
  if (VARIANT == V_PAGED && blockDim.x == 256 && block_base + 256 <= n) {       // workgroup-uniform
    rollout_wave<true, false, false, true, 4>(a, s, le, lane, wave_base, stage, block_base);
  } else if (full && VARIANT == V_NORMALIZED_PACED) {
    rollout_wave<true, false, true, false, 2, true, true>(a, s, le, lane, wave_base, stage, block_base);
  } else if (full && !NORMALIZE) {
    // external actions: 8, so that the loads run 8 to 16 steps ahead of their use (4: 0.69 ms at
    // N = 65536 x T = 1000, 8: 0.46 ms) -- a load queues behind the wavefront's own stores
    constexpr int CHUNK = (VARIANT == V_RAW_2 || VARIANT == V_PACED) ? 2 : (VARIANT == V_RAW_8 || EXTERNAL) ? 8 : 4;
    constexpr bool PACED = VARIANT == V_PACED || VARIANT == V_EXTERNAL_PACED;
    rollout_wave<true, EXTERNAL, false, false, CHUNK, PACED, PACED>(a, s, le, lane, wave_base, stage, block_base);
  } else {                              // ragged wavefront; the normalised form always
    rollout_wave<false, EXTERNAL, NORMALIZE, false, 4>(a, s, le, lane, wave_base, stage, block_base);
  }
  if (live) pong_store(a.state, n, i, s);
  flush_wave_stats<false>(a.stats, le);
}

// env_step (T = 1) as a kernel of its own: the step and nothing else, launched with its
// descriptor as a kernel argument (pong_step_kernel) or, in a steady loop, without any argument
// (pong_step_resident_kernel; see kernels.hpp for why and when).  Both run pong_single_step: same
// results, bit for bit.  N = 4096: 3.1 us per step without arguments (device-bound), 3.8-4.6 us
// with (host-bound).
template <bool EXTERNAL_ACTIONS, bool NORMALIZE>
__device__ __forceinline__ void pong_single_step(const PongLaunch& a, const uint64_t step) {
  const int64_t n = a.n;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const bool live = i < n;
  const int64_t ic = live ? i : n - 1;                          // idle lanes shadow the last environment
  // the draw does not depend on the state: its multiply chain runs under the state's loads
  const Draw4 d = philox_draw(a.seed, (uint32_t)ic, step, 0u);
  PongLane s = pong_load(a.state, n, ic);
  const float move = EXTERNAL_ACTIONS ? pong_move_of_action((int)a.actions[ic]) : pong_move_of_word(d.w0);
  const PongEvent ev = pong_transition_move(s, move, d.w1, d.w2, a.max_score);
  const bool done = live && ev.done;
  LaneEpisodes le;
  if (done) { le.count = 1; le.length_sum = ev.fin_len; le.ret_sum_i = ev.fin_ret; le.min_key = ev.fin_ret; le.max_key = ev.fin_ret; }
  if (live) {
    float4 lo, hi;
    pong_observe<NORMALIZE>(s, a.inv_score, lo, hi);
    float4* o = reinterpret_cast<float4*>(a.obs + i * PONG_OBS);
    o[0] = lo;
    o[1] = hi;
    a.reward[i] = ev.reward;
    a.done[i] = done ? 1 : 0;
    pong_store(a.state, n, i, s);
  }
  flush_wave_stats<false, 4>(a.stats, le);
}

template <bool EXTERNAL_ACTIONS, bool NORMALIZE>
__global__ __launch_bounds__(256) void pong_step_kernel(PongLaunch a) {
  const uint64_t step = first_step_of_launch(a.counter, a.step0);
  pong_single_step<EXTERNAL_ACTIONS, NORMALIZE>(a, step);
  if (a.counter && a.ticket) finish_launch_steps(a.counter, step, 1, gridDim.x);
}

struct StepRecord {
  PongLaunch a;        // step0, counter and ticket are not used
};
__device__ StepRecord g_step_records[STEP_RECORD_SLOTS];
// The record's step index, one copy per wavefront of the launch: a wavefront reads its own copy
// at the start and writes copy + 1 at the end, so no wavefront waits for another and nothing is
// atomic.  Every copy moves by one per launch; the host rewrites them all when it rewrites the record.
__device__ unsigned long long g_step_record_steps[STEP_RECORD_SLOTS][STEP_RECORD_MAX_GROUPS * 4];

template <int SLOT>
__global__ __launch_bounds__(256) void pong_step_resident_kernel() {
  PongLaunch a = g_step_records[SLOT].a;
  a.state = known_global(a.state);
  a.actions = known_global(a.actions);
  a.obs = known_global(a.obs);
  a.reward = known_global(a.reward);
  a.done = known_global(a.done);
  a.stats = known_global(a.stats);
  unsigned long long* const mine = &g_step_record_steps[SLOT][blockIdx.x * 4u + (threadIdx.x >> 6)];
  const unsigned long long s = *mine;
  const uint64_t step = ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(s >> 32)) << 32) |
                        __builtin_amdgcn_readfirstlane((uint32_t)s);
  if (a.actions) {
    if (a.normalize) pong_single_step<true, true>(a, step);
    else pong_single_step<true, false>(a, step);
  } else {
    if (a.normalize) pong_single_step<false, true>(a, step);
    else pong_single_step<false, false>(a, step);
  }
  if ((threadIdx.x & 63u) == 0u) *mine = step + 1;
}

// One workgroup of 256 threads: the record, and every wavefront's copy of the step index.
__global__ __launch_bounds__(256) void step_record_write_kernel(int slot, PongLaunch a, unsigned long long step) {
  if (threadIdx.x == 0) g_step_records[slot].a = a;
  g_step_record_steps[slot][threadIdx.x] = step;
}
static_assert(STEP_RECORD_MAX_GROUPS * 4 == 256, "step_record_write_kernel writes one copy per thread");

// Small batches (fewer wavefronts than SIMDs): two wavefronts per 64 environments.  A launch of
// 16384 environments occupies a quarter of the device's SIMDs.  The Philox draws do not depend on
// the state, so a second wavefront (on another SIMD of the same CU) draws them, SPLIT_STEPS steps
// at a time, and hands the three words a step uses to the first through LDS, two buffers taking
// turns, one workgroup barrier per hand-over.  The first wavefront is left with the transitions
// and the stores.  Both wavefronts pass the same number of barriers (1 + ceil(T / SPLIT_STEPS));
// the buffer the producer fills in a round is the one the consumer finished with before the
// previous barrier.  N <= 16384 (one workgroup per CU): 0.245 against 0.307 ms per 1000 steps; up
// to N = 32768, where CUs hold two workgroups: 0.30-0.31 against 0.311, so the launcher stops at
// 16384.  A second producer changes nothing: what is left is the dependent chain of the
// transition itself (paddles, flight, hits, point, scores, episode end), about 590 cycles per
// step for 75 instructions; and giving the consumer two sets of environments to take side by side
// only serialises what idle SIMDs would do in parallel (0.44 ms).
constexpr int SPLIT_STEPS = 8;

template <bool FULL>
__global__ __launch_bounds__(128) void pong_split_rollout_kernel(PongLaunch a) {
  a.step0 = launch_first_step(a.counter, a.step0, a.T, a.ticket != 0);
  __shared__ uint32_t words[2][SPLIT_STEPS][3][WAVE];   // 12 KiB
  const int lane = threadIdx.x & (WAVE - 1);
  const int producer = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // wave-uniform: 0 = the consumer
  const unsigned per_xcd = gridDim.x >> 3;
  const unsigned logical_block = a.xcd_remap ? (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3) : blockIdx.x;
  const int64_t wave_base = (int64_t)logical_block * WAVE;
  const int64_t n = a.n;
  if (wave_base >= n) return;                             // the whole workgroup
  const int32_t rounds = (a.T + SPLIT_STEPS - 1) / SPLIT_STEPS;

  if (producer) {
    const uint32_t env = (uint32_t)(wave_base + lane);    // lanes past the end draw blocks nobody reads
    auto fill = [&](const int32_t round) {
#pragma unroll
      for (int k = 0; k < SPLIT_STEPS; ++k) {
        const Draw4 d = philox_draw(a.seed, env, a.step0 + (uint64_t)(round * SPLIT_STEPS + k), 0u);
        words[round & 1][k][0][lane] = d.w0;
        words[round & 1][k][1][lane] = d.w1;
        words[round & 1][k][2][lane] = d.w2;
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

  const int64_t i = wave_base + lane;
  const bool live = FULL || i < n;
  PongLane s = live ? pong_load(a.state, n, i) : pong_idle_lane();
  LaneEpisodes le;
  PongBooks books = pong_books_open(s);
  float* obs_row = a.obs + wave_base * PONG_OBS;
  float* rew_row = a.reward + wave_base;
  uint8_t* done_row = a.done + wave_base;
  auto one_step = [&](const int round, const int k, const uint32_t steps_taken) {
    const uint32_t w0 = words[round & 1][k][0][lane], w1 = words[round & 1][k][1][lane],
                   w2 = words[round & 1][k][2][lane];
    bool ended;
    const PongFlight ev = pong_transition_booked(s, books, pong_move_of_word(w0), w1, w2, a.max_score,
                                                 steps_taken, ended);
    const bool done = live && ended;
    if (live) {
      float4 lo, hi;
      pong_observe<false>(s, 0.0f, lo, hi);
      float4* o = reinterpret_cast<float4*>(obs_row + lane * PONG_OBS);
      o[0] = lo;
      o[1] = hi;
      rew_row[lane] = ev.reward;
      done_row[lane] = done ? 1 : 0;
    }
    obs_row += n * PONG_OBS;
    rew_row += n;
    done_row += n;
  };
  __syncthreads();
  for (int32_t r = 0; r < rounds; ++r) {
    const int32_t t = r * SPLIT_STEPS;
    if (t + SPLIT_STEPS <= a.T) {                         // wave-uniform
#pragma unroll
      for (int k = 0; k < SPLIT_STEPS; ++k) one_step(r, k, (uint32_t)(t + k + 1));
    } else {
      for (int k = 0; t + k < a.T; ++k) one_step(r, k, (uint32_t)(t + k + 1));
    }
    pong_books_flush(books, le, live);
    __syncthreads();
  }
  pong_books_close(s, books, le, (uint32_t)a.T, live);
  if (live) pong_store(a.state, n, i, s);
  flush_wave_stats<false>(a.stats, le);
}

int g_rollout_block = 0;   // 0 = choose from N
int g_rollout_split = 0;   // 0 = choose from N and T, 1 = never, 2 = whenever possible
int g_paged_mode = 2;      // 0 never, 1 whenever possible, 2 = choose from N
int g_xcd_remap = 1;
int g_rollout_chunk = 0;   // 0 = choose from N
int g_rollout_pace = 0;    // GB/s the paced variant keeps the write stream to; 0 = choose from N, -1 = never paced
int g_step_kernel = 1;     // T = 1 launches: 1 = the step kernel, resident form where it applies; 2 = the step kernel with arguments; 0 = the rollout kernel's T = 1 path
int g_measure_pace = 1;    // 1 = measure once per device and batch size whether pacing pays, 0 = the table decides

}  // namespace

hipError_t launch_pong_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                             const StepCounter* counter, float* obs, bool normalize, hipStream_t stream) {
  const unsigned blocks = (unsigned)((n + 255) / 256);
  hipLaunchKernelGGL(pong_reset_kernel, dim3(blocks), dim3(256), 0, stream, state, n, seed, step, counter,
                     obs, normalize);
  return hipGetLastError();
}

// Measurement knob: threads per workgroup of the rollout kernel (64, 128, 256; 0 = automatic).
bool set_paged_stores(int mode) {
  if (mode < 0 || mode > 2) return false;
  g_paged_mode = mode;
  return true;
}

bool set_rollout_chunk(int steps) {
  if (steps != 0 && steps != 2 && steps != 4 && steps != 8) return false;
  g_rollout_chunk = steps;
  return true;
}

bool set_rollout_split(int mode) {
  if (mode < 0 || mode > 2) return false;
  g_rollout_split = mode;
  return true;
}

bool set_rollout_pace(int gb_per_s) {
  if (gb_per_s < -1 || gb_per_s > 8000) return false;
  g_rollout_pace = gb_per_s;
  return true;
}

bool set_step_kernel(int on) {
  if (on < 0 || on > 2) return false;
  g_step_kernel = on;
  return true;
}

bool set_measure_pace(int on) {
  if (on != 0 && on != 1) return false;
  g_measure_pace = on;
  return true;
}

bool set_rollout_block(int threads, int xcd_remap) {
  if (threads != 0 && threads != 64 && threads != 128 && threads != 256) return false;
  g_rollout_block = threads;
  g_xcd_remap = xcd_remap;
  return true;
}

namespace {

// Time per chunk of the paced loops, in 1/256 of a tick of the constant clock (100 MHz on this
// device; asked of the runtime rather than assumed).
int32_t pace_period(int64_t n, int rate_gb_per_s, double rows) {
  static int khz_of_device[64] = {};                       // asked once per device
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); dev = -1; }
  if (dev >= 0 && dev < 64) khz = khz_of_device[dev];
  if (khz <= 0) {
    if (dev < 0 || hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) {
      (void)hipGetLastError();
      khz = 100000;
    }
    if (dev >= 0 && dev < 64) khz_of_device[dev] = khz;
  }
  const double q = rows * (double)n * 37.0 / ((double)rate_gb_per_s * 1e9) * ((double)khz * 1e3) * 256.0;
  return q < 1073741824.0 ? (int32_t)q : 1073741824;       // 32-bit clock arithmetic in the kernel
}

// The launcher's table: the rate (GB/s) the paced loop is held to for a batch of n, -1 = not paced.
int table_rate(int64_t n) {
  return n < PACED_MIN_ENVS || n > PACED_MAX_ENVS ? -1 : n <= 65536 ? 6600 : n <= 131072 ? 5800 : 5600;
}

template <bool TRIAL>
void dispatch_variant(int variant, dim3 g, dim3 b, hipStream_t stream, const PongLaunch& a2) {
  switch (variant) {
    case V_RAW_2: hipLaunchKernelGGL((pong_rollout_kernel<V_RAW_2, TRIAL>), g, b, 0, stream, a2); break;
    case V_RAW_4: hipLaunchKernelGGL((pong_rollout_kernel<V_RAW_4, TRIAL>), g, b, 0, stream, a2); break;
    case V_RAW_8: hipLaunchKernelGGL((pong_rollout_kernel<V_RAW_8, TRIAL>), g, b, 0, stream, a2); break;
    case V_PACED: hipLaunchKernelGGL((pong_rollout_kernel<V_PACED, TRIAL>), g, b, 0, stream, a2); break;
    case V_PAGED: hipLaunchKernelGGL((pong_rollout_kernel<V_PAGED, TRIAL>), g, b, 0, stream, a2); break;
    default: break;
  }
}

// What the measurement below found for (device, n): rate > 0 paced at that rate, -1 not paced.
struct PaceChoice { int device; int64_t n; int rate; };
std::mutex g_choice_mutex;
PaceChoice g_choices[32] = {};
int g_choices_used = 0;

bool known_choice(int device, int64_t n, int* rate) {
  std::lock_guard<std::mutex> lock(g_choice_mutex);
  for (int k = 0; k < g_choices_used; ++k)
    if (g_choices[k].device == device && g_choices[k].n == n) { *rate = g_choices[k].rate; return true; }
  return false;
}

void remember_choice(int device, int64_t n, int rate) {
  std::lock_guard<std::mutex> lock(g_choice_mutex);
  if (g_choices_used < 32) g_choices[g_choices_used++] = {device, n, rate};
}

// Paced or not, and at which rate: measured once per device and batch size, on the handle's trial
// state, with the loops themselves.  The table's rates were found on a few devices of one pool, a
// rate above what the memory system of the device at hand drains is worse than no pacing at all,
// and a launch that has fallen behind its schedule does not recover -- so the table is only the
// starting point: the plain loop and the paced loop at the table's rate and at rates 4 and 8 %
// below it (and 4 % above, where the loop's own pace is not the limit) each run a launch of the
// caller's length a few times and the fastest wins; the paced loop has to beat the plain one by 1 % to be chosen.  The
// device runs on lower clocks for some 30 ms after any idle period, during which the plain loop
// looks better than it is, so the trials are preceded by 50 ms of the paced loop itself.  All of
// it writes to the caller's output buffers (rows the real launch overwrites right afterwards),
// to the trial state and the trial statistics: nothing of it is visible afterwards.  Costs 70 to
// 120 ms, once; returns the table's rate without measuring when the launch is too short to matter,
// when the stream is being captured, or when anything fails.
int measured_rate(const PongLaunch& a, dim3 g, dim3 b, hipStream_t stream) {
  const int fallback = table_rate(a.n);
  // as long as the caller's own launch, up to 1024 steps: the plain loop's wavefronts drift apart as
  // a launch goes on, so short trials flatter it (N = 61440: 256-step trials picked the plain loop,
  // which then ran the caller's 1000 steps in 0.429 ms against the paced loop's 0.374)
  constexpr int32_t TRIAL_MIN_T = 256;
  const int32_t TRIAL_T = a.T < 1024 ? a.T : 1024;
  if (!a.trial_state || !a.trial_stats || a.T < TRIAL_MIN_T || fallback <= 0) return fallback;
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) { (void)hipGetLastError(); return fallback; }
  int rate = fallback;
  if (known_choice(device, a.n, &rate)) return rate;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &cs) != hipSuccess) { (void)hipGetLastError(); return fallback; }
  if (cs != hipStreamCaptureStatusNone) return fallback;

  PongLaunch t = a;
  t.state = a.trial_state; t.stats = a.trial_stats; t.counter = nullptr; t.ticket = 0;
  t.step0 = a.step0; t.T = TRIAL_T; t.actions = nullptr; t.normalize = 0;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool ok = hipMemcpyAsync(t.state, a.state, (size_t)PONG_FIELDS * (size_t)a.n * 4, hipMemcpyDeviceToDevice, stream) == hipSuccess &&
            hipMemsetAsync(t.stats, 0, STATS_STRIPES * sizeof(DeviceStats), stream) == hipSuccess &&
            hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
  auto launch = [&](int r) {
    PongLaunch x = t;
    int variant = V_RAW_2;
    x.paged = 0;
    if (r > 0) { variant = V_PACED; x.pace = pace_period(a.n, r, 2.0); }
    else if (a.n >= 73728 && b.x == 256) { variant = V_PAGED; x.paged = 1; }
    dispatch_variant<true>(variant, g, b, stream, x);
    ok = ok && hipGetLastError() == hipSuccess;
  };
  auto timed = [&](int r) -> float {
    for (int k = 0; k < 2 && ok; ++k) launch(r);
    ok = ok && hipEventRecord(e0, stream) == hipSuccess;
    for (int k = 0; k < 6 && ok; ++k) launch(r);
    float ms = 0.0f;
    ok = ok && hipEventRecord(e1, stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
         hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    return ms;
  };
  if (ok) {
    // 50 ms at the table's rate: launches of TRIAL_T steps take TRIAL_T * n * 37 B / rate each
    const double each_ms = (double)TRIAL_T * (double)a.n * 37.0 / ((double)fallback * 1e9) * 1e3;
    const int warm = (int)(50.0 / each_ms) + 1;
    for (int k = 0; k < warm && ok; ++k) launch(fallback);
    const float plain = timed(-1);
    float best_ms = 0.0f;
    int best_rate = -1;
    const int percent[4] = {92, 96, 100, 104};
    for (int k = 0; k < 4 && ok; ++k) {
      const int r = fallback * percent[k] / 100;
      if (r > 6600 && a.n <= 65536) continue;              // there the loop's own pace is the limit already
      const float ms = timed(r);
      if (ok && (best_rate < 0 || ms < best_ms)) { best_ms = ms; best_rate = r; }
    }
    if (ok) rate = (best_rate > 0 && best_ms < 0.99f * plain) ? best_rate : -1;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (!ok) { (void)hipGetLastError(); return fallback; }
  remember_choice(device, a.n, rate);
  return rate;
}

}  // namespace

// For the benchmark and the tests: what was measured for (current device, n): the rate in GB/s, -1
// for "not paced", 0 if nothing has been measured for that batch size yet.
int pong_pace_choice(int64_t n) {
  int device = -1, rate = 0;
  if (hipGetDevice(&device) != hipSuccess) { (void)hipGetLastError(); return 0; }
  return known_choice(device, n, &rate) ? rate : 0;
}

namespace {

std::atomic<unsigned long long> g_resident_launches{0};

// Ownership of the launch records, per device (host side).
std::mutex g_step_slot_mutex;
struct StepSlots { int device; bool taken[STEP_RECORD_SLOTS]; };
std::vector<StepSlots> g_step_slots;

template <int SLOT>
void launch_resident(unsigned groups, hipStream_t stream) {
  hipLaunchKernelGGL(pong_step_resident_kernel<SLOT>, dim3(groups), dim3(256), 0, stream);
}

}  // namespace

unsigned long long resident_step_launches() { return g_resident_launches.load(std::memory_order_relaxed); }
void count_resident_step_launch() { g_resident_launches.fetch_add(1, std::memory_order_relaxed); }
int step_kernel_mode() { return g_step_kernel; }

int step_slot_acquire(int device) {
  std::lock_guard<std::mutex> lock(g_step_slot_mutex);
  StepSlots* d = nullptr;
  for (auto& x : g_step_slots)
    if (x.device == device) d = &x;
  if (!d) {
    g_step_slots.push_back(StepSlots{device, {}});
    d = &g_step_slots.back();
  }
  for (int k = 0; k < STEP_RECORD_SLOTS; ++k)
    if (!d->taken[k]) {
      d->taken[k] = true;
      return k;
    }
  return -1;
}

void step_resident_release(StepResident& r) {
  if (r.slot < 0) return;
  std::lock_guard<std::mutex> lock(g_step_slot_mutex);
  for (auto& x : g_step_slots)
    if (x.device == r.device) x.taken[r.slot] = false;
  r.slot = -1;
  r.on_device = false;
}

hipError_t launch_pong_rollout(const PongLaunch& a, hipStream_t stream, StepResident* resident) {
  const int block = g_rollout_block ? g_rollout_block : ROLLOUT_BLOCK;
  unsigned blocks = (unsigned)((a.n + block - 1) / block);
  blocks = (blocks + 7u) & ~7u;   // multiple of the XCD count; surplus workgroups exit at once
  const dim3 g(blocks), b(block);
  PongLaunch a2 = a;
  a2.ticket = blocks <= TICKET_MAX_BLOCKS;
  a2.xcd_remap = g_xcd_remap;
  if (a.T == 1 && g_step_kernel) {
    const unsigned groups = (unsigned)((a.n + 255) / 256);
    hipError_t re = hipSuccess;
    if (resident_step_try(
            resident, a, groups, stream,
            [&](int slot, const PongLaunch& rec, unsigned long long step) {
              hipLaunchKernelGGL(step_record_write_kernel, dim3(1), dim3(256), 0, stream, slot, rec, step);
            },
            [&](int slot, unsigned g2) {
              switch (slot) {
                case 0: launch_resident<0>(g2, stream); break;
                case 1: launch_resident<1>(g2, stream); break;
                case 2: launch_resident<2>(g2, stream); break;
                default: launch_resident<3>(g2, stream); break;
              }
              static_assert(STEP_RECORD_SLOTS == 4, "one case per record");
            },
            &re))
      return re;
    a2.ticket = groups <= TICKET_MAX_BLOCKS;
    const dim3 sg(groups), sb(256);
    if (a.actions && a.normalize) hipLaunchKernelGGL((pong_step_kernel<true, true>), sg, sb, 0, stream, a2);
    else if (a.actions) hipLaunchKernelGGL((pong_step_kernel<true, false>), sg, sb, 0, stream, a2);
    else if (a.normalize) hipLaunchKernelGGL((pong_step_kernel<false, true>), sg, sb, 0, stream, a2);
    else hipLaunchKernelGGL((pong_step_kernel<false, false>), sg, sb, 0, stream, a2);
    const hipError_t e = hipGetLastError();
    return e != hipSuccess ? e : advance_step_counter_behind(a.counter, 1, groups, stream);
  }
  // Which loop runs the in-kernel-action, raw-observation rollout (ms per launch at T = 1000, one
  // box, same process):
  //  * N <= 53248 (fewer wavefronts than SIMDs, latency bound): 8 steps per chunk -- long chunks
  //    give the scheduler more independent work to cover latency with (N = 16384: 0.337 / 0.323 /
  //    0.309 with 2 / 4 / 8 steps).
  //  * up to N = 61440: 2 steps per chunk (N = 57344: 0.337 / 0.410 / 0.419).  A wavefront takes a
  //    step every 337 ns here, and the memory system still keeps up with N x 37 B per 337 ns.
  //  * N = 61440 ... 262144: above that it does not keep up, stores queue, the wavefronts drift
  //    over many rows of the trajectory arrays and the write stream drops from 6.4 to 5.4 TB/s
  //    (N = 65536: 0.432 ms).  The paced loop holds every wavefront to one chunk per
  //    (rows x N x 37 B / rate) of the constant 100 MHz clock, a rate just under what the memory
  //    system drains: N = 65536: 0.380 ms at 6.6 TB/s; N = 81920: 0.536 (unpaced 0.730, paged
  //    0.609) and N = 131072: 0.847 (1.009, 0.957) at 5.8 TB/s; N = 262144: 1.742 (2.090, 1.840)
  //    at 5.6 TB/s.  Whether it pays, and at which rate, depends on the device at hand, so it is
  //    measured once per device and batch size (measured_rate above; the rates just quoted are
  //    the table it starts from, and what it falls back to when it cannot measure).  At
  //    N <= 65536 the loop's own pace (0.372 ms per 1000 steps) is the limit.
  //  * above N = 262144 the wavefronts are not all resident at once and a clock cannot align them:
  //    observation stores paged through LDS (N = 2^20: 7.4 ms per 1000 steps against 8.6 direct).
  //    Paged stores pay a barrier and an LDS round trip per step, which is exposed latency with
  //    one wavefront per SIMD (N = 65536: 0.484 ms).
  int rate = g_rollout_pace;
  if (rate == 0) rate = g_measure_pace ? measured_rate(a2, g, b, stream) : table_rate(a.n);
  a2.paged = g_paged_mode == 2 ? (a.n >= 73728 && rate <= 0) : g_paged_mode;
  const int chunk = g_rollout_chunk ? g_rollout_chunk : (a.n <= 53248 ? 8 : 2);
  // two wavefronts per 64 environments: in-kernel actions, raw observations, a launch of at most
  // one workgroup per CU that is long enough for the hand-over to pay
  const bool split = !a.normalize && !a.actions && g_paged_mode != 1 && rate <= 0 && g_rollout_chunk == 0 &&
                     (g_rollout_split == 2 || (g_rollout_split == 0 && a.n <= 16384 && a.T >= 4 * SPLIT_STEPS));
  if (split) {
    unsigned wgs = (unsigned)((a.n + WAVE - 1) / WAVE);
    wgs = (wgs + 7u) & ~7u;
    a2.ticket = wgs <= TICKET_MAX_BLOCKS;
    if (a.n % WAVE == 0) hipLaunchKernelGGL(pong_split_rollout_kernel<true>, dim3(wgs), dim3(128), 0, stream, a2);
    else hipLaunchKernelGGL(pong_split_rollout_kernel<false>, dim3(wgs), dim3(128), 0, stream, a2);
    const hipError_t e = hipGetLastError();
    return e != hipSuccess ? e : advance_step_counter_behind(a.counter, a.T, wgs, stream);
  }
  int variant;
  if (a.normalize) variant = a.actions ? V_NORMALIZED_EXTERNAL : rate > 0 ? V_NORMALIZED_PACED : V_NORMALIZED;
  // external actions: pacing pays only from two wavefronts per SIMD on (N = 131072: 1.24 against
  // 1.37 ms, N = 262144: 2.54 against 2.80; N = 65536: 0.56 against 0.46)
  else if (a.actions) variant = rate > 0 && (g_rollout_pace > 0 || a.n > 98304) ? V_EXTERNAL_PACED : V_EXTERNAL;
  else if (a2.paged && block == 256) variant = V_PAGED;
  else if (rate > 0) variant = V_PACED;
  else variant = chunk == 2 ? V_RAW_2 : chunk == 8 ? V_RAW_8 : V_RAW_4;
  if (variant == V_PACED || variant == V_EXTERNAL_PACED || variant == V_NORMALIZED_PACED)
    a2.pace = pace_period(a.n, rate, variant == V_EXTERNAL_PACED ? 8.0 : 2.0);
  switch (variant) {
    case V_EXTERNAL_PACED: hipLaunchKernelGGL(pong_rollout_kernel<V_EXTERNAL_PACED>, g, b, 0, stream, a2); break;
    case V_EXTERNAL: hipLaunchKernelGGL(pong_rollout_kernel<V_EXTERNAL>, g, b, 0, stream, a2); break;
    case V_NORMALIZED: hipLaunchKernelGGL(pong_rollout_kernel<V_NORMALIZED>, g, b, 0, stream, a2); break;
    case V_NORMALIZED_PACED: hipLaunchKernelGGL(pong_rollout_kernel<V_NORMALIZED_PACED>, g, b, 0, stream, a2); break;
    case V_NORMALIZED_EXTERNAL: hipLaunchKernelGGL(pong_rollout_kernel<V_NORMALIZED_EXTERNAL>, g, b, 0, stream, a2); break;
    default: dispatch_variant<false>(variant, g, b, stream, a2); break;
  }
  const hipError_t err = hipGetLastError();
  return err != hipSuccess ? err : advance_step_counter_behind(a.counter, a.T, blocks, stream);
}

}  // namespace envk
