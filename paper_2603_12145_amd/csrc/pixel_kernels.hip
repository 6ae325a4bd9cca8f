// Pong with pixel observations: dynamics per lane, rendering per wavefront.
//
// Each 84x84 uint8 frame (7056 B = 441 x 16 B) is black except for at most 54 lit pixels (two
// paddles, one ball), so the cost of a frame is its HBM write, not its arithmetic.  A wavefront owns
// a private 7056-byte LDS tile that is kept all-zero between frames.  For each of its environments
// it (1) pokes the lit pixels of the three rectangles into the tile (a handful of ds_write_b8),
// (2) streams the tile to HBM with 441 fully coalesced 16-byte stores (every store instruction of
// the wavefront covers 1 KiB of contiguous memory), (3) clears the poked bytes again.  No
// workgroup barrier is needed: a tile is only ever touched by its own wavefront, whose LDS
// operations execute in program order.
//
// Rasterisation rule (any overlap): pixel (r,c) is lit iff some rectangle [x0,x0+w) x [y0,y0+h)
// overlaps the cell [160c/84, 160(c+1)/84) x [210r/84, 210(r+1)/84), decided in float32 as
//   x0*84 < 160(c+1)  &&  (x0+w)*84 > 160c  &&  y0*84 < 210(r+1)  &&  (y0+h)*84 > 210r.
// Both column conditions are monotone in c (rows likewise), so each rectangle lights an axis-
// aligned block of cells whose four bounds are found per lane with one floor and an exact fix-up.
#include "kernels.hpp"
#include "pong_device.hpp"

namespace envk {

namespace {

constexpr int WAVE = 64;
constexpr int WAVES_PER_BLOCK = 4;
constexpr int CHUNKS = FRAME_BYTES / 16;  // 441
constexpr int64_t TRAJ_MIN_FRAMES = 1 << 18;   // frames of trajectory staging every pixel handle has at least

enum PixelMode { MODE_RESET = 0, MODE_RING = 1, MODE_FRAMES = 2 };

// smallest integer c with a < size * (c + 1)
__device__ __forceinline__ int first_cell(float a, float size, float inv_size) {
  int g = (int)floorf(a * inv_size);
  if (!(a < size * (float)(g + 1))) g += 1;
  else if (a < size * (float)g) g -= 1;
  return g;
}
// largest integer c with size * c < b
__device__ __forceinline__ int last_cell(float b, float size, float inv_size) {
  int h = (int)floorf(b * inv_size);
  if (!(size * (float)h < b)) h -= 1;
  else if (size * (float)(h + 1) < b) h += 1;
  return h;
}

// Cell block of one rectangle packed as bytes: col_lo | col_end << 8 | row_lo << 16 | row_end << 24
// (ends exclusive, all clipped to [0,84]; an empty block has end <= lo).
__device__ __forceinline__ uint32_t cell_block(float x0, float y0, float w, float h) {
  int c_lo = first_cell(x0 * 84.0f, 160.0f, 1.0f / 160.0f);
  int c_end = last_cell((x0 + w) * 84.0f, 160.0f, 1.0f / 160.0f) + 1;
  int r_lo = first_cell(y0 * 84.0f, 210.0f, 1.0f / 210.0f);
  int r_end = last_cell((y0 + h) * 84.0f, 210.0f, 1.0f / 210.0f) + 1;
  c_lo = min(max(c_lo, 0), FRAME_SIDE); c_end = min(max(c_end, 0), FRAME_SIDE);
  r_lo = min(max(r_lo, 0), FRAME_SIDE); r_end = min(max(r_end, 0), FRAME_SIDE);
  return (uint32_t)c_lo | ((uint32_t)c_end << 8) | ((uint32_t)r_lo << 16) | ((uint32_t)r_end << 24);
}

// All lanes: write `value` to every pixel of the (wave-uniform) block.  Lane l covers column
// offset l & 3 and row offset l >> 2 of a 4 x 16 patch; blocks are at most 4 x 8 for the paddles
// and 3 x 2 for the ball, so the loops run once.
__device__ __forceinline__ void poke_block(uint8_t* tile, uint32_t block, int lane, uint8_t value) {
  const int c_lo = block & 0xff, c_end = (block >> 8) & 0xff;
  const int r_lo = (block >> 16) & 0xff, r_end = block >> 24;
  for (int rr = r_lo; rr < r_end; rr += 16)
    for (int cc = c_lo; cc < c_end; cc += 4) {
      const int r = rr + (lane >> 2), c = cc + (lane & 3);
      if (r < r_end && c < c_end) tile[r * FRAME_SIDE + c] = value;
    }
}

// Order the wavefront's own LDS traffic: later reads must see earlier pokes of other lanes.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

typedef uint32_t chunk_t __attribute__((ext_vector_type(4)));   // 16 bytes, one dwordx4 access

template <bool STREAMING>
__device__ __forceinline__ void store_chunk(chunk_t* dst, const chunk_t v) {
  if (STREAMING) __builtin_nontemporal_store(v, dst);
  else *dst = v;
}

template <int EPW, int MODE, bool STREAMING>
__global__ __launch_bounds__(WAVES_PER_BLOCK * WAVE) void pixel_kernel(PixelLaunch a) {
  __shared__ __align__(16) uint8_t tiles[WAVES_PER_BLOCK][FRAME_BYTES];
  // a handle that keeps its step counter in device memory: read it (and, for a step, advance it)
  // before any wavefront leaves
  if (MODE == MODE_RESET) a.pong.step0 = read_step(a.pong.counter, a.pong.step0);
  else a.pong.step0 = launch_first_step(a.pong.counter, a.pong.step0, a.pong.T, a.pong.ticket != 0);
  const int lane = threadIdx.x & (WAVE - 1);
  const int wave = threadIdx.x >> 6;
  const int64_t n = a.pong.n;
  const int64_t env0 = ((int64_t)blockIdx.x * WAVES_PER_BLOCK + wave) * EPW;
  if (env0 >= n) return;                       // whole wavefront leaves together
  const int64_t i = env0 + lane;
  const bool live = (lane < EPW) && (i < n);
  const int here = (int)min((int64_t)EPW, n - env0);   // environments of this wavefront

  uint8_t* tile = tiles[wave];
  chunk_t* tile16 = reinterpret_cast<chunk_t*>(tile);
  for (int k = lane; k < CHUNKS; k += WAVE) tile16[k] = chunk_t{0, 0, 0, 0};
  wave_lds_sync();

  PongLane s;
  if (MODE == MODE_RESET) {
    s = pong_initial(a.pong.seed, (uint32_t)i, a.pong.step0);
    if (live) pong_store(a.pong.state, n, i, s);
  } else {
    s = live ? pong_load(a.pong.state, n, i) : pong_idle_lane();
  }
  LaneEpisodes le;
  const int32_t T = (MODE == MODE_RESET) ? 1 : a.pong.T;

  for (int32_t t = 0; t < T; ++t) {
    const uint64_t step = a.pong.step0 + (uint64_t)t;
    if (MODE != MODE_RESET) {
      const Draw4 d = philox_draw(a.pong.seed, (uint32_t)i, step, 0u);
      const int64_t row = (int64_t)t * n;
      int action = pong_action_from_word(d.w0);
      if (a.pong.actions) action = live ? (int)a.pong.actions[row + i] : 0;
      const PongEvent ev = pong_transition(s, action, d.w1, d.w2, a.pong.max_score);
      if (live) {
        a.pong.reward[row + i] = ev.reward;
        a.pong.done[row + i] = ev.done ? 1 : 0;
        if (ev.done) {
          le.count += 1;
          le.length_sum += ev.fin_len;
          le.ret_sum_i += ev.fin_ret;
          le.min_key = min(le.min_key, ev.fin_ret);
          le.max_key = max(le.max_key, ev.fin_ret);
        }
      }
    }

    const uint32_t blk_agent = cell_block(140.0f, s.pa, 4.0f, 16.0f);
    const uint32_t blk_opp = cell_block(16.0f, s.po, 4.0f, 16.0f);
    const uint32_t blk_ball = cell_block(s.bx, s.by, 2.0f, 2.0f);

    for (int e = 0; e < here; ++e) {
      const uint32_t b0 = __builtin_amdgcn_readlane(blk_agent, e);
      const uint32_t b1 = __builtin_amdgcn_readlane(blk_opp, e);
      const uint32_t b2 = __builtin_amdgcn_readlane(blk_ball, e);
      poke_block(tile, b0, lane, 255);
      poke_block(tile, b1, lane, 255);
      poke_block(tile, b2, lane, 255);
      wave_lds_sync();

      const int64_t env = env0 + e;
      if (MODE == MODE_FRAMES) {
        chunk_t* dst = reinterpret_cast<chunk_t*>(a.frames + ((int64_t)t * n + env) * FRAME_BYTES);
#pragma unroll
        for (int k = lane; k < CHUNKS; k += WAVE) store_chunk<STREAMING>(dst + k, tile16[k]);
      } else if (MODE == MODE_RING) {
        const int64_t slot = (int64_t)(step & 3);
        const int64_t frame = a.slot_major ? slot * n + env : env * 4 + slot;
        chunk_t* dst = reinterpret_cast<chunk_t*>(a.ring + frame * FRAME_BYTES);
#pragma unroll
        for (int k = lane; k < CHUNKS; k += WAVE) store_chunk<STREAMING>(dst + k, tile16[k]);
      } else {  // reset: the same frame into all four slots
        const int64_t first = a.slot_major ? env : env * 4;
        const int64_t pitch = a.slot_major ? n : 1;            // frames between slots
        chunk_t* dst = reinterpret_cast<chunk_t*>(a.ring + first * FRAME_BYTES);
        for (int k = lane; k < CHUNKS; k += WAVE) {
          const chunk_t v = tile16[k];
          for (int slot = 0; slot < 4; ++slot) store_chunk<STREAMING>(dst + slot * pitch * CHUNKS + k, v);
        }
      }
      wave_lds_sync();
      poke_block(tile, b0, lane, 0);
      poke_block(tile, b1, lane, 0);
      poke_block(tile, b2, lane, 0);
      wave_lds_sync();
    }
  }

  if (MODE != MODE_RESET) {
    if (live) pong_store(a.pong.state, n, i, s);
    flush_wave_stats<false>(a.pong.stats, le);
  }
}

// ---------------------------------------------------------------------------------------------
// Slot-major ring: one step rewrites one whole plane of N frames, a single dense N*7056-byte
// stream.  Measured on MI355X, the write pattern that gets closest to HBM peak is "one workgroup
// writes one 4 KiB-aligned page with one 16-byte store per thread, workgroups dispatched in address
// order" (about 6.8 TB/s for a plain fill against about 5.3 TB/s for any scheme in which a
// wavefront streams several KiB on its own).  The plane is therefore rendered page by page from
// 12 bytes per environment (the three rectangles' cell blocks), which a lane-per-environment
// dynamics pass stages in library scratch one step ahead of the renderer.
// ---------------------------------------------------------------------------------------------
// Staging buffers of one step (library scratch): what the dynamics produce for the renderer and for
// the caller.
struct Staged {
  uint32_t* blocks;     // [3][n]
  float* reward;        // [n]
  uint8_t* done;        // [n]
  int32_t* fin_ret;     // [n], valid where done
  int32_t* fin_len;
};

// Dynamics of one step for environment i: state_in -> state_out and the staging buffers.
// RESET: draw the initial state instead (state_in unused, only state_out and blocks written).
template <bool RESET>
__device__ __forceinline__ void stage_step(const PongLaunch& a, const uint32_t* __restrict__ state_in,
                                           uint32_t* __restrict__ state_out, const Staged& st, int64_t i) {
  const int64_t n = a.n;
  if (i >= n) return;
  PongLane s;
  if (RESET) {
    s = pong_initial(a.seed, (uint32_t)i, a.step0);
  } else {
    s = pong_load(state_in, n, i);
    const Draw4 d = philox_draw(a.seed, (uint32_t)i, a.step0, 0u);
    const int action = a.actions ? (int)a.actions[i] : pong_action_from_word(d.w0);
    const PongEvent ev = pong_transition(s, action, d.w1, d.w2, a.max_score);
    st.reward[i] = ev.reward;
    st.done[i] = ev.done ? 1 : 0;
    st.fin_ret[i] = ev.fin_ret;
    st.fin_len[i] = ev.fin_len;
  }
  pong_store(state_out, n, i, s);
  st.blocks[0 * n + i] = cell_block(140.0f, s.pa, 4.0f, 16.0f);
  st.blocks[1 * n + i] = cell_block(16.0f, s.po, 4.0f, 16.0f);
  st.blocks[2 * n + i] = cell_block(s.bx, s.by, 2.0f, 2.0f);
}

template <bool RESET>
__global__ __launch_bounds__(256) void pixel_dynamics_kernel(PongLaunch a, const uint32_t* state_in,
                                                             uint32_t* state_out, Staged st) {
  stage_step<RESET>(a, state_in, state_out, st, (int64_t)blockIdx.x * 256 + threadIdx.x);
}

// T steps of environment i in registers; per step the three cell blocks of the frame after the step
// go to blocks[k][t * n + i] (k = agent paddle, opponent paddle, ball; `frames` = T * n entries per
// k), reward and done to the caller's [T][n] rows; the state is loaded and stored once.
// The loop takes TRIP steps per trip with no branch inside a trip; the Philox blocks and (EXTERNAL)
// the actions of a trip are fetched during the trip before.  The first loads are waited for once,
// in front of the loop: otherwise the compiler's wait-count bookkeeping carries "just issued,
// nothing behind them" into the loop header and every trip begins by waiting for all stores in
// flight (1.25 us per step instead of 0.4 in this latency-bound pass).
template <bool EXTERNAL>
__global__ __launch_bounds__(256) void pixel_traj_dynamics_kernel(PongLaunch a, uint32_t* __restrict__ blocks,
                                                                  int64_t frames) {
  // every thread reaches the end of this kernel: the counter is read with a plain load here and
  // the ticket taken behind the last store (see step_counter.hpp)
  a.step0 = first_step_of_launch(a.counter, a.step0);
  const int64_t n = a.n;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const bool live = i < n;
  const int64_t ic = live ? i : n - 1;
  PongLane s = pong_load(a.state, n, ic);
  LaneEpisodes le;
  constexpr int TRIP = 8;
  // rows past the end read the last row, so that the loads stay unconditional
  auto fetch_action = [&](int32_t row) -> int {
    return EXTERNAL ? (int)a.actions[(int64_t)(row < a.T ? row : a.T - 1) * n + ic] : 0;
  };
  auto one_step = [&](const int32_t t, const Draw4& d, const int external_action) {
    const int action = EXTERNAL ? external_action : pong_action_from_word(d.w0);
    const PongEvent ev = pong_transition(s, action, d.w1, d.w2, a.max_score);
    const bool done = live && ev.done;
    le.count += done ? 1 : 0;
    le.length_sum += done ? ev.fin_len : 0;
    le.ret_sum_i += done ? ev.fin_ret : 0;
    le.min_key = done ? min(le.min_key, ev.fin_ret) : le.min_key;
    le.max_key = done ? max(le.max_key, ev.fin_ret) : le.max_key;
    if (live) {
      const int64_t f = (int64_t)t * n + i;
      blocks[0 * frames + f] = cell_block(140.0f, s.pa, 4.0f, 16.0f);
      blocks[1 * frames + f] = cell_block(16.0f, s.po, 4.0f, 16.0f);
      blocks[2 * frames + f] = cell_block(s.bx, s.by, 2.0f, 2.0f);
      a.reward[f] = ev.reward;
      a.done[f] = done ? 1 : 0;
    }
  };
  if (a.T >= TRIP) {                                                           // uniform
    int pending[TRIP];
    Draw4 cur[TRIP];
#pragma unroll
    for (int k = 0; k < TRIP; ++k) {
      pending[k] = fetch_action(k);
      cur[k] = philox_draw(a.seed, (uint32_t)ic, a.step0 + (uint64_t)k, 0u);
    }
    if (EXTERNAL) {
#pragma unroll
      for (int k = 0; k < TRIP; ++k) asm volatile("" : : "v"(pending[k]));
    }
    asm volatile("" : : "v"(s.bx), "v"(s.by), "v"(s.vx), "v"(s.vy), "v"(s.pa), "v"(s.po), "v"(s.sa), "v"(s.so),
                 "v"(s.ep_ret), "v"(s.ep_len));                               // the state's loads too
    int32_t t = 0;
    for (; t + TRIP <= a.T; t += TRIP) {
      Draw4 nxt[TRIP];
#pragma unroll
      for (int k = 0; k < TRIP; ++k) {
        nxt[k] = philox_draw(a.seed, (uint32_t)ic, a.step0 + (uint64_t)(t + TRIP + k), 0u);
        const int action = pending[k];
        pending[k] = fetch_action(t + TRIP + k);
        one_step(t + k, cur[k], action);
      }
#pragma unroll
      for (int k = 0; k < TRIP; ++k) cur[k] = nxt[k];
    }
    // fewer than TRIP steps are left; their Philox blocks and actions are at hand
#pragma unroll
    for (int k = 0; k < TRIP; ++k)
      if (t + k < a.T) one_step(t + k, cur[k], pending[k]);                   // uniform
  } else {
    for (int32_t t = 0; t < a.T; ++t)
      one_step(t, philox_draw(a.seed, (uint32_t)ic, a.step0 + (uint64_t)t, 0u), fetch_action(t));
  }
  if (live) pong_store(a.state, n, i, s);
  flush_wave_stats<false>(a.stats, le);
  if (a.counter && a.ticket) finish_launch_steps(a.counter, a.step0, a.T, gridDim.x);
}

constexpr int PAGE = 4096;

// U consecutive 4 KiB-aligned pages of a plane: zero U LDS pages, poke the lit pixels of the (at
// most two) frames overlapping each page -- 192 candidate pixels per page, one per thread -- store
// 16 bytes per thread and page.  Offsets are counted in 16-byte chunks (441 per frame, 256 per
// page) and fit 32 bits: the host only takes this path for n * 441 < 2^31.  With U > 1 the cell
// blocks of all U pages are loaded up front and the workgroup passes two barriers for U pages
// instead of two per page: on planes of hundreds of megabytes a workgroup's life is otherwise
// mostly the latency of that load (frame trajectories of 262144 frames: 4.9 TB/s with U = 1).
template <int U>
__device__ __forceinline__ void render_pages(const uint32_t* __restrict__ blocks, int64_t n,
                                             uint8_t* __restrict__ plane, unsigned group_index, uint8_t* pages) {
  const int tid = threadIdx.x;
  const int total = (int)n * CHUNKS;                                  // chunks in the plane
  // chunk offsets relative to the start of the plane; the first page may begin before it
  const int lead = (int)((reinterpret_cast<uintptr_t>(plane) & (PAGE - 1)) >> 4);
  // threads 0..191: (frame, rectangle) pair tid / 32, pixel tid % 32 of a 4-column x 8-row patch
  // (a paddle covers at most 4 x 8 cells, the ball at most 3 x 2).  The cell blocks are loaded
  // before the pages are zeroed so that their latency overlaps the zeroing and the barrier.
  const int pair = tid >> 5;
  const bool from_last = pair >= 3;
  int page_off[U], lo[U], hi[U], f[U];
  bool candidate[U];
  uint32_t blk[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    page_off[u] = (int)(group_index * (unsigned)U + (unsigned)u) * (PAGE / 16) - lead;
    lo[u] = page_off[u] < 0 ? 0 : page_off[u];
    hi[u] = page_off[u] + PAGE / 16 < total ? page_off[u] + PAGE / 16 : total;
    const bool any = lo[u] < hi[u];                                    // a page past the end of the plane: nothing to do
    const int f_first = (int)((unsigned)lo[u] / (unsigned)CHUNKS);
    const int f_last = any ? (int)((unsigned)(hi[u] - 1) / (unsigned)CHUNKS) : f_first;   // f_first or f_first + 1
    candidate[u] = any && pair < 6 && !(from_last && f_last == f_first);
    f[u] = from_last ? f_last : f_first;
    blk[u] = 0;
    if (candidate[u]) blk[u] = blocks[(int64_t)(from_last ? pair - 3 : pair) * n + f[u]];
  }

  chunk_t* pages16 = reinterpret_cast<chunk_t*>(pages);
#pragma unroll
  for (int u = 0; u < U; ++u) pages16[u * (PAGE / 16) + tid] = chunk_t{0, 0, 0, 0};
  __syncthreads();

#pragma unroll
  for (int u = 0; u < U; ++u) {
    if (candidate[u]) {
      const int c_lo = blk[u] & 0xff, c_end = (blk[u] >> 8) & 0xff;
      const int r_lo = (blk[u] >> 16) & 0xff, r_end = blk[u] >> 24;
      const int c = c_lo + (tid & 3), r = r_lo + ((tid >> 2) & 7);
      const int off = (f[u] * CHUNKS - page_off[u]) * 16 + r * FRAME_SIDE + c;   // byte offset inside the page
      if (c < c_end && r < r_end && off >= 0 && off < PAGE) pages[u * PAGE + off] = 255;
    }
  }
  __syncthreads();

#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int mine = page_off[u] + tid;
    // One page per workgroup is the path of planes under 256 MB, which the 256 MB last-level cache
    // holds: there streaming (non-temporal) stores are faster (N = 16384: 18.9 against 20.2 us per
    // step, N = 32768: 33.8 against 35.6), apparently because less is left to write back when the
    // kernel ends.  On longer planes they lose (N = 65536: 82.8 against 72.1 us).
    if (mine >= lo[u] && mine < hi[u]) {
      if (U == 1) __builtin_nontemporal_store(pages16[u * (PAGE / 16) + tid], reinterpret_cast<chunk_t*>(plane) + mine);
      else reinterpret_cast<chunk_t*>(plane)[mine] = pages16[u * (PAGE / 16) + tid];
    }
  }
}

__device__ __forceinline__ void render_page(const uint32_t* __restrict__ blocks, int64_t n,
                                            uint8_t* __restrict__ plane, unsigned page_index, uint8_t* page) {
  render_pages<1>(blocks, n, plane, page_index, page);
}

constexpr int RENDER_U = 4;   // pages per render workgroup on long planes (2: 4.9 TB/s, 4: 5.7, 8: 5.5)
// U = 1: one page per workgroup; U = RENDER_U: that many consecutive pages per workgroup
template <int U>
__global__ __launch_bounds__(256) void plane_render_kernel(const uint32_t* __restrict__ blocks, int64_t n,
                                                           uint8_t* __restrict__ plane) {
  __shared__ __align__(16) uint8_t pages[U * PAGE];
  render_pages<U>(blocks, n, plane, blockIdx.x, pages);
}

// The plane of the step that the previous launch on the stream just took, for a handle whose step
// counter lives in device memory: that launch advanced the counter to s + 1, the frame after step s
// goes to ring slot s mod 4.  The grid covers the slot with the most pages (a slot's first and last
// page depend on its alignment); workgroups beyond this slot's pages leave.
__global__ __launch_bounds__(256) void plane_render_counted_kernel(const uint32_t* __restrict__ blocks, int64_t n,
                                                                   uint8_t* __restrict__ ring,
                                                                   const StepCounter* __restrict__ counter) {
  __shared__ __align__(16) uint8_t page[PAGE];
  const uint64_t slot = (counter->step - 1ull) & 3ull;
  uint8_t* plane = ring + (int64_t)slot * n * FRAME_BYTES;
  const uintptr_t base = reinterpret_cast<uintptr_t>(plane);
  const uintptr_t end = base + (uintptr_t)n * FRAME_BYTES;
  const unsigned pages = (unsigned)(((end + PAGE - 1) >> 12) - (base >> 12));
  if (blockIdx.x >= pages) return;
  render_page(blocks, n, plane, blockIdx.x, page);
}

// ---- delta updates ----------------------------------------------------------------------------
// A frame differs from the one four steps earlier in the pixels of three small rectangles, so a ring
// slot can be brought up to date by clearing the pixels that went dark and setting those that lit
// up; the four channels of an ordered stack (channel k: the frame 3 - k steps back) each change by
// one step's worth of pixels.  The library keeps the cell blocks of the last five frames (entry =
// step mod 5) and one launch takes the step and repairs the observation buffer.
//
// Whether the buffer holds what the kept blocks say is recorded in device memory, so that the
// decision is taken inside the launch and a launch recorded in a HIP graph decides anew at every
// replay: the buffer the record is about, and the first step from which it is good.  A step with
// another buffer, or before that step, writes whole frames instead (ring: the slot from the new
// blocks; stack: the channels moved down physically, the new frame on top) and four such steps in
// a row make the record good again.
struct PixelBook {
  unsigned long long valid_from;       // delta updates are right from this step on; NOT_KNOWN until a step sets it
  unsigned long long ring;             // address of the observation buffer that is about
  unsigned long long delta_steps, full_steps;
};
constexpr unsigned long long NOT_KNOWN = ~0ull;

// The rule, for the host's copy of the record and the device's alike.
__host__ __device__ inline bool record_says_known(const PixelBook* book, unsigned long long step, const uint8_t* ring) {
  return book->valid_from != NOT_KNOWN && step >= book->valid_from &&
         book->ring == (unsigned long long)reinterpret_cast<uintptr_t>(ring);
}
// ... and what a step does to the record: a step that could not repair starts (or continues) a run
// of four whole-frame steps.
__host__ __device__ inline void record_after_step(PixelBook* book, unsigned long long step, const uint8_t* ring) {
  const unsigned long long r = (unsigned long long)reinterpret_cast<uintptr_t>(ring);
  const bool known = record_says_known(book, step, ring);
  if (book->valid_from == NOT_KNOWN || book->ring != r) {
    book->ring = r;
    book->valid_from = step + 4ull;
  }
  (known ? book->delta_steps : book->full_steps) += 1ull;
}

struct UpdateStep {
  PongLaunch pong;      // T = 1; pong.counter may be null (then pong.step0 is the step)
  int known_by_host;    // host step counter: the host's copy of the record says the buffer can be repaired
                        // (picks the kernel's instantiation; the launch itself does not read it)
  PixelBook* book;      // device step counter: the record, read by the launch
  uint32_t* hist;       // [5][3][n]
  uint8_t* ring;
  int64_t stride;       // bytes from an environment's frame (stack) to the next environment's
  int64_t slot_pitch;   // ring: bytes from a slot to the next
  // host step counter only (the launch works these out itself otherwise):
  uint32_t* entry[5];   // history entries of the steps s - 4 .. s
  uint8_t* base;        // frame 0 of the slot this step writes; the stack's start
};

// 16 bytes of a frame (chunk c = pixels 16 c .. 16 c + 15) from its three cell blocks.
__device__ __forceinline__ chunk_t chunk_of_blocks(const uint32_t b0, const uint32_t b1, const uint32_t b2, int chunk) {
  const uint32_t b[3] = {b0, b1, b2};
  uint32_t words[4] = {0, 0, 0, 0};
#pragma unroll
  for (int byte = 0; byte < 16; ++byte) {
    const int p = chunk * 16 + byte, r = p / FRAME_SIDE, c = p - r * FRAME_SIDE;
    bool lit = false;
#pragma unroll
    for (int k = 0; k < 3; ++k)
      lit = lit || (c >= (int)(b[k] & 0xff) && c < (int)((b[k] >> 8) & 0xff) && r >= (int)((b[k] >> 16) & 0xff) &&
                    r < (int)(b[k] >> 24));
    words[byte >> 2] |= lit ? 0xffu << (8 * (byte & 3)) : 0u;
  }
  return chunk_t{words[0], words[1], words[2], words[3]};
}

// 32 lanes, one rectangle: lane l stands for pixel (l & 3, l >> 2) of a 4-column x 8-row patch (a
// paddle covers at most 4 x 8 cells, the ball at most 3 x 2), once anchored at the old block's corner
// -- there it clears its pixel unless one of the new frame's blocks covers it (rectangles may
// overlap: the ball in front of a paddle) -- and once at the new block's corner, where it sets its
// pixel unless the old block covered it.
__device__ __forceinline__ void repair_rectangle(uint8_t* __restrict__ frame, const uint32_t was, const uint32_t now,
                                                 const uint32_t n0, const uint32_t n1, const uint32_t n2) {
  const int dc = threadIdx.x & 3, dr = (threadIdx.x >> 2) & 7;
  const int wc0 = was & 0xff, wc1 = (was >> 8) & 0xff, wr0 = (was >> 16) & 0xff, wr1 = was >> 24;
  const int nc0 = now & 0xff, nc1 = (now >> 8) & 0xff, nr0 = (now >> 16) & 0xff, nr1 = now >> 24;
  {
    const int c = wc0 + dc, r = wr0 + dr;
    const uint32_t q[3] = {n0, n1, n2};
    bool lit = false;
#pragma unroll
    for (int j = 0; j < 3; ++j)
      lit = lit || (c >= (int)(q[j] & 0xff) && c < (int)((q[j] >> 8) & 0xff) && r >= (int)((q[j] >> 16) & 0xff) &&
                    r < (int)(q[j] >> 24));
    if (c < wc1 && r < wr1 && !lit) frame[r * FRAME_SIDE + c] = 0;
  }
  {
    const int c = nc0 + dc, r = nr0 + dr;
    if (c < nc1 && r < nr1 && !(c >= wc0 && c < wc1 && r >= wr0 && r < wr1)) frame[r * FRAME_SIDE + c] = 255;
  }
}

// A workgroup owns ENVS environments.  Thread 0 finds out the step and whether the buffer can be
// repaired.  Then the first wavefront takes the environments' step, one lane each (reward / done to the caller, state in
// place, episode statistics, the new cell blocks to the history) and leaves old and new blocks in
// LDS; after the barrier all four wavefronts repair the frames, 32 lanes per rectangle, or write
// them whole.
// MODE: the host knows the step and has decided (repair / whole frames), or the launch finds out.
enum UpdateMode { HOST_REPAIR = 0, HOST_WHOLE = 1, DEVICE_DECIDES = 2 };

template <int ENVS, bool ORDERED, int MODE>
__global__ __launch_bounds__(256) void pixel_update_step_kernel(UpdateStep a) {
  constexpr int FRAMES = ORDERED ? 5 : 2;                // frames whose blocks are staged; the last is the new one
  __shared__ uint32_t blk[FRAMES][3][ENVS];
  __shared__ unsigned long long shared_step;
  __shared__ int shared_known;
  // With the step counter on the host, the host also keeps the record and passes the answer.  With
  // the counter in device memory thread 0 reads counter and record (plain loads: both are written
  // only by the one-thread launch that follows this one on the stream).  A ticket scheme like the
  // other kernels' would have thousands of workgroups queue for one atomic here, which costs ten
  // times the step.
  uint64_t step = a.pong.step0;
  bool known = MODE == HOST_REPAIR;
  if (MODE == DEVICE_DECIDES) {
    if (threadIdx.x == 0) {
      const unsigned long long s = __hip_atomic_load(&a.pong.counter->step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      shared_step = s;
      shared_known = record_says_known(a.book, s, a.ring) ? 1 : 0;
    }
    __syncthreads();
    step = shared_step;
    known = shared_known != 0;
  }
  const int64_t n = a.pong.n;
  const int64_t env0 = (int64_t)blockIdx.x * ENVS;
  // History entries of the steps s - 4 + f, f = 0..4 (the last one receives the new frame's blocks),
  // and where frame 0 of the slot (or stack) starts: from the host when it knows the step, else
  // worked out here (step s - 4 lives in entry (s + 1) mod 5).
  uint32_t* entry[5];
  uint8_t* base = a.base;
#pragma unroll
  for (int f = 0; f < 5; ++f) entry[f] = a.entry[f];
  if (MODE == DEVICE_DECIDES) {
    // (s + 1) mod 5 in 32-bit arithmetic (2^32 = 1 mod 5): a 64-bit remainder is a long routine here
    const unsigned first = ((unsigned)step % 5u + (unsigned)(step >> 32) % 5u + 1u) % 5u;
#pragma unroll
    for (int f = 0; f < 5; ++f) {
      const unsigned e = first + (unsigned)f;
      entry[f] = a.hist + (int64_t)(e >= 5u ? e - 5u : e) * 3 * n;
    }
    base = a.ring + (ORDERED ? 0 : (int64_t)(step & 3) * a.slot_pitch);
  }
  uint32_t* new_blocks = entry[4];
  if (threadIdx.x < WAVE) {
    const int lane = threadIdx.x;
    const int64_t i = env0 + lane;
    const bool live = lane < ENVS && i < n;
    const int64_t ic = live ? i : n - 1;
    PongLane s = pong_load(a.pong.state, n, ic);
    // The kept blocks (ring: of the frame in the slot, f = 0; stack: of the four channels' frames)
    // do not depend on the step: all loads go out together with the state's, ahead of the
    // dependent chain of the transition.  Idle lanes read environment n - 1's, a valid address.
    uint32_t kept[FRAMES - 1][3];
#pragma unroll
    for (int f = 0; f < FRAMES - 1; ++f)
#pragma unroll
      for (int k = 0; k < 3; ++k) kept[f][k] = known ? entry[f][(int64_t)k * n + ic] : 0u;
    const Draw4 d = philox_draw(a.pong.seed, (uint32_t)ic, step, 0u);
    const int action = a.pong.actions ? (int)a.pong.actions[ic] : pong_action_from_word(d.w0);
    const PongEvent ev = pong_transition(s, action, d.w1, d.w2, a.pong.max_score);
    LaneEpisodes le;
    if (live && ev.done) {
      le.count = 1; le.length_sum = ev.fin_len; le.ret_sum_i = ev.fin_ret;
      le.min_key = ev.fin_ret; le.max_key = ev.fin_ret;
    }
    const uint32_t nb[3] = {cell_block(140.0f, s.pa, 4.0f, 16.0f), cell_block(16.0f, s.po, 4.0f, 16.0f),
                            cell_block(s.bx, s.by, 2.0f, 2.0f)};
    if (lane < ENVS) {
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        blk[FRAMES - 1][k][lane] = nb[k];
#pragma unroll
        for (int f = 0; f < FRAMES - 1; ++f) {
          // ring: the slot's frame, step s - 4; stack: steps s - 4 .. s - 1.  An idle lane shows no change.
          blk[f][k][lane] = (live && known) ? kept[f][k] : nb[k];      // an idle lane shows no change
        }
      }
    }
    if (live) {
#pragma unroll
      for (int k = 0; k < 3; ++k) new_blocks[(int64_t)k * n + i] = nb[k];
      a.pong.reward[i] = ev.reward;
      a.pong.done[i] = ev.done ? 1 : 0;
      pong_store(a.pong.state, n, i, s);
    }
    flush_wave_stats<false>(a.pong.stats, le);
  }
  __syncthreads();

  auto frame_of = [&](int e, int channel) -> uint8_t* {     // channel: of the stack; the ring has its slot in `base`
    if (ORDERED) return base + ((env0 + e) * 4 + channel) * (int64_t)FRAME_BYTES;
    return base + (env0 + e) * a.stride;
  };
  if (known) {
    constexpr int ITEMS = (ORDERED ? 12 : 3) * ENVS;
    for (int item = threadIdx.x >> 5; item < ITEMS; item += 8) {
      const int e = item % ENVS, rect = (item / ENVS) % 3, ch = item / (3 * ENVS);
      const uint32_t was = blk[ch][rect][e], now = blk[ch + 1][rect][e];
      if (was == now) continue;
      repair_rectangle(frame_of(e, ch), was, now, blk[ch + 1][0][e], blk[ch + 1][1][e],
                       blk[ch + 1][2][e]);
    }
  } else {
    for (int e = 0; e < ENVS; ++e) {
      if (env0 + e >= n) break;
      const uint32_t b0 = blk[FRAMES - 1][0][e], b1 = blk[FRAMES - 1][1][e], b2 = blk[FRAMES - 1][2][e];
      if (ORDERED) {
        // channels 1..3 move down by one, the new frame goes on top; a thread reads its chunk of the
        // three channels before it writes any of them
        chunk_t* stack = reinterpret_cast<chunk_t*>(frame_of(e, 0));
        for (int chunk = threadIdx.x; chunk < CHUNKS; chunk += 256) {
          const chunk_t c1 = stack[1 * CHUNKS + chunk], c2 = stack[2 * CHUNKS + chunk], c3 = stack[3 * CHUNKS + chunk];
          stack[0 * CHUNKS + chunk] = c1;
          stack[1 * CHUNKS + chunk] = c2;
          stack[2 * CHUNKS + chunk] = c3;
          stack[3 * CHUNKS + chunk] = chunk_of_blocks(b0, b1, b2, chunk);
        }
      } else {
        chunk_t* frame = reinterpret_cast<chunk_t*>(frame_of(e, 0));
        for (int chunk = threadIdx.x; chunk < CHUNKS; chunk += 256) frame[chunk] = chunk_of_blocks(b0, b1, b2, chunk);
      }
    }
  }
}

// After env_reset has written the initial frame to all four slots (channels) of `ring`: that is as
// if the steps s - 4 .. s - 1 (s = the next step) had each put that frame there, so their history
// entries get the blocks of the state as it stands and the record is good from step s on.
__global__ __launch_bounds__(256) void pixel_book_reset_kernel(const uint32_t* __restrict__ state, int64_t n,
                                                               uint64_t host_step,
                                                               const StepCounter* __restrict__ counter,
                                                               PixelBook* __restrict__ book, uint32_t* __restrict__ hist,
                                                               const uint8_t* ring) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const uint64_t step = read_step(counter, host_step);
  if (i == 0) {
    book->valid_from = step;
    book->ring = (unsigned long long)reinterpret_cast<uintptr_t>(ring);
  }
  if (i >= n) return;
  const PongLane s = pong_load(state, n, i);
  const uint32_t b0 = cell_block(140.0f, s.pa, 4.0f, 16.0f), b1 = cell_block(16.0f, s.po, 4.0f, 16.0f);
  const uint32_t b2 = cell_block(s.bx, s.by, 2.0f, 2.0f);
#pragma unroll
  for (int f = 0; f < 4; ++f) {
    uint32_t* entry = hist + (int64_t)((step + 1 + f) % 5) * 3 * n;
    entry[0 * n + i] = b0; entry[1 * n + i] = b1; entry[2 * n + i] = b2;
  }
}

// Behind a step of a handle whose step counter lives in device memory: the step's launch only read
// counter and record; this one thread brings both up to date.
__global__ void pixel_book_commit_kernel(StepCounter* counter, PixelBook* book, const uint8_t* ring) {
  const unsigned long long s = counter->step;
  record_after_step(book, s, ring);
  counter->step = s + 1ull;
}

// The observation buffer no longer matches the kept blocks (state restored, steps taken that did
// not write it): the next four steps write whole frames.
__global__ void pixel_book_forget_kernel(PixelBook* book) { book->valid_from = NOT_KNOWN; }

// F(t): the first ceil(n / 256) workgroups commit step t (reward / done to the caller, episode
// statistics) and, if `ahead`, stage step t+1; the remaining workgroups render step t's plane.
struct FusedStep {
  PongLaunch next;              // step0 = t + 1, actions = nullptr; reward / done = the CALLER's for step t
  const uint32_t* state_now;    // state after step t
  uint32_t* state_next;         // receives the state after step t + 1
  Staged now, ahead_to;         // staged step t (read), staging buffers for step t + 1 (written)
  uint8_t* plane;
  unsigned commit_blocks;       // ceil(n / 256)
  unsigned commit_at;           // index of the first commit workgroup: 0 = in front of the render groups
  int ahead;
};

// U: pages per render workgroup (see render_pages; 4 on long planes)
template <int U>
__global__ __launch_bounds__(256) void pixel_fused_step_kernel(FusedStep a) {
  __shared__ __align__(16) uint8_t page[U * PAGE];
  // The commit / lookahead workgroups sit in front of the render groups, where their latency hides
  // completely under the render, or, for the batch sizes where a few hundred workgroups in front of
  // the page stream cost more than they hide (measured, see the launcher), three quarters in.
  const unsigned pages = gridDim.x - a.commit_blocks;
  const unsigned first_commit = a.commit_at < pages ? a.commit_at : pages;
  if (blockIdx.x < first_commit || blockIdx.x >= first_commit + a.commit_blocks) {
    render_pages<U>(a.now.blocks, a.next.n, a.plane, blockIdx.x < first_commit ? blockIdx.x : blockIdx.x - a.commit_blocks, page);
    return;
  }
  const int64_t n = a.next.n;
  const int64_t i = (int64_t)(blockIdx.x - first_commit) * 256 + threadIdx.x;
  LaneEpisodes le;
  if (i < n) {
    const uint8_t d = a.now.done[i];
    a.next.reward[i] = a.now.reward[i];
    a.next.done[i] = d;
    if (d) {
      const int r = a.now.fin_ret[i];
      le.count = 1; le.length_sum = a.now.fin_len[i]; le.ret_sum_i = r; le.min_key = r; le.max_key = r;
    }
  }
  flush_wave_stats<false>(a.next.stats, le);
  if (a.ahead) stage_step<false>(a.next, a.state_now, a.state_next, a.ahead_to, i);
}

// ---- the fused step with the step counter in device memory ------------------------------------
// A launch recorded in a graph has frozen arguments, so everything the host alternates in
// pixel_pipe_step -- which staging buffers hold this step, which state buffer is current, which ring
// slot is written -- is derived inside the kernels from the counter: step s uses the staging
// buffers of parity s & 1 and ring slot s & 3.  The staged step's state is kept in the staging
// area too (stage_state) and copied into the handle's one state array when the step is committed,
// so that every other kernel of the handle keeps reading one committed state.  A device word says
// which step the staging buffers hold; only the fused launch writes it, only the launch in front
// of it reads it, and any step taken another way moves the counter past it.
struct CountedStep {
  PongLaunch pong;               // state = the committed state; reward / done = the caller's; counter
  uint32_t* stage_state[2];
  Staged stage[2];
  unsigned long long* staged_for;
  uint8_t* ring;
  unsigned commit_blocks;        // ceil(n / 256)
  unsigned commit_at;            // index of the first commit workgroup among the render groups
  int ahead;                     // stage the next step (in-kernel actions) under this step's render
};

constexpr int PREPARE_THREADS = 256;
// One workgroup: reads the counter, computes step s into the staging buffers unless they hold it
// already (the common case: the previous fused launch staged it), advances the counter.  A single
// workgroup needs no tickets: every thread has the counter's value before thread 0 moves it.
__global__ __launch_bounds__(PREPARE_THREADS) void pixel_counted_prepare_kernel(CountedStep a) {
  __shared__ unsigned long long seen[2];
  if (threadIdx.x == 0) {
    seen[0] = __hip_atomic_load(&a.pong.counter->step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    seen[1] = *a.staged_for;
  }
  __syncthreads();
  const unsigned long long s = seen[0];
  if (seen[1] != s) {                                        // workgroup-uniform
    PongLaunch p = a.pong;
    p.step0 = s;
    p.actions = nullptr;
    const int k = (int)(s & 1ull);
    for (int64_t i = threadIdx.x; i < p.n; i += PREPARE_THREADS) stage_step<false>(p, a.pong.state, a.stage_state[k], a.stage[k], i);
  }
  if (threadIdx.x == 0) a.pong.counter->step = s + 1ull;
}

template <int U>
__global__ __launch_bounds__(256) void pixel_fused_counted_kernel(CountedStep a) {
  __shared__ __align__(16) uint8_t page[U * PAGE];
  // the launch in front advanced the counter: this is the step with index counter - 1
  const unsigned long long c = __hip_atomic_load(&a.pong.counter->step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - 1ull;
  const uint32_t s_lo = __builtin_amdgcn_readfirstlane((uint32_t)c);
  const uint32_t s_hi = __builtin_amdgcn_readfirstlane((uint32_t)(c >> 32));
  const uint64_t s = ((uint64_t)s_hi << 32) | s_lo;
  const int k = (int)(s_lo & 1u);
  const int64_t n = a.pong.n;
  uint8_t* plane = a.ring + (int64_t)(s_lo & 3u) * n * FRAME_BYTES;
  // the grid is sized for the ring slot with the most pages; groups past this slot's pages find
  // nothing to do in render_pages
  const unsigned render_groups = gridDim.x - a.commit_blocks;
  const unsigned first_commit = a.commit_at < render_groups ? a.commit_at : render_groups;
  if (blockIdx.x < first_commit || blockIdx.x >= first_commit + a.commit_blocks) {
    render_pages<U>(a.stage[k].blocks, n, plane, blockIdx.x < first_commit ? blockIdx.x : blockIdx.x - a.commit_blocks, page);
    return;
  }
  const int64_t i = (int64_t)(blockIdx.x - first_commit) * 256 + threadIdx.x;
  LaneEpisodes le;
  if (i < n) {
    const uint8_t d = a.stage[k].done[i];
    a.pong.reward[i] = a.stage[k].reward[i];
    a.pong.done[i] = d;
    if (d) {
      const int r = a.stage[k].fin_ret[i];
      le.count = 1; le.length_sum = a.stage[k].fin_len[i]; le.ret_sum_i = r; le.min_key = r; le.max_key = r;
    }
    pong_store(a.pong.state, n, i, pong_load(a.stage_state[k], n, i));      // commit the state after step s
  }
  flush_wave_stats<false>(a.pong.stats, le);
  if (a.ahead) {
    PongLaunch next = a.pong;
    next.step0 = s + 1;
    next.actions = nullptr;
    stage_step<false>(next, a.stage_state[k], a.stage_state[k ^ 1], a.stage[k ^ 1], i);
  }
  if (blockIdx.x == first_commit && threadIdx.x == 0) *a.staged_for = a.ahead ? s + 1 : ~0ull;
}

__global__ void pixel_counted_forget_kernel(unsigned long long* staged_for) { *staged_for = ~0ull; }

int g_envs_per_wave = 0;   // 0 = chosen from N
bool g_streaming = false;

template <int MODE>
hipError_t launch_mode(const PixelLaunch& launch, hipStream_t stream) {
  // environments per wavefront: 16; 8 for small batches, which then spread over twice the SIMDs
  // (env-major ring step at N = 8192: 16.1 against 25.7 us; N = 16384: 29.8 / 30.2)
  const int epw = g_envs_per_wave ? g_envs_per_wave : (launch.pong.n <= 12288 ? 8 : 16);
  const int64_t waves = (launch.pong.n + epw - 1) / epw;
  const unsigned blocks = (unsigned)((waves + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
  const dim3 grid(blocks), block(WAVES_PER_BLOCK * WAVE);
  PixelLaunch a = launch;
  a.pong.ticket = blocks <= TICKET_MAX_BLOCKS;
#define MI355ENV_PIXEL_CASE(E)                                                                \
  case E:                                                                                     \
    if (g_streaming) hipLaunchKernelGGL((pixel_kernel<E, MODE, true>), grid, block, 0, stream, a); \
    else hipLaunchKernelGGL((pixel_kernel<E, MODE, false>), grid, block, 0, stream, a);       \
    break;
  switch (epw) {
    MI355ENV_PIXEL_CASE(4)
    MI355ENV_PIXEL_CASE(8)
    MI355ENV_PIXEL_CASE(16)
    MI355ENV_PIXEL_CASE(32)
    MI355ENV_PIXEL_CASE(64)
    default: return hipErrorInvalidValue;
  }
#undef MI355ENV_PIXEL_CASE
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess || MODE == MODE_RESET) return err;      // a reset only reads the counter
  return advance_step_counter_behind(a.pong.counter, a.pong.T, blocks, stream);
}

}  // namespace

// Launch-shape knobs for measurement sweeps: environments per wavefront (4..64, power of two) and
// whether frame stores carry the non-temporal hint.
bool set_pixel_tuning(int envs_per_wave, int streaming) {
  if (envs_per_wave != 0 && envs_per_wave != 4 && envs_per_wave != 8 && envs_per_wave != 16 &&
      envs_per_wave != 32 && envs_per_wave != 64)
    return false;
  g_envs_per_wave = envs_per_wave;
  g_streaming = streaming != 0;
  return true;
}

namespace {

int g_plane_path = 2;   // slot-major ring steps: 0 wave renderer, 1 page renderer without lookahead, 2 with
int g_traj_mode = 2;    // frame trajectories: 0 single launch, 1 chunked wherever possible, 2 = chosen from N

unsigned plane_pages(const uint8_t* plane, int64_t n) {
  const uintptr_t base = reinterpret_cast<uintptr_t>(plane);
  const uintptr_t end = base + (uintptr_t)n * FRAME_BYTES;
  return (unsigned)(((end + PAGE - 1) >> 12) - (base >> 12));
}

Staged staged_of(const PixelPipe& p, int k) {
  return Staged{p.blocks[k], p.reward[k], p.done[k], p.fin_ret[k], p.fin_len[k]};
}

}  // namespace

bool set_traj_mode(int mode) {
  if (mode < 0 || mode > 2) return false;
  g_traj_mode = mode;
  return true;
}

bool set_plane_path(int mode) {
  if (mode < 0 || mode > 2) return false;
  g_plane_path = mode;
  return true;
}
int pixel_plane_mode() { return g_plane_path; }

hipError_t pixel_pipe_create(PixelPipe& p, int64_t n, bool delta_updates, bool device_counter) {
  auto up = [](size_t b) { return (b + 255) & ~(size_t)255; };
  const size_t state_b = up((size_t)PONG_FIELDS * n * 4), blocks_b = up((size_t)3 * n * 4);
  const size_t word_b = up((size_t)n * 4), done_b = up((size_t)n);
  // trajectory staging: room for at least one step of all environments and for a few hundred
  // thousand frames, so that small batches are rendered many steps at a time
  p.traj_cap = n > TRAJ_MIN_FRAMES ? n : TRAJ_MIN_FRAMES;
  const size_t traj_b = up((size_t)3 * (size_t)p.traj_cap * 4);
  const size_t hist_b = delta_updates ? up((size_t)5 * 3 * (size_t)n * 4) : 0;
  const size_t book_b = delta_updates ? up(sizeof(PixelBook)) : 0;
  const size_t counted_b = device_counter ? state_b + 256 : 0;
  hipError_t err = hipMalloc(&p.slab, state_b + 2 * (blocks_b + 3 * word_b + done_b) + traj_b + hist_b + book_b + counted_b);
  if (err != hipSuccess) return err;
  char* at = static_cast<char*>(p.slab);
  if (device_counter) {
    p.staged_for = reinterpret_cast<unsigned long long*>(at); at += 256;
    p.stage_state[1] = reinterpret_cast<uint32_t*>(at); at += state_b;
    const unsigned long long none = ~0ull;
    err = hipMemcpy(p.staged_for, &none, sizeof none, hipMemcpyHostToDevice);
    if (err != hipSuccess) { (void)hipFree(p.slab); p.slab = nullptr; return err; }
  }
  if (delta_updates) {
    p.hist = reinterpret_cast<uint32_t*>(at); at += hist_b;
    p.book = at; at += book_b;
    const PixelBook fresh = {NOT_KNOWN, 0ull, 0ull, 0ull};
    *reinterpret_cast<PixelBook*>(p.host_book) = fresh;
    err = hipMemcpy(p.book, &fresh, sizeof fresh, hipMemcpyHostToDevice);
    if (err != hipSuccess) { (void)hipFree(p.slab); p.slab = nullptr; return err; }
  }
  p.state_alt = reinterpret_cast<uint32_t*>(at); at += state_b;
  if (device_counter) p.stage_state[0] = p.state_alt;      // such a handle never alternates its state buffers
  p.traj_blocks = reinterpret_cast<uint32_t*>(at); at += traj_b;
  for (int k = 0; k < 2; ++k) {
    p.blocks[k] = reinterpret_cast<uint32_t*>(at); at += blocks_b;
    p.reward[k] = reinterpret_cast<float*>(at); at += word_b;
    p.fin_ret[k] = reinterpret_cast<int32_t*>(at); at += word_b;
    p.fin_len[k] = reinterpret_cast<int32_t*>(at); at += word_b;
    p.done[k] = reinterpret_cast<uint8_t*>(at); at += done_b;
  }
  p.staged = false;
  return hipSuccess;
}

void pixel_pipe_destroy(PixelPipe& p) {
  if (p.slab) { (void)hipFree(p.slab); p.slab = nullptr; }
  p.staged = false;
}

hipError_t pixel_pipe_step(PixelPipe& p, uint32_t*& state, const PixelLaunch& a, bool lookahead,
                           hipStream_t stream) {
  const int64_t n = a.pong.n;
  const int k = (int)(a.pong.step0 & 1);
  const unsigned commit_blocks = (unsigned)((n + 255) / 256);
  if (!(p.staged && a.pong.actions == nullptr)) {
    // D(t): stage this step from the committed state into the other state buffer
    hipLaunchKernelGGL(pixel_dynamics_kernel<false>, dim3(commit_blocks), dim3(256), 0, stream, a.pong,
                       state, p.state_alt, staged_of(p, k));
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  // whichever launch staged step t wrote its state into state_alt: that is the committed state now
  uint32_t* const after_t = p.state_alt;
  p.state_alt = state;
  state = after_t;

  FusedStep f{};
  f.next = a.pong;
  f.next.step0 = a.pong.step0 + 1;
  f.next.actions = nullptr;
  f.state_now = state;
  f.state_next = p.state_alt;
  f.now = staged_of(p, k);
  f.ahead_to = staged_of(p, k ^ 1);
  f.plane = a.ring + (int64_t)(a.pong.step0 & 3) * n * FRAME_BYTES;
  f.commit_blocks = commit_blocks;
  // Where the commit / lookahead workgroups sit among the render groups (us per step, in front /
  // three quarters in / behind): N = 32768: 42.0 / 37.0 / 38.0; N = 65536 (four pages per render
  // workgroup from here on): 75.7 / 85.6 / 85.0; N = 262144: 297.5 / 309.1 / 315.8.
  const unsigned render_pages_total = plane_pages(f.plane, n);
  f.commit_at = (n <= 24576 || render_pages_total >= 65536u) ? 0u : render_pages_total / 4u * 3u;
  f.ahead = lookahead ? 1 : 0;
  // long planes: four pages per render workgroup (N = 131072: 187 -> 163 us per step, N = 262144:
  // 393 -> 317 us; see render_pages)
  const unsigned pages = plane_pages(f.plane, n);
  if (pages >= 65536u)
    hipLaunchKernelGGL(pixel_fused_step_kernel<4>, dim3(f.commit_blocks + (pages + 3u) / 4u), dim3(256), 0, stream, f);
  else
    hipLaunchKernelGGL(pixel_fused_step_kernel<1>, dim3(f.commit_blocks + pages), dim3(256), 0, stream, f);
  p.staged = lookahead;
  return hipGetLastError();
}

// One ring step of a slot-major handle with a device step counter: the lane-per-environment pass
// (reads and advances the counter, writes reward / done to the caller and the cell blocks to
// library scratch), then the page renderer, which derives the slot from the advanced counter.
hipError_t pixel_counted_forget(const PixelPipe& p, hipStream_t stream) {
  if (!p.staged_for) return hipSuccess;
  hipLaunchKernelGGL(pixel_counted_forget_kernel, dim3(1), dim3(1), 0, stream, p.staged_for);
  return hipGetLastError();
}

hipError_t pixel_counted_step(const PixelPipe& p, const PixelLaunch& a, hipStream_t stream) {
  const int64_t n = a.pong.n;
  if (!a.pong.actions && p.staged_for && g_plane_path == 2) {
    // Step s = the counter's value: (1) one workgroup makes sure the staging buffers of parity s & 1
    // hold step s and moves the counter on; (2) the fused launch hands step s to the caller, commits
    // its state, renders its plane and stages step s + 1 under the render.  N = 16384: 22.5 us per
    // step against 23.0 for dynamics launch + renderer and 18.0 for the host-counter path, which
    // needs no launch in front: that launch's loads and store queue behind the plane the previous
    // launch is still writing back (1.2 us at best, 4.6 us on average in the kernel trace, 1024 or
    // 256 threads alike), and only a kernel boundary tells that every workgroup has read the
    // counter before it moves.
    CountedStep c{};
    c.pong = a.pong;
    c.pong.T = 1;
    for (int k = 0; k < 2; ++k) { c.stage_state[k] = p.stage_state[k]; c.stage[k] = staged_of(p, k); }
    c.staged_for = p.staged_for;
    c.ring = a.ring;
    c.commit_blocks = (unsigned)((n + 255) / 256);
    c.ahead = 1;
    unsigned pages = 0;
    for (int slot = 0; slot < 4; ++slot) {
      const unsigned here = plane_pages(a.ring + (int64_t)slot * n * FRAME_BYTES, n);
      pages = here > pages ? here : pages;
    }
    c.commit_at = (n <= 24576 || pages >= 65536u) ? 0u : pages / 4u * 3u;
    hipLaunchKernelGGL(pixel_counted_prepare_kernel, dim3(1), dim3(PREPARE_THREADS), 0, stream, c);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    if (pages >= 65536u)
      hipLaunchKernelGGL(pixel_fused_counted_kernel<4>, dim3(c.commit_blocks + (pages + 3u) / 4u), dim3(256), 0, stream, c);
    else
      hipLaunchKernelGGL(pixel_fused_counted_kernel<1>, dim3(c.commit_blocks + pages), dim3(256), 0, stream, c);
    return hipGetLastError();
  }
  PongLaunch d = a.pong;
  d.T = 1;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  d.ticket = blocks <= TICKET_MAX_BLOCKS;
  if (d.actions) hipLaunchKernelGGL(pixel_traj_dynamics_kernel<true>, dim3(blocks), dim3(256), 0, stream, d, p.blocks[0], n);
  else hipLaunchKernelGGL(pixel_traj_dynamics_kernel<false>, dim3(blocks), dim3(256), 0, stream, d, p.blocks[0], n);
  hipError_t err = hipGetLastError();
  if (err == hipSuccess) err = advance_step_counter_behind(d.counter, 1, blocks, stream);   // before the renderer reads it
  if (err != hipSuccess) return err;
  unsigned pages = 0;
  for (int slot = 0; slot < 4; ++slot) {
    const unsigned here = plane_pages(a.ring + (int64_t)slot * n * FRAME_BYTES, n);
    pages = here > pages ? here : pages;
  }
  hipLaunchKernelGGL(plane_render_counted_kernel, dim3(pages), dim3(256), 0, stream, p.blocks[0], n, a.ring,
                     a.pong.counter);
  return hipGetLastError();
}

// The host's copy of the record lives in PixelPipe::host_book (same layout).
static PixelBook* host_record(PixelPipe& p) { return reinterpret_cast<PixelBook*>(p.host_book); }
static_assert(sizeof(PixelBook) <= sizeof(PixelPipe::host_book), "PixelPipe::host_book is too small for the record");

hipError_t pixel_update_after_reset(PixelPipe& p, const uint32_t* state, int64_t n, uint64_t step,
                                    const StepCounter* counter, const uint8_t* ring, hipStream_t stream) {
  if (!p.hist || !p.book) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pixel_book_reset_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, state, n,
                     step, counter, static_cast<PixelBook*>(p.book), p.hist, ring);
  const hipError_t err = hipGetLastError();
  if (err == hipSuccess && !counter) {
    host_record(p)->valid_from = step;
    host_record(p)->ring = (unsigned long long)reinterpret_cast<uintptr_t>(ring);
  }
  return err;
}

hipError_t pixel_update_forget(PixelPipe& p, hipStream_t stream) {
  if (!p.book) return hipSuccess;
  host_record(p)->valid_from = NOT_KNOWN;
  hipLaunchKernelGGL(pixel_book_forget_kernel, dim3(1), dim3(1), 0, stream, static_cast<PixelBook*>(p.book));
  return hipGetLastError();
}

hipError_t pixel_update_counts(PixelPipe& p, bool device_counter, int64_t* delta_steps, int64_t* full_steps,
                               hipStream_t stream) {
  *delta_steps = 0; *full_steps = 0;
  if (!p.book) return hipSuccess;
  PixelBook host = *host_record(p);
  if (device_counter) {
    hipError_t err = hipMemcpyAsync(&host, p.book, sizeof host, hipMemcpyDeviceToHost, stream);
    if (err == hipSuccess) err = hipStreamSynchronize(stream);
    if (err != hipSuccess) return err;
  }
  *delta_steps = (int64_t)host.delta_steps;
  *full_steps = (int64_t)host.full_steps;
  return hipSuccess;
}

hipError_t pixel_update_step(PixelPipe& p, const PixelLaunch& a, bool ordered, hipStream_t stream) {
  if (!p.hist || !p.book || !a.ring) return hipErrorInvalidValue;
  const int64_t n = a.pong.n;
  UpdateStep u{};
  u.pong = a.pong;
  u.pong.T = 1;
  u.known_by_host = (!a.pong.counter && record_says_known(host_record(p), a.pong.step0, a.ring)) ? 1 : 0;
  u.book = static_cast<PixelBook*>(p.book);
  u.hist = p.hist;
  u.ring = a.ring;
  // frame of slot k of environment i: slot-major (k n + i) frames into the ring, else (4 i + k)
  const bool planes = !ordered && a.slot_major;
  u.stride = planes ? FRAME_BYTES : 4 * (int64_t)FRAME_BYTES;
  u.slot_pitch = planes ? n * (int64_t)FRAME_BYTES : FRAME_BYTES;
  if (!a.pong.counter) {
    const uint64_t s = a.pong.step0;
    for (int f = 0; f < 5; ++f) u.entry[f] = p.hist + (int64_t)((s + 1 + f) % 5) * 3 * n;
    u.base = a.ring + (ordered ? 0 : (int64_t)(s & 3) * u.slot_pitch);
  }
  // Few environments per workgroup: their step runs on one wavefront while the other three wait,
  // so small groups start their pixel work sooner (ring, N = 16384: 15.6 us per step with 64
  // environments per workgroup, 10.7 with 32, 9.3 with 16, 8.8 with 8; stack: 22.1 with 16, 19.0
  // with 8, 22.1 with 4); large batches have workgroups enough to hide that and prefer fewer of
  // them (ring, N = 131072: 55.7 us with 16, 61.3 with 8).
  const bool small = n <= 32768;
  const dim3 grid((unsigned)(small ? (n + 7) / 8 : (n + 15) / 16)), block(256);
  const int mode = u.pong.counter ? DEVICE_DECIDES : (u.known_by_host ? HOST_REPAIR : HOST_WHOLE);
#define MI355ENV_UPDATE_CASE(ORD, MODE)                                                                    \
  if (ordered == ORD && mode == MODE) {                                                                   \
    if (small) hipLaunchKernelGGL((pixel_update_step_kernel<8, ORD, MODE>), grid, block, 0, stream, u);   \
    else hipLaunchKernelGGL((pixel_update_step_kernel<16, ORD, MODE>), grid, block, 0, stream, u);        \
  }
  MI355ENV_UPDATE_CASE(false, HOST_REPAIR)
  MI355ENV_UPDATE_CASE(false, HOST_WHOLE)
  MI355ENV_UPDATE_CASE(false, DEVICE_DECIDES)
  MI355ENV_UPDATE_CASE(true, HOST_REPAIR)
  MI355ENV_UPDATE_CASE(true, HOST_WHOLE)
  MI355ENV_UPDATE_CASE(true, DEVICE_DECIDES)
#undef MI355ENV_UPDATE_CASE
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  if (u.pong.counter) {
    hipLaunchKernelGGL(pixel_book_commit_kernel, dim3(1), dim3(1), 0, stream, u.pong.counter, u.book,
                       static_cast<const uint8_t*>(a.ring));
    err = hipGetLastError();
  } else {
    record_after_step(host_record(p), a.pong.step0, a.ring);
  }
  return err;
}

hipError_t launch_pixel_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                              const StepCounter* counter, uint8_t* ring, bool slot_major, uint32_t* blocks,
                              hipStream_t stream) {
  // the page renderer's dynamics pass takes the step from the host; a device counter goes through
  // the single-launch renderer, which reads it
  if (!counter && slot_major && g_plane_path != 0 && blocks && n < (int64_t)4000000) {
    PongLaunch p{};
    p.state = state; p.n = n; p.seed = seed; p.step0 = step; p.T = 1;
    const Staged st{blocks, nullptr, nullptr, nullptr, nullptr};
    hipLaunchKernelGGL(pixel_dynamics_kernel<true>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       stream, p, static_cast<const uint32_t*>(nullptr), state, st);
    hipError_t err = hipGetLastError();
    for (int slot = 0; slot < 4 && err == hipSuccess; ++slot) {
      uint8_t* plane = ring + (int64_t)slot * n * FRAME_BYTES;
      hipLaunchKernelGGL(plane_render_kernel<1>, dim3(plane_pages(plane, n)), dim3(256), 0, stream, blocks, n, plane);
      err = hipGetLastError();
    }
    return err;
  }
  PixelLaunch a{};
  a.slot_major = slot_major;
  a.pong.state = state; a.pong.n = n; a.pong.seed = seed; a.pong.step0 = step; a.pong.T = 1;
  a.pong.counter = const_cast<StepCounter*>(counter);      // only read by the reset kernel
  a.ring = ring;
  return launch_mode<MODE_RESET>(a, stream);
}

// Frame trajectory frames[T][n][84][84].  Rendering is independent per frame, only the dynamics are
// sequential, so the launch is cut into chunks of as many steps as the staging area holds: a
// lane-per-environment pass runs the chunk's steps and leaves 12 bytes per frame (three cell
// blocks), then the page renderer writes the chunk's frames as one long plane.  Parallelism is then
// steps x environments, not environments: N = 1024 x T = 256 goes from 0.36 to 3.4 TB/s, N = 4096 x
// T = 64 from 1.4 to 4.9 TB/s.  The single-launch renderer, whose wavefronts each own a few
// environments for all T steps, gives 5.6 TB/s at N = 16384 and 5.0-5.1 TB/s from N = 32768 on; the
// staged path gives 5.5 and 5.6-5.7 TB/s there, so it takes every size but N = 16384 ... 24575
// (batches beyond the staging area and handles with a device step counter take the single launch).
hipError_t launch_pixel_rollout(const PixelLaunch& a, PixelPipe& pipe, hipStream_t stream) {
  if (!a.frames) return launch_mode<MODE_RING>(a, stream);
  const int64_t n = a.pong.n;
  // the chunks' step indices are computed on the host: not with a step counter in device memory
  const bool chunked = !a.pong.counter && (g_traj_mode == 1 || (g_traj_mode == 2 && (n < 16384 || n >= 24576)));
  if (!chunked || !pipe.traj_blocks || n > pipe.traj_cap || pipe.traj_cap >= (int64_t)4000000)
    return launch_mode<MODE_FRAMES>(a, stream);
  const int32_t steps_per_chunk = (int32_t)(pipe.traj_cap / n);
  for (int32_t t0 = 0; t0 < a.pong.T; t0 += steps_per_chunk) {
    const int32_t tc = a.pong.T - t0 < steps_per_chunk ? a.pong.T - t0 : steps_per_chunk;
    PongLaunch p = a.pong;
    p.step0 = a.pong.step0 + (uint64_t)t0;
    p.T = tc;
    if (p.actions) p.actions += (int64_t)t0 * n;
    p.reward += (int64_t)t0 * n;
    p.done += (int64_t)t0 * n;
    const int64_t frames = (int64_t)tc * n;
    if (p.actions)
      hipLaunchKernelGGL(pixel_traj_dynamics_kernel<true>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p,
                         pipe.traj_blocks, frames);
    else
      hipLaunchKernelGGL(pixel_traj_dynamics_kernel<false>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p,
                         pipe.traj_blocks, frames);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    uint8_t* plane = a.frames + (int64_t)t0 * n * FRAME_BYTES;
    // long planes: several pages per workgroup (see render_pages)
    const unsigned pages = plane_pages(plane, frames);
    if (pages >= 65536u)
      hipLaunchKernelGGL(plane_render_kernel<RENDER_U>, dim3((pages + RENDER_U - 1) / RENDER_U), dim3(256), 0, stream,
                         pipe.traj_blocks, frames, plane);
    else
      hipLaunchKernelGGL(plane_render_kernel<1>, dim3(pages), dim3(256), 0, stream, pipe.traj_blocks, frames, plane);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  return hipSuccess;
}

}  // namespace envk

// ---- one entry point that allocates nothing ---------------------------------------------------
// env_step_pixels_noalloc (include/mi355env.h): the slot-major pixel step without a handle, for
// callers that cannot allocate.  The two kinds of scratch a handle's pixel step keeps in memory from
// env_create -- the 256 partial copies of the episode statistics and the staged cell blocks that
// the lane-per-environment pass hands to the page renderer, 12 bytes per environment -- live in
// one file-scope device array instead, of fixed size.  Every device has its own copy of the array
// at its own address; the address is asked for once per device and kept.
#include <mutex>

#include "../../include/mi355env.h"

namespace envk {
namespace {

struct NoAllocScratch {
  DeviceStats stripes[STATS_STRIPES];                      // partial episode statistics, 32 KiB
  uint32_t blocks[3 * ENV_NOALLOC_MAX_ENVS];               // staged cell blocks [3][n], 768 KiB
};

__global__ __launch_bounds__(STATS_STRIPES) void noalloc_clear_stats_kernel(DeviceStats* __restrict__ stripes) {
  DeviceStats z;
  z.episodes = 0; z.length_sum = 0; z.return_sum_i = 0; z.return_sum_f = 0.0;
  z.return_min_key = INT32_MAX; z.return_max_key = INT32_MIN; z.nonfinite = 0;
  stripes[threadIdx.x] = z;
}

// One wavefront adds the copies up and writes the result in the boundary's layout.
__global__ __launch_bounds__(64) void noalloc_reduce_stats_kernel(const DeviceStats* __restrict__ stripes,
                                                                  env_stats_t* __restrict__ out) {
  long long episodes = 0, length = 0, ret = 0;
  int mn = INT32_MAX, mx = INT32_MIN;
  for (int k = threadIdx.x; k < STATS_STRIPES; k += 64) {
    const DeviceStats s = stripes[k];
    episodes += (long long)s.episodes; length += (long long)s.length_sum; ret += s.return_sum_i;
    mn = min(mn, s.return_min_key); mx = max(mx, s.return_max_key);
  }
  episodes = wave_sum(episodes); length = wave_sum(length); ret = wave_sum(ret);
  mn = wave_min(mn); mx = wave_max(mx);
  if (threadIdx.x == 0) {
    out->episodes = episodes; out->length_sum = length; out->return_sum = (double)ret;
    out->return_min = episodes > 0 ? (double)mn : (double)INFINITY;
    out->return_max = episodes > 0 ? (double)mx : -(double)INFINITY;
    out->nonfinite = 0;
  }
}

}  // namespace
}  // namespace envk

static __device__ __align__(256) unsigned char scratch[sizeof(envk::NoAllocScratch)];

namespace {

constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_noalloc_mutex;
void* g_scratch_of_device[NOALLOC_MAX_DEVICES] = {};        // device address of `scratch`, per device
struct CheckedRange { int device; const void* p; size_t bytes; };
CheckedRange g_noalloc_seen[16] = {};
int g_noalloc_seen_next = 0;

// Device address of this device's copy of `scratch` (the array's name is only a host-side handle).
int noalloc_scratch(int device, envk::NoAllocScratch** out) {
  std::lock_guard<std::mutex> lock(g_noalloc_mutex);
  if (!g_scratch_of_device[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return ENV_E_HIP; }
    g_scratch_of_device[device] = p;
  }
  *out = static_cast<envk::NoAllocScratch*>(g_scratch_of_device[device]);
  return ENV_OK;
}

// [p, p + bytes) lies inside one device allocation; ranges that passed are remembered (no driver
// query for them again, so that a call with known buffers can be recorded by a stream capture).
bool noalloc_range_ok(int device, const void* p, size_t bytes, size_t align) {
  if (!p || (reinterpret_cast<uintptr_t>(p) & (align - 1))) return false;
  std::lock_guard<std::mutex> lock(g_noalloc_mutex);
  for (const CheckedRange& r : g_noalloc_seen)
    if (r.p == p && r.device == device && r.bytes >= bytes) return true;
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, p) != hipSuccess) { (void)hipGetLastError(); return false; }
  if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) return false;
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange(&base, &size, const_cast<void*>(p)) != hipSuccess) { (void)hipGetLastError(); return false; }
  const uintptr_t lo = reinterpret_cast<uintptr_t>(base), q = reinterpret_cast<uintptr_t>(p);
  if (q < lo || q + bytes > lo + size) return false;
  g_noalloc_seen[g_noalloc_seen_next] = {device, p, bytes};
  g_noalloc_seen_next = (g_noalloc_seen_next + 1) % 16;
  return true;
}

}  // namespace

extern "C" int env_step_pixels_noalloc(int64_t n_envs, uint64_t seed, uint64_t step, int32_t max_score,
                                       void* state_dev, const uint8_t* actions_dev, uint8_t* ring_dev,
                                       float* reward_dev, uint8_t* done_dev, env_stats_t* stats_dev,
                                       void* hip_stream) {
  using namespace envk;
  if (n_envs <= 0 || max_score <= 0) return ENV_E_ARG;
  if (n_envs > ENV_NOALLOC_MAX_ENVS) return ENV_E_TOO_LARGE;
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) { (void)hipGetLastError(); return ENV_E_HIP; }
  if (device < 0 || device >= NOALLOC_MAX_DEVICES) return ENV_E_UNSUPPORTED;
  const size_t n = (size_t)n_envs;
  if (!noalloc_range_ok(device, state_dev, n * PONG_FIELDS * 4, 4)) return ENV_E_ARG;
  if (!noalloc_range_ok(device, ring_dev, n * 4 * FRAME_BYTES, 16)) return ENV_E_ARG;
  if (!noalloc_range_ok(device, reward_dev, n * sizeof(float), 4)) return ENV_E_ARG;
  if (!noalloc_range_ok(device, done_dev, n, 1)) return ENV_E_ARG;
  if (actions_dev && !noalloc_range_ok(device, actions_dev, n, 1)) return ENV_E_ARG;
  if (stats_dev && !noalloc_range_ok(device, stats_dev, sizeof(env_stats_t), 8)) return ENV_E_ARG;
  NoAllocScratch* sc = nullptr;
  const int rc = noalloc_scratch(device, &sc);
  if (rc != ENV_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);

  // the array keeps the previous call's contents: the statistics must start empty (a fill kernel,
  // not a memset node, so that the call can be recorded in a graph); the cell blocks of all n
  // environments are written by the pass below before the renderer reads them
  hipLaunchKernelGGL(noalloc_clear_stats_kernel, dim3(1), dim3(STATS_STRIPES), 0, stream, sc->stripes);
  if (hipGetLastError() != hipSuccess) return ENV_E_HIP;
  PongLaunch d{};
  d.state = static_cast<uint32_t*>(state_dev); d.n = n_envs; d.seed = seed; d.step0 = step;
  d.counter = nullptr; d.ticket = 0; d.T = 1; d.max_score = max_score; d.actions = actions_dev;
  d.obs = nullptr; d.reward = reward_dev; d.done = done_dev; d.stats = sc->stripes;
  const unsigned groups = (unsigned)((n_envs + 255) / 256);
  if (actions_dev) hipLaunchKernelGGL(pixel_traj_dynamics_kernel<true>, dim3(groups), dim3(256), 0, stream, d, sc->blocks, n_envs);
  else hipLaunchKernelGGL(pixel_traj_dynamics_kernel<false>, dim3(groups), dim3(256), 0, stream, d, sc->blocks, n_envs);
  if (hipGetLastError() != hipSuccess) return ENV_E_HIP;
  uint8_t* plane = ring_dev + (int64_t)(step & 3ull) * n_envs * FRAME_BYTES;
  const unsigned pages = plane_pages(plane, n_envs);
  if (pages >= 65536u)
    hipLaunchKernelGGL(plane_render_kernel<RENDER_U>, dim3((pages + RENDER_U - 1) / RENDER_U), dim3(256), 0, stream,
                       sc->blocks, n_envs, plane);
  else
    hipLaunchKernelGGL(plane_render_kernel<1>, dim3(pages), dim3(256), 0, stream, sc->blocks, n_envs, plane);
  if (hipGetLastError() != hipSuccess) return ENV_E_HIP;
  if (stats_dev) {
    hipLaunchKernelGGL(noalloc_reduce_stats_kernel, dim3(1), dim3(64), 0, stream, sc->stripes, stats_dev);
    if (hipGetLastError() != hipSuccess) return ENV_E_HIP;
  }
  return ENV_OK;
}

