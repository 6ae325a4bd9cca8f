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
// wavefront streams several KiB on its own).  The plane is therefore rendered by two launches:
//   1. pixel_dynamics_kernel: one lane per environment; transition, state / reward / done stores,
//      and the three cell blocks of the new frame (12 bytes per environment) into `blocks`;
//   2. plane_render_kernel: one workgroup per 4 KiB page of the plane.  A page overlaps at most two
//      frames; their six cell blocks arrive by scalar loads, the lit pixels that fall inside the
//      page are poked into a zeroed 4 KiB LDS page, and every thread stores its 16 bytes.
// ---------------------------------------------------------------------------------------------
template <bool RESET>
__global__ __launch_bounds__(256) void pixel_dynamics_kernel(PongLaunch a, uint32_t* __restrict__ blocks) {
  const int64_t n = a.n;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool live = i < n;
  PongLane s;
  LaneEpisodes le;
  if (RESET) {
    s = pong_initial(a.seed, (uint32_t)i, a.step0);
  } else {
    s = live ? pong_load(a.state, n, i) : pong_idle_lane();
    const Draw4 d = philox_draw(a.seed, (uint32_t)i, a.step0, 0u);
    int action = pong_action_from_word(d.w0);
    if (a.actions) action = live ? (int)a.actions[i] : 0;
    const PongEvent ev = pong_transition(s, action, d.w1, d.w2, a.max_score);
    if (live) {
      a.reward[i] = ev.reward;
      a.done[i] = ev.done ? 1 : 0;
      if (ev.done) {
        le.count = 1; le.length_sum = ev.fin_len; le.ret_sum_i = ev.fin_ret;
        le.min_key = ev.fin_ret; le.max_key = ev.fin_ret;
      }
    }
  }
  if (live) {
    pong_store(a.state, n, i, s);
    blocks[0 * n + i] = cell_block(140.0f, s.pa, 4.0f, 16.0f);
    blocks[1 * n + i] = cell_block(16.0f, s.po, 4.0f, 16.0f);
    blocks[2 * n + i] = cell_block(s.bx, s.by, 2.0f, 2.0f);
  }
  if (!RESET) flush_wave_stats<false>(a.stats, le);
}

constexpr int PAGE = 4096;

// plane: first byte of the plane (16-byte aligned), n frames long.  Workgroup b handles the b-th
// 4 KiB-aligned page that intersects it.
__global__ __launch_bounds__(256) void plane_render_kernel(const uint32_t* __restrict__ blocks, int64_t n,
                                                           uint8_t* __restrict__ plane) {
  __shared__ __align__(16) uint8_t page[PAGE];
  const int tid = threadIdx.x;
  const uintptr_t base = reinterpret_cast<uintptr_t>(plane);
  const int64_t total = n * FRAME_BYTES;
  // byte offsets relative to the start of the plane; the first page may begin before it
  const int64_t page_off = (int64_t)blockIdx.x * PAGE - (int64_t)(base & (PAGE - 1));
  const int64_t lo = page_off < 0 ? 0 : page_off;
  const int64_t hi = page_off + PAGE < total ? page_off + PAGE : total;
  const int64_t f_first = lo / FRAME_BYTES;
  const int64_t f_last = (hi - 1) / FRAME_BYTES;      // f_first or f_first + 1

  // threads 0..191: (frame, rectangle) pair tid / 32, pixel tid % 32 of a 4-column x 8-row patch
  // (a paddle covers at most 4 x 8 cells, the ball at most 3 x 2).  The cell block is loaded
  // before the page is zeroed so that its latency overlaps the zeroing and the barrier.
  const int pair = tid >> 5;
  const bool from_last = pair >= 3;
  const bool candidate = pair < 6 && !(from_last && f_last == f_first);
  const int64_t f = from_last ? f_last : f_first;
  uint32_t blk = 0;
  if (candidate) blk = blocks[(int64_t)(from_last ? pair - 3 : pair) * n + f];

  chunk_t* page16 = reinterpret_cast<chunk_t*>(page);
  page16[tid] = chunk_t{0, 0, 0, 0};
  __syncthreads();

  if (candidate) {
    const int c_lo = blk & 0xff, c_end = (blk >> 8) & 0xff;
    const int r_lo = (blk >> 16) & 0xff, r_end = blk >> 24;
    const int c = c_lo + (tid & 3), r = r_lo + ((tid >> 2) & 7);
    const int64_t off = f * FRAME_BYTES + r * FRAME_SIDE + c - page_off;
    if (c < c_end && r < r_end && off >= 0 && off < PAGE) page[off] = 255;
  }
  __syncthreads();

  const int64_t mine = page_off + 16 * tid;
  if (mine >= lo && mine < hi) *reinterpret_cast<chunk_t*>(plane + mine) = page16[tid];
}

int g_envs_per_wave = 16;
bool g_streaming = false;

template <int MODE>
hipError_t launch_mode(const PixelLaunch& a, hipStream_t stream) {
  const int epw = g_envs_per_wave;
  const int64_t waves = (a.pong.n + epw - 1) / epw;
  const unsigned blocks = (unsigned)((waves + WAVES_PER_BLOCK - 1) / WAVES_PER_BLOCK);
  const dim3 grid(blocks), block(WAVES_PER_BLOCK * WAVE);
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
  return hipGetLastError();
}

}  // namespace

// Launch-shape knobs for measurement sweeps: environments per wavefront (4..64, power of two) and
// whether frame stores carry the non-temporal hint.
bool set_pixel_tuning(int envs_per_wave, int streaming) {
  if (envs_per_wave != 4 && envs_per_wave != 8 && envs_per_wave != 16 && envs_per_wave != 32 &&
      envs_per_wave != 64)
    return false;
  g_envs_per_wave = envs_per_wave;
  g_streaming = streaming != 0;
  return true;
}

namespace {

bool g_plane_path = true;   // slot-major ring steps go through the two-launch plane renderer

hipError_t launch_plane(const uint32_t* blocks, int64_t n, uint8_t* plane, hipStream_t stream) {
  const uintptr_t base = reinterpret_cast<uintptr_t>(plane);
  const uintptr_t end = base + (uintptr_t)n * FRAME_BYTES;
  const unsigned pages = (unsigned)(((end + PAGE - 1) >> 12) - (base >> 12));
  hipLaunchKernelGGL(plane_render_kernel, dim3(pages), dim3(256), 0, stream, blocks, n, plane);
  return hipGetLastError();
}

}  // namespace

bool set_plane_path(int on) { g_plane_path = on != 0; return true; }

hipError_t launch_pixel_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                              uint8_t* ring, bool slot_major, uint32_t* blocks, hipStream_t stream) {
  if (slot_major && g_plane_path && blocks) {
    PongLaunch p{};
    p.state = state; p.n = n; p.seed = seed; p.step0 = step; p.T = 1;
    hipLaunchKernelGGL(pixel_dynamics_kernel<true>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                       stream, p, blocks);
    hipError_t err = hipGetLastError();
    for (int slot = 0; slot < 4 && err == hipSuccess; ++slot)
      err = launch_plane(blocks, n, ring + (int64_t)slot * n * FRAME_BYTES, stream);
    return err;
  }
  PixelLaunch a{};
  a.slot_major = slot_major;
  a.pong.state = state; a.pong.n = n; a.pong.seed = seed; a.pong.step0 = step; a.pong.T = 1;
  a.ring = ring;
  return launch_mode<MODE_RESET>(a, stream);
}

hipError_t launch_pixel_rollout(const PixelLaunch& a, hipStream_t stream) {
  if (a.ring && a.slot_major && g_plane_path && a.blocks && a.pong.T == 1) {
    hipLaunchKernelGGL(pixel_dynamics_kernel<false>, dim3((unsigned)((a.pong.n + 255) / 256)), dim3(256),
                       0, stream, a.pong, a.blocks);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int64_t slot = (int64_t)(a.pong.step0 & 3);
    return launch_plane(a.blocks, a.pong.n, a.ring + slot * a.pong.n * FRAME_BYTES, stream);
  }
  if (a.frames) return launch_mode<MODE_FRAMES>(a, stream);
  return launch_mode<MODE_RING>(a, stream);
}

}  // namespace envk
