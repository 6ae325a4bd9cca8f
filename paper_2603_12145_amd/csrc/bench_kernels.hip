// Yardstick kernels for measurements (not part of the environment path): a plain fill and a plain
// copy with 16-byte accesses.  They calibrate the HBM counters (known bytes per launch) and give
// the write / copy bandwidth a trivial kernel reaches on the same device.
#include <hip/hip_runtime.h>
#include <chrono>
#include <stdint.h>

namespace {

typedef uint32_t vec16 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void fill16_kernel(vec16* __restrict__ dst, size_t chunks, uint32_t value) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const vec16 v = {value, value, value, value};
  for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < chunks; k += stride) dst[k] = v;
}

__global__ __launch_bounds__(256) void copy16_kernel(vec16* __restrict__ dst, const vec16* __restrict__ src,
                                                     size_t chunks) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < chunks; k += stride) dst[k] = src[k];
}

// One 4 KiB page per 256-thread workgroup, one 16-byte store per thread, workgroups in address
// order: the launch shape with the highest write rate found on this device.
__global__ __launch_bounds__(256) void fill_pages_kernel(vec16* __restrict__ dst, size_t chunks, uint32_t value) {
  const size_t k = (size_t)blockIdx.x * 256 + threadIdx.x;
  const vec16 v = {value, value, value, value};
  if (k < chunks) dst[k] = v;
}

// The stores of the fused Pong rollout and nothing else: per step every lane writes the 32-byte
// observation of its environment (two 16-byte stores), a reward dword and a done byte into
// obs[T][n][8], reward[T][n], done[T][n], with the rollout's workgroup-to-XCD mapping.  SLEEP > 0
// puts the wavefront to sleep for SLEEP x 64 cycles after every step: issued as fast as they can be,
// the stores of different wavefronts drift over many rows of the trajectory and the memory system
// thrashes (5.6 TB/s at N = 65536); paced to the rate it drains at, all wavefronts stay on the same
// row and it takes 6.7 TB/s.
template <int SLEEP>
__global__ __launch_bounds__(256) void trajectory_stores_kernel(float* __restrict__ obs, float* __restrict__ reward,
                                                                uint8_t* __restrict__ done, int64_t n, int T) {
  const unsigned per_xcd = gridDim.x >> 3;
  const unsigned logical_block = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
  const int64_t i = (int64_t)logical_block * 256 + threadIdx.x;
  if (i >= n) return;
  const float4 v = make_float4(1.0f, 2.0f, 3.0f, (float)threadIdx.x);
  for (int t = 0; t < T; ++t) {
    const int64_t k = (int64_t)t * n + i;
    float4* o = reinterpret_cast<float4*>(obs + k * 8);
    o[0] = v;
    o[1] = v;
    reward[k] = 1.0f;
    done[k] = 0;
    if (SLEEP > 0) __builtin_amdgcn_s_sleep(SLEEP);
  }
}

__global__ void empty_kernel() {}

// What a launch costs with and without a kernel-argument segment: the same 4-byte-per-thread store,
// once with its descriptor as kernel arguments, once read from a record in device memory by a
// kernel that takes no argument and asks for neither gridDim nor blockDim.
struct StoreRecord { uint32_t* dst; uint32_t words; uint32_t value; };
__device__ StoreRecord g_store_record;

__global__ __launch_bounds__(256) void store_with_arguments_kernel(uint32_t* dst, uint32_t words, uint32_t value) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < words) dst[i] = value;
}

__global__ __launch_bounds__(256) void store_from_record_kernel() {
  const StoreRecord r = g_store_record;
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < r.words) r.dst[i] = r.value;
}

__global__ void store_record_write_kernel(StoreRecord r) { g_store_record = r; }

double seconds_now() {
  return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

unsigned grid_for(size_t chunks) {
  const size_t want = (chunks + 255) / 256;
  const size_t cap = 256 * 32;   // 32 workgroups per CU
  return (unsigned)(want < cap ? (want ? want : 1) : cap);
}

}  // namespace

extern "C" {

// dst_dev: device memory, 16-byte aligned, bytes a multiple of 16.  Returns 0 or -3.
int mi355env_bench_fill(void* dst_dev, size_t bytes, uint32_t value, void* hip_stream) {
  if (!dst_dev || (bytes & 15) || (reinterpret_cast<uintptr_t>(dst_dev) & 15)) return -1;
  const size_t chunks = bytes / 16;
  hipLaunchKernelGGL(fill16_kernel, dim3(grid_for(chunks)), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<vec16*>(dst_dev), chunks, value);
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

// Same contract; bytes must also be below 2^32 * 4096.
int mi355env_bench_fill_pages(void* dst_dev, size_t bytes, uint32_t value, void* hip_stream) {
  if (!dst_dev || (bytes & 15) || (reinterpret_cast<uintptr_t>(dst_dev) & 15)) return -1;
  const size_t chunks = bytes / 16, blocks = (chunks + 255) / 256;
  if (blocks == 0 || blocks > 0x7fffffffull) return -1;
  hipLaunchKernelGGL(fill_pages_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<vec16*>(dst_dev), chunks, value);
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

// obs_dev float32[T][n][8] (16-byte aligned), reward_dev float32[T][n], done_dev uint8[T][n];
// sleep: 0 (none), or 8..15 units of 64 cycles per step.
int mi355env_bench_trajectory_stores_paced(void* obs_dev, void* reward_dev, void* done_dev, int64_t n, int32_t T,
                                           int32_t sleep, void* hip_stream) {
  if (!obs_dev || !reward_dev || !done_dev || n <= 0 || T <= 0 || n > (int64_t(1) << 30) ||
      (reinterpret_cast<uintptr_t>(obs_dev) & 15) || (reinterpret_cast<uintptr_t>(reward_dev) & 3))
    return -1;
  unsigned blocks = (unsigned)((n + 255) / 256);
  blocks = (blocks + 7u) & ~7u;
  const dim3 g(blocks), b(256);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* o = static_cast<float*>(obs_dev);
  float* r = static_cast<float*>(reward_dev);
  uint8_t* d = static_cast<uint8_t*>(done_dev);
  switch (sleep) {
    case 0: hipLaunchKernelGGL(trajectory_stores_kernel<0>, g, b, 0, st, o, r, d, n, T); break;
    case 8: hipLaunchKernelGGL(trajectory_stores_kernel<8>, g, b, 0, st, o, r, d, n, T); break;
    case 9: hipLaunchKernelGGL(trajectory_stores_kernel<9>, g, b, 0, st, o, r, d, n, T); break;
    case 10: hipLaunchKernelGGL(trajectory_stores_kernel<10>, g, b, 0, st, o, r, d, n, T); break;
    case 11: hipLaunchKernelGGL(trajectory_stores_kernel<11>, g, b, 0, st, o, r, d, n, T); break;
    case 12: hipLaunchKernelGGL(trajectory_stores_kernel<12>, g, b, 0, st, o, r, d, n, T); break;
    case 13: hipLaunchKernelGGL(trajectory_stores_kernel<13>, g, b, 0, st, o, r, d, n, T); break;
    case 14: hipLaunchKernelGGL(trajectory_stores_kernel<14>, g, b, 0, st, o, r, d, n, T); break;
    case 15: hipLaunchKernelGGL(trajectory_stores_kernel<15>, g, b, 0, st, o, r, d, n, T); break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

int mi355env_bench_trajectory_stores(void* obs_dev, void* reward_dev, void* done_dev, int64_t n, int32_t T,
                                     void* hip_stream) {
  return mi355env_bench_trajectory_stores_paced(obs_dev, reward_dev, done_dev, n, T, 0, hip_stream);
}

// One workgroup that does nothing: the floor of what a launch costs on this stream.
int mi355env_bench_empty(void* hip_stream) {
  hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream));
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

// A loop of `launches` launches on hip_stream, enqueued from C++ with nothing in between.
// kind 0: an empty kernel; 1: 256-thread workgroups store bytes / 4 words, descriptor passed as
// kernel arguments; 2: the same store, descriptor read from device memory, no kernel-argument
// segment.  dst_dev: device memory of `bytes` bytes (a multiple of 1024, at most 1 MiB; unused for
// kind 0).  *host_us_out: host time per launch until the last one is enqueued; *total_us_out: per
// launch until the stream has drained.  Synchronises the stream before and after.
int mi355env_bench_launch_loop(int kind, int launches, void* dst_dev, size_t bytes, void* hip_stream,
                               double* host_us_out, double* total_us_out) {
  if (kind < 0 || kind > 2 || launches <= 0 || launches > 10000000 || !host_us_out || !total_us_out) return -1;
  if (kind != 0 && (!dst_dev || bytes == 0 || (bytes & 1023) || bytes > (size_t(1) << 20) ||
                    (reinterpret_cast<uintptr_t>(dst_dev) & 3)))
    return -1;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  uint32_t* dst = static_cast<uint32_t*>(dst_dev);
  const uint32_t words = (uint32_t)(bytes / 4);
  const dim3 g(kind == 0 ? 1u : words / 256u), b(kind == 0 ? 64u : 256u);
  if (kind == 2) hipLaunchKernelGGL(store_record_write_kernel, dim3(1), dim3(1), 0, st, StoreRecord{dst, words, 1u});
  if (hipStreamSynchronize(st) != hipSuccess) return -3;
  const double t0 = seconds_now();
  for (int k = 0; k < launches; ++k) {
    if (kind == 0) hipLaunchKernelGGL(empty_kernel, g, b, 0, st);
    else if (kind == 1) hipLaunchKernelGGL(store_with_arguments_kernel, g, b, 0, st, dst, words, 1u);
    else hipLaunchKernelGGL(store_from_record_kernel, g, b, 0, st);
  }
  const double t1 = seconds_now();
  if (hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess) return -3;
  const double t2 = seconds_now();
  *host_us_out = (t1 - t0) / launches * 1e6;
  *total_us_out = (t2 - t0) / launches * 1e6;
  return 0;
}

int mi355env_bench_copy(void* dst_dev, const void* src_dev, size_t bytes, void* hip_stream) {
  if (!dst_dev || !src_dev || (bytes & 15) || (reinterpret_cast<uintptr_t>(dst_dev) & 15) ||
      (reinterpret_cast<uintptr_t>(src_dev) & 15))
    return -1;
  const size_t chunks = bytes / 16;
  hipLaunchKernelGGL(copy16_kernel, dim3(grid_for(chunks)), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), static_cast<vec16*>(dst_dev),
                     static_cast<const vec16*>(src_dev), chunks);
  return hipGetLastError() == hipSuccess ? 0 : -3;
}

}  // extern "C"
