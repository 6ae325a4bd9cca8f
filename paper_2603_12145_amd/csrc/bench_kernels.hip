// Yardstick kernels for measurements (not part of the environment path): a plain fill and a plain
// copy with 16-byte accesses.  They calibrate the HBM counters (known bytes per launch) and give
// the write / copy bandwidth a trivial kernel reaches on the same device.
#include <hip/hip_runtime.h>
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

__global__ void empty_kernel() {}

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

// One workgroup that does nothing: the floor of what a launch costs on this stream.
int mi355env_bench_empty(void* hip_stream) {
  hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream));
  return hipGetLastError() == hipSuccess ? 0 : -3;
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
