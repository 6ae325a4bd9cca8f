// Step counter kept in device memory, for launches that are recorded once in a HIP graph and
// replayed: a kernel argument is frozen at capture time, so the index of the launch's first step
// (which keys every Philox draw) is read from memory instead, and the launch advances it itself.
//
// Small grids advance it themselves: thread 0 of every workgroup reads the counter, then (once the
// value has arrived) takes a ticket; the workgroup that takes the last ticket knows every other
// workgroup has already read, so it alone writes counter + T and clears the tickets.  The
// tickets are one atomic on one address, about 45 ns each back to back, so above
// TICKET_MAX_BLOCKS workgroups (a per-step launch of 262144 Pong environments has 1024: 37 us of
// tickets around 6 us of work) the launch only reads and a one-thread launch behind it does the
// adding.  Either way the next launch on the stream starts after the counter has moved.  Two
// launches that use one counter must not overlap.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace envk {

struct StepCounter {
  unsigned long long step;
  unsigned int ticket;
  unsigned int pad;
};

constexpr unsigned TICKET_MAX_BLOCKS = 64;

// Must be called by every thread of every workgroup of a one-dimensional launch, before any early
// exit.  counter == nullptr: the host passed the step as a kernel argument; nothing is touched.
// ticket: this launch advances the counter itself (else advance_step_counter_behind follows it).
// The result is wave-uniform (kept in scalar registers).
__device__ __forceinline__ uint64_t launch_first_step(StepCounter* counter, uint64_t host_step0, int32_t T,
                                                      bool ticket) {
  if (!counter) return host_step0;
  if (!ticket) {
    const unsigned long long s = __hip_atomic_load(&counter->step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)s);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(s >> 32));
    return ((uint64_t)hi << 32) | lo;
  }
  __shared__ unsigned long long shared_step;
  if (threadIdx.x == 0) {
    // The ticket has to be taken after the counter's value has arrived, and that is all it has to
    // wait for: relaxed atomics with a workgroup-scope fence between them (which waits for the
    // load and touches no cache), not acquire / release at device scope, each of which writes
    // back and invalidates an L2 slice on this multi-die part.  The last ticket is known only
    // once its atomic has returned, so the write of counter + T comes after every other
    // workgroup's read; the next launch on the stream reads it behind the kernel boundary.
    const unsigned long long s = __hip_atomic_load(&counter->step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    shared_step = s;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    const unsigned int t =
        __hip_atomic_fetch_add(&counter->ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == gridDim.x - 1u) {
      __hip_atomic_store(&counter->ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&counter->step, s + (unsigned long long)T, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();
  const unsigned long long s = shared_step;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)s);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(s >> 32));
  return ((uint64_t)hi << 32) | lo;
}

// The same small-grid protocol with the ticket at the end of the launch instead of in front of its
// work, for kernels in which every thread reaches the end: first_step_of_launch at the start (a
// plain load that runs beside the launch's other loads), finish_launch_steps after the last store.
// By the barrier every wavefront of the workgroup has used its copy of the counter (the loads have
// returned), so the ticket can be a relaxed atomic: what it orders is only "this workgroup has
// read", and the count itself tells the last workgroup that all have.  (Release / acquire at
// device scope would make every workgroup write back and invalidate its L2 slice, which costs
// more than the step.)  The workgroup that takes the last ticket writes first + T; the next
// launch on the stream reads it behind the kernel boundary.
__device__ __forceinline__ uint64_t first_step_of_launch(const StepCounter* counter, uint64_t host_step0) {
  if (!counter) return host_step0;
  const unsigned long long s = __hip_atomic_load(&counter->step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)s);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(s >> 32));
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ void finish_launch_steps(StepCounter* counter, uint64_t first, int32_t T,
                                                    unsigned blocks) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int t =
        __hip_atomic_fetch_add(&counter->ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (t == blocks - 1u) {
      __hip_atomic_store(&counter->ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&counter->step, (unsigned long long)first + (unsigned long long)T, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// For kernels that read their launch descriptor from device memory: a pointer read from memory is
// a generic one to the compiler (flat loads and stores), while kernel arguments are known to point
// to global memory.  Says the same of such a pointer.  By way of the integer: a generic -> global ->
// generic cast pair is folded away.
template <class T>
__device__ __forceinline__ T* known_global(T* p) {
  return (T*)(__attribute__((address_space(1))) T*)(uintptr_t)p;
}

// For kernels that only read the counter (reset): no ticket, no write.
__device__ __forceinline__ uint64_t read_step(const StepCounter* counter, uint64_t host_step) {
  return counter ? __hip_atomic_load(&counter->step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : host_step;
}

namespace {
__global__ void step_counter_advance_kernel(StepCounter* counter, int32_t T) {
  counter->step = counter->step + (unsigned long long)T;
}
}  // namespace

// Host side of the second protocol: right behind a launch of `blocks` workgroups that only read.
inline hipError_t advance_step_counter_behind(StepCounter* counter, int32_t T, unsigned blocks, hipStream_t stream) {
  if (!counter || blocks <= TICKET_MAX_BLOCKS) return hipSuccess;
  hipLaunchKernelGGL(step_counter_advance_kernel, dim3(1), dim3(1), 0, stream, counter, T);
  return hipGetLastError();
}

}  // namespace envk
