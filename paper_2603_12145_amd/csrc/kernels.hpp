// Host-callable launchers of the HIP kernels (internal to the library; the public boundary is
// include/mi355env.h).  Every launcher validates nothing: the C-ABI layer has already checked
// sizes, alignment and pointer residency.  All return the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "stats.hpp"
#include "step_counter.hpp"

namespace envk {

constexpr int FRAME_SIDE = 84;
constexpr int FRAME_BYTES = FRAME_SIDE * FRAME_SIDE;  // 7056 = 441 * 16

struct PongLaunch {
  uint32_t* state;        // SoA [10][n]
  int64_t n;
  uint64_t seed;
  uint64_t step0;         // index of the first step of this launch (used when counter == nullptr)
  StepCounter* counter;   // device-resident step counter, or nullptr
  int32_t ticket;         // set by the launcher: the launch advances `counter` itself (small grids)
  int32_t T;
  int32_t max_score;
  const uint8_t* actions; // [T,n] or nullptr
  float* obs;             // [T,n,8]
  float* reward;          // [T,n]
  uint8_t* done;          // [T,n]
  DeviceStats* stats;
  int32_t paged;          // set by the launcher: observation stores go through LDS, one 4 KiB page at a time
  int32_t xcd_remap;      // set by the launcher (Pong rollout): each XCD owns a contiguous eighth of the batch
  int32_t pace;           // set by the launcher (paced loop): least time between two chunks, in 1/256 of 10 ns
  int32_t normalize;      // Pong vector obs only: 1 = scale every component at the source
  float inv_score;        // 1 / max_score in float32 (used when normalize)
  // Scratch of the handle for the launcher's one-time choice between the paced and the plain loop
  // (null: no measurement, the launcher's table decides): a second state array [10][n] and a second
  // statistics block, so that the timed launches touch nothing the caller can see but the output
  // buffers, which the real launch then overwrites.
  uint32_t* trial_state;
  DeviceStats* trial_stats;
};

// Batch sizes for which the Pong rollout may run paced (see launch_pong_rollout)
constexpr int64_t PACED_MIN_ENVS = 61440, PACED_MAX_ENVS = 262144;

// reset launchers: counter != nullptr -> the step is read from it instead of `step`
hipError_t launch_pong_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                             const StepCounter* counter, float* obs, bool normalize, hipStream_t stream);
// Per-step launches without kernel arguments (Pong with vector observations, CartPole).
// On this runtime a loop of small launches is bound by the host's launch path whenever the kernel
// has a kernel-argument segment (2.4 us per launch, whatever the kernel does) and by the device
// (1.5-2.1 us) when it has none.  A caller that steps in a loop passes the same buffers every time,
// so all that changes between two launches is the step index: the launch descriptor is kept in
// device memory (one record per handle, STEP_RECORD_SLOTS handles per device; further handles
// launch with arguments), the step index with it, one copy per wavefront of the launch -- a
// wavefront reads its copy at the start and writes copy + 1 at the end, so nothing is atomic and
// no wavefront waits for another -- and the step kernel takes no argument and asks for neither
// gridDim nor blockDim.  The host rewrites the record (a one-workgroup launch that carries it as
// its argument) only when a call differs from it: other buffers, another stream, a step index
// that did not come from the last resident launch (reset, rollout or set_state in between).
constexpr int STEP_RECORD_SLOTS = 4;
constexpr unsigned STEP_RECORD_MAX_GROUPS = 64;    // workgroups of 256: 16384 environments; larger batches are not launch-bound

// What a handle remembers of its per-step launches (host side): the launch record it owns in
// device memory, what that record holds, and what the last call asked for.
struct StepResident {
  int device = -1, slot = -1;    // slot < 0: no record owned (not asked for yet, or none was free)
  bool asked = false;
  bool on_device = false;        // the record in device memory equals `rec` and counts `next_step`
  bool have_last = false;
  PongLaunch rec{}, last{};
  hipStream_t rec_stream = nullptr, last_stream = nullptr;
  uint64_t next_step = 0;
};
int step_slot_acquire(int device);          // -1: all records of the device are taken
void step_resident_release(StepResident& r);
void count_resident_step_launch();
int step_kernel_mode();                     // mi355env_tune_step_kernel's value

// What a resident launch depends on: everything a step reads from its descriptor.
inline bool same_step_request(const PongLaunch& x, const PongLaunch& y) {
  return x.state == y.state && x.n == y.n && x.seed == y.seed && x.max_score == y.max_score &&
         x.actions == y.actions && x.obs == y.obs && x.reward == y.reward && x.done == y.done &&
         x.stats == y.stats && x.normalize == y.normalize && x.inv_score == y.inv_score;
}

// The host side of a T = 1 launch that may go without arguments: for a handle with the host step
// counter (so the call is never part of a stream capture), at most STEP_RECORD_MAX_GROUPS
// workgroups, and a call that asks for what the call before it asked for.  A caller that
// alternates between buffers never takes the path and never pays for a rewrite of the record; a
// steady loop takes it from its second call on.  write(slot, a, step) launches the kernel that
// rewrites record `slot`, launch(slot, groups) the step kernel that reads it.  Returns false if
// the call is to be launched with arguments instead.
template <class Write, class Launch>
bool resident_step_try(StepResident* resident, const PongLaunch& a, unsigned groups, hipStream_t stream,
                       Write write, Launch launch, hipError_t* err) {
  if (!resident || a.counter || step_kernel_mode() != 1 || groups > STEP_RECORD_MAX_GROUPS) return false;
  StepResident& r = *resident;
  const bool repeat = r.have_last && r.last_stream == stream && same_step_request(r.last, a);
  r.last = a;
  r.last_stream = stream;
  r.have_last = true;
  if (repeat && !r.asked) {
    r.asked = true;
    if (hipGetDevice(&r.device) == hipSuccess) r.slot = step_slot_acquire(r.device);
    else (void)hipGetLastError();
  }
  if (!repeat || r.slot < 0) return false;
  if (!(r.on_device && r.rec_stream == stream && r.next_step == a.step0 && same_step_request(r.rec, a))) {
    write(r.slot, a, (unsigned long long)a.step0);
    *err = hipGetLastError();
    if (*err != hipSuccess) return true;
    r.rec = a;
    r.rec_stream = stream;
    r.on_device = true;
  }
  launch(r.slot, groups);
  *err = hipGetLastError();
  if (*err != hipSuccess) r.on_device = false;
  r.next_step = a.step0 + 1;
  count_resident_step_launch();
  return true;
}

// resident: the calling handle's StepResident, or null
hipError_t launch_pong_rollout(const PongLaunch& a, hipStream_t stream, StepResident* resident = nullptr);

// CartPole: same launch descriptor (max_score carries max_episode_steps; obs is [T,n,4]).
constexpr int CARTPOLE_FIELDS = 6;   // x xdot theta thetadot | ep_ret ep_len
constexpr int CARTPOLE_OBS = 4;
hipError_t launch_cartpole_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                                 const StepCounter* counter, float* obs, hipStream_t stream);
hipError_t launch_cartpole_rollout(const PongLaunch& a, hipStream_t stream, StepResident* resident = nullptr);

// Pixel observations.  ring != nullptr: frame after step s goes to ring[i][s & 3] (T must be 1 or
// the ring is rewritten in place T times); frames != nullptr: frame t of the launch goes to
// frames[t][i].
struct PixelLaunch {
  PongLaunch pong;        // obs unused
  uint8_t* ring;          // 4-slot ring or nullptr
  uint8_t* frames;        // [T,n,84,84] or nullptr
  bool slot_major;        // ring layout: [4,n,84,84] (true) or [n,4,84,84] (false)
  uint32_t* blocks;       // library scratch [3][n]: packed cell blocks of the newest frame
};
hipError_t launch_pixel_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                              const StepCounter* counter, uint8_t* ring, bool slot_major, uint32_t* blocks,
                              hipStream_t stream);
struct PixelPipe;
// pipe: the handle's scratch; its trajectory staging area lets a frame trajectory be rendered
// a chunk of steps at a time (see launch_pixel_rollout in pixel_kernels.hip).
hipError_t launch_pixel_rollout(const PixelLaunch& a, PixelPipe& pipe, hipStream_t stream);

// Slot-major pixel step with one-step lookahead.  Every step is the launch F(t) = { hand step t's
// staged reward / done to the caller and flush its episode statistics; render step t's plane;
// compute step t+1 (in-kernel actions) from the state after t into the staging buffers of the other
// parity }.  The three parts are independent, so the dynamics of the next step hide under the
// render of this one inside a single launch.  If the staged step is not the one asked for (first
// step, external actions, state restored), the dynamics launch D(t) runs first.
struct PixelPipe {
  void* slab = nullptr;                            // one allocation holding everything below
  uint32_t* state_alt = nullptr;                   // second state buffer [10][n] (ping-pong)
  uint32_t* blocks[2] = {nullptr, nullptr};        // [3][n] cell blocks of the staged frame
  float* reward[2] = {nullptr, nullptr};           // [n]
  uint8_t* done[2] = {nullptr, nullptr};           // [n]
  int32_t* fin_ret[2] = {nullptr, nullptr};        // [n] return / length of an episode that ended
  int32_t* fin_len[2] = {nullptr, nullptr};
  bool staged = false;                             // staging buffers of parity (step & 1) hold `step`
  uint32_t* traj_blocks = nullptr;                 // [3][traj_cap] cell blocks of a chunk of a frame trajectory
  int64_t traj_cap = 0;                            // frames (environment-steps) per chunk
  // Delta updates of the observation buffer (only for handles created with pixel_update = delta or
  // the ordered layout)
  uint32_t* hist = nullptr;                        // [5][3][n] cell blocks of the last five frames, entry = step mod 5
  void* book = nullptr;                            // record of what the observation buffer holds, in device memory
  unsigned long long host_book[4] = {~0ull, 0, 0, 0};   // ... and the host's copy (handles with the host step counter)
  // Lookahead of a handle whose step counter lives in device memory (see pixel_counted_step)
  uint32_t* stage_state[2] = {nullptr, nullptr};   // [10][n] state after the staged step, per parity of its index
  unsigned long long* staged_for = nullptr;        // device word: index of the step the staging buffers hold, ~0 = none
};
hipError_t pixel_pipe_create(PixelPipe& p, int64_t n, bool delta_updates, bool device_counter);
void pixel_pipe_destroy(PixelPipe& p);
// One slot-major ring step.  `state` is the handle's committed-state pointer and is swapped with
// p.state_alt.  a.pong.actions may be null (staged lookahead usable) or external.
hipError_t pixel_pipe_step(PixelPipe& p, uint32_t*& state, const PixelLaunch& a, bool lookahead,
                           hipStream_t stream);
inline void pixel_pipe_invalidate(PixelPipe& p) { p.staged = false; }
// The same step for a handle whose step counter lives in device memory (a.pong.counter): nothing is
// alternated from the host, so that the call can be recorded in a graph and replayed.  In-kernel
// actions: a one-workgroup launch that reads and advances the counter (and, only if the staging
// buffers do not hold this step, computes it), then the fused launch with the lookahead.  External
// actions: dynamics launch, then the page renderer.
hipError_t pixel_counted_step(const PixelPipe& p, const PixelLaunch& a, hipStream_t stream);
// The state changed without the step counter moving (env_reset, env_set_state): whatever is staged
// ahead is void.
hipError_t pixel_counted_forget(const PixelPipe& p, hipStream_t stream);
// One step of a handle that keeps its observation buffer current by delta updates: a ring slot
// (ordered = false; a.slot_major says which ring) or all four channels of the ordered stack.  One
// launch; it decides by itself, from a record in device memory, whether the buffer can be repaired
// or has to be written whole, so it may be recorded in a HIP graph (a.pong.counter set) as well.
hipError_t pixel_update_step(PixelPipe& p, const PixelLaunch& a, bool ordered, hipStream_t stream);
// After env_reset has written the initial frame to all four slots / channels of `ring`.
hipError_t pixel_update_after_reset(PixelPipe& p, const uint32_t* state, int64_t n, uint64_t step,
                                    const StepCounter* counter, const uint8_t* ring, hipStream_t stream);
// The buffer no longer matches what the library keeps: the next four steps write whole frames.
hipError_t pixel_update_forget(PixelPipe& p, hipStream_t stream);
// Steps that repaired / wrote whole frames since creation (synchronises the stream).
hipError_t pixel_update_counts(PixelPipe& p, bool device_counter, int64_t* delta_steps, int64_t* full_steps,
                               hipStream_t stream);
int pixel_plane_mode();

}  // namespace envk
