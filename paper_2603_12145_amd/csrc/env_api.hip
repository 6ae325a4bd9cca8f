// C-ABI layer of libmi355env.so: argument checks, handle bookkeeping and kernel launches.
// The contract of every entry point is stated in include/mi355env.h.
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <new>
#include <vector>

#include "../../include/mi355env.h"
#include "kernels.hpp"
#include "pong_device.hpp"
#include "body_kernels.hpp"

using namespace envk;

namespace envk {
bool set_pixel_tuning(int envs_per_wave, int streaming);
bool set_rollout_block(int threads, int xcd_remap);
bool set_rollout_chunk(int steps);
bool set_rollout_pace(int gb_per_s);
bool set_measure_pace(int on);
bool set_step_kernel(int on);
unsigned long long resident_step_launches();
bool set_cartpole_split(int mode);
int pong_pace_choice(int64_t n);
bool set_rollout_split(int mode);
bool set_paged_stores(int mode);
bool set_traj_mode(int mode);
bool set_plane_path(int on);
}

struct mi355env {
  int kind;
  int device;
  int64_t n;
  uint64_t seed;
  uint64_t step;          // env steps taken since creation (all environments move in lock-step)
  hipStream_t stream;
  env_config_t cfg;
  uint32_t* state;        // device SoA [fields][n], every field 4 bytes (pixels: may point into pipe)
  uint32_t* state_alloc;  // the allocation made for it by env_create
  int fields;
  DeviceStats* stats;     // device, STATS_STRIPES copies
  StepCounter* counter;   // device, behind stats in the same allocation
  bool device_counter;    // launches read and advance `counter` instead of taking `step` as an argument
  PixelPipe pipe;         // pixels only: second state buffer and the staging buffers of the lookahead
  uint32_t* trial_state;  // Pong, batch sizes that may run paced: scratch for the launcher's one-time
  DeviceStats* trial_stats;   // measurement (a second state array and statistics block), else null
  StepResident resident;  // Pong, CartPole: what the per-step launches keep in device memory between calls
  bool was_reset;
  // last device ranges that passed the residency check (avoids a driver query per step)
  struct Range { const void* p; size_t bytes; } seen[8];
  int seen_next;
};

namespace {

constexpr int64_t MAX_ENVS = int64_t(1) << 30;

int fields_of(int kind) {
  return kind == ENV_BODY ? BODY_FIELDS : kind == ENV_CARTPOLE ? CARTPOLE_FIELDS : PONG_FIELDS;
}

env_config_t default_config(int kind) {
  env_config_t c;
  std::memset(&c, 0, sizeof c);
  c.struct_size = sizeof(env_config_t);
  c.max_score = 21;
  c.max_episode_steps = kind == ENV_CARTPOLE ? 500 : 1000;
  c.armature = BODY_DEFAULT_ARMATURE;
  c.joint_damping = BODY_DEFAULT_JOINT_DAMPING;
  c.friction_mu = BODY_DEFAULT_FRICTION_MU;
  c.pixel_layout = ENV_PIXELS_SLOT_MAJOR;
  c.step_counter = ENV_STEP_COUNTER_HOST;
  c.obs_scaling = ENV_OBS_RAW;
  c.contact_solver = ENV_CONTACT_PENALTY;
  c.pixel_update = ENV_PIXELS_FULL;
  c.body_arithmetic = ENV_BODY_F64;
  (void)kind;
  return c;
}

#define FIELD_END(type, member) (offsetof(type, member) + sizeof(((type*)0)->member))

int merge_config(env_config_t* dst, const env_config_t* src) {
  if (!src) return ENV_OK;
  const uint32_t sz = src->struct_size;
  if (sz < sizeof(uint32_t) || sz > 4096) return ENV_E_ARG;
  if (sz >= FIELD_END(env_config_t, max_score) && src->max_score > 0) dst->max_score = src->max_score;
  if (sz >= FIELD_END(env_config_t, max_episode_steps) && src->max_episode_steps > 0)
    dst->max_episode_steps = src->max_episode_steps;
  if (sz >= FIELD_END(env_config_t, armature) && src->armature >= 0.0f) dst->armature = src->armature;
  if (sz >= FIELD_END(env_config_t, joint_damping) && src->joint_damping >= 0.0f)
    dst->joint_damping = src->joint_damping;
  if (sz >= FIELD_END(env_config_t, friction_mu) && src->friction_mu >= 0.0f)
    dst->friction_mu = src->friction_mu;
  if (sz >= FIELD_END(env_config_t, pixel_layout) && src->pixel_layout != 0) {
    if (src->pixel_layout != ENV_PIXELS_SLOT_MAJOR && src->pixel_layout != ENV_PIXELS_ENV_MAJOR &&
        src->pixel_layout != ENV_PIXELS_ORDERED)
      return ENV_E_ARG;
    dst->pixel_layout = src->pixel_layout;
  }
  if (sz >= FIELD_END(env_config_t, step_counter) && src->step_counter != 0) {
    if (src->step_counter != ENV_STEP_COUNTER_HOST && src->step_counter != ENV_STEP_COUNTER_DEVICE)
      return ENV_E_ARG;
    dst->step_counter = src->step_counter;
  }
  if (sz >= FIELD_END(env_config_t, obs_scaling) && src->obs_scaling != 0) {
    if (src->obs_scaling != ENV_OBS_RAW && src->obs_scaling != ENV_OBS_NORMALIZED) return ENV_E_ARG;
    dst->obs_scaling = src->obs_scaling;
  }
  if (sz >= FIELD_END(env_config_t, contact_solver) && src->contact_solver != 0) {
    if (src->contact_solver != ENV_CONTACT_PENALTY && src->contact_solver != ENV_CONTACT_NEWTON)
      return ENV_E_ARG;
    dst->contact_solver = src->contact_solver;
  }
  if (sz >= FIELD_END(env_config_t, pixel_update) && src->pixel_update != 0) {
    if (src->pixel_update != ENV_PIXELS_FULL && src->pixel_update != ENV_PIXELS_DELTA) return ENV_E_ARG;
    dst->pixel_update = src->pixel_update;
  }
  if (sz >= FIELD_END(env_config_t, body_arithmetic) && src->body_arithmetic != 0) {
    if (src->body_arithmetic != ENV_BODY_F64 && src->body_arithmetic != ENV_BODY_F32) return ENV_E_ARG;
    dst->body_arithmetic = src->body_arithmetic;
  }
  if (!std::isfinite(dst->armature) || !std::isfinite(dst->joint_damping) ||
      !std::isfinite(dst->friction_mu))
    return ENV_E_ARG;
  return ENV_OK;
}

DeviceStats empty_stats() {
  DeviceStats s;
  std::memset(&s, 0, sizeof s);
  s.return_min_key = std::numeric_limits<int>::max();
  s.return_max_key = std::numeric_limits<int>::min();
  return s;
}

// All copies of the statistics block, empty (host side; 32 KiB).
struct EmptyStats {
  DeviceStats stripes[STATS_STRIPES];
  EmptyStats() { for (auto& s : stripes) s = empty_stats(); }
};

float key_to_float(int key) {
  const int b = key ^ ((key >> 31) & 0x7fffffff);
  float f;
  std::memcpy(&f, &b, sizeof f);
  return f;
}

// True iff [p, p+bytes) lies inside one device allocation visible to this process.
bool device_range_ok(env_t* e, const void* p, size_t bytes, size_t align) {
  if (!p || (reinterpret_cast<uintptr_t>(p) & (align - 1))) return false;
  for (auto& r : e->seen)
    if (r.p == p && r.bytes >= bytes) return true;
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, p) != hipSuccess) { (void)hipGetLastError(); return false; }
  if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) return false;
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange(&base, &size, const_cast<void*>(p)) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  const uintptr_t lo = reinterpret_cast<uintptr_t>(base), q = reinterpret_cast<uintptr_t>(p);
  if (q < lo || q + bytes > lo + size) return false;
  e->seen[e->seen_next] = {p, bytes};
  e->seen_next = (e->seen_next + 1) % 8;
  return true;
}

// Launches and copies go to the current device: refuse a call made with another device current than
// the one the handle's memory lives on.
bool on_own_device(const env_t* e) {
  int d = -1;
  if (hipGetDevice(&d) != hipSuccess) { (void)hipGetLastError(); return false; }
  return d == e->device;
}

int read_device_step(const env_t* e, uint64_t* out) {
  unsigned long long s = 0;
  if (hipMemcpyAsync(&s, &e->counter->step, sizeof s, hipMemcpyDeviceToHost, e->stream) != hipSuccess ||
      hipStreamSynchronize(e->stream) != hipSuccess)
    return ENV_E_HIP;
  *out = s;
  return ENV_OK;
}

size_t obs_bytes_per_env_step(int kind) {
  switch (kind) {
    case ENV_PONG: return PONG_OBS * sizeof(float);
    case ENV_PONG_PIXELS: return (size_t)FRAME_BYTES;
    case ENV_BODY: return BODY_OBS * sizeof(float);
    case ENV_CARTPOLE: return CARTPOLE_OBS * sizeof(float);
  }
  return 0;
}

size_t action_bytes_per_env_step(int kind) {
  return kind == ENV_BODY ? BODY_ACT * sizeof(float) : sizeof(uint8_t);
}

int run(env_t* e, int32_t T, bool ring_mode, const void* actions, void* obs, float* reward,
        uint8_t* done) {
  if (!e) return ENV_E_ARG;
  if (T <= 0) return ENV_E_ARG;
  if (!e->was_reset) return ENV_E_STATE;
  if (!on_own_device(e)) return ENV_E_STATE;
  // T * n * (bytes per env-step, at most 7056) must fit a size_t with room to spare
  if ((uint64_t)T > (uint64_t(1) << 48) / (uint64_t)e->n) return ENV_E_ARG;
  if (!e->device_counter) {
    // A launch recorded by stream capture would replay with the step index frozen at capture time
    // (same random draws every replay): refuse instead of producing silently wrong trajectories.
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(e->stream, &cs) != hipSuccess) (void)hipGetLastError();
    else if (cs != hipStreamCaptureStatusNone) return ENV_E_STATE;
  }
  const size_t tn = (size_t)T * (size_t)e->n;
  const size_t obs_bytes = (e->kind == ENV_PONG_PIXELS && ring_mode)
                               ? (size_t)e->n * 4 * FRAME_BYTES
                               : tn * obs_bytes_per_env_step(e->kind);
  if (!device_range_ok(e, obs, obs_bytes, e->kind == ENV_BODY ? 4 : 16)) return ENV_E_ARG;
  if (!device_range_ok(e, reward, tn * sizeof(float), 4)) return ENV_E_ARG;
  if (!device_range_ok(e, done, tn, 1)) return ENV_E_ARG;
  if (actions &&
      !device_range_ok(e, actions, tn * action_bytes_per_env_step(e->kind), e->kind == ENV_BODY ? 4 : 1))
    return ENV_E_ARG;

  hipError_t err = hipSuccess;
  if (e->kind == ENV_BODY) {
    BodyLaunch b{};
    b.state = e->state; b.n = e->n; b.seed = e->seed; b.step0 = e->step; b.T = T;
    b.counter = e->device_counter ? e->counter : nullptr;
    b.max_episode_steps = e->cfg.max_episode_steps;
    b.armature = e->cfg.armature; b.joint_damping = e->cfg.joint_damping;
    b.friction_mu = e->cfg.friction_mu;
    b.newton = e->cfg.contact_solver == ENV_CONTACT_NEWTON;
    b.f32 = e->cfg.body_arithmetic == ENV_BODY_F32;
    b.actions = static_cast<const float*>(actions);
    b.obs = static_cast<float*>(obs); b.reward = reward; b.done = done; b.stats = e->stats;
    err = launch_body_rollout(b, e->stream);
  } else {
    PongLaunch p{};
    p.state = e->state; p.n = e->n; p.seed = e->seed; p.step0 = e->step; p.T = T;
    p.counter = e->device_counter ? e->counter : nullptr;
    p.normalize = e->cfg.obs_scaling == ENV_OBS_NORMALIZED;
    p.inv_score = 1.0f / (float)e->cfg.max_score;
    p.max_score = e->cfg.max_score;
    p.actions = static_cast<const uint8_t*>(actions);
    p.obs = static_cast<float*>(obs); p.reward = reward; p.done = done; p.stats = e->stats;
    if (e->kind == ENV_PONG) {
      p.trial_state = e->trial_state; p.trial_stats = e->trial_stats;
      err = launch_pong_rollout(p, e->stream, &e->resident);
    } else if (e->kind == ENV_CARTPOLE) {
      p.max_score = e->cfg.max_episode_steps;
      err = launch_cartpole_rollout(p, e->stream, &e->resident);
    } else {
      PixelLaunch x{};
      x.pong = p; x.pong.obs = nullptr;
      x.slot_major = e->cfg.pixel_layout == ENV_PIXELS_SLOT_MAJOR;
      x.blocks = e->pipe.blocks[0];
      if (ring_mode) x.ring = static_cast<uint8_t*>(obs);
      else x.frames = static_cast<uint8_t*>(obs);
      const bool plane_step = ring_mode && x.slot_major && T == 1 && pixel_plane_mode() != 0 &&
                              e->n < (int64_t)4000000;
      if (ring_mode && T == 1 && e->cfg.pixel_update == ENV_PIXELS_DELTA) {
        err = pixel_update_step(e->pipe, x, e->cfg.pixel_layout == ENV_PIXELS_ORDERED, e->stream);
      } else if (plane_step && e->device_counter) {
        // no lookahead and no buffers alternated from the host: a replayed graph could do neither
        pixel_pipe_invalidate(e->pipe);
        err = pixel_counted_step(e->pipe, x, e->stream);
      } else if (plane_step) {
        err = pixel_pipe_step(e->pipe, e->state, x, pixel_plane_mode() == 2, e->stream);
      } else {
        pixel_pipe_invalidate(e->pipe);      // the state moves without the lookahead knowing
        err = launch_pixel_rollout(x, e->pipe, e->stream);
        // ... and steps pass without their frames reaching a delta-updated observation buffer
        if (err == hipSuccess && e->cfg.pixel_update == ENV_PIXELS_DELTA) err = pixel_update_forget(e->pipe, e->stream);
      }
    }
  }
  if (err != hipSuccess) return ENV_E_HIP;
  e->step += (uint64_t)T;
  return ENV_OK;
}

}  // namespace

extern "C" {

int env_create(env_t** out, int kind, int64_t n_envs, uint64_t seed, const env_config_t* cfg,
               void* hip_stream) {
  if (!out) return ENV_E_ARG;
  if (kind != ENV_PONG && kind != ENV_PONG_PIXELS && kind != ENV_BODY && kind != ENV_CARTPOLE) return ENV_E_ARG;
  if (n_envs <= 0 || n_envs > MAX_ENVS) return ENV_E_ARG;
  env_config_t c = default_config(kind);
  if (merge_config(&c, cfg) != ENV_OK) return ENV_E_ARG;
  if (c.obs_scaling == ENV_OBS_NORMALIZED && kind != ENV_PONG) return ENV_E_UNSUPPORTED;
  if (c.contact_solver == ENV_CONTACT_NEWTON && kind != ENV_BODY) return ENV_E_UNSUPPORTED;
  if (c.body_arithmetic == ENV_BODY_F32 && kind != ENV_BODY) return ENV_E_UNSUPPORTED;
  if (kind == ENV_PONG_PIXELS && c.pixel_layout == ENV_PIXELS_ORDERED) c.pixel_update = ENV_PIXELS_DELTA;
  if (c.pixel_update == ENV_PIXELS_DELTA && kind != ENV_PONG_PIXELS) return ENV_E_UNSUPPORTED;

  env_t* e = new (std::nothrow) env_t();
  if (!e) return ENV_E_ALLOC;
  e->kind = kind; e->n = n_envs; e->seed = seed; e->step = 0;
  e->stream = static_cast<hipStream_t>(hip_stream);
  e->cfg = c; e->fields = fields_of(kind); e->was_reset = false;
  e->state = nullptr; e->stats = nullptr; e->counter = nullptr; e->seen_next = 0;
  e->trial_state = nullptr; e->trial_stats = nullptr;
  e->device_counter = c.step_counter == ENV_STEP_COUNTER_DEVICE;
  for (auto& r : e->seen) r = {nullptr, 0};
  if (hipGetDevice(&e->device) != hipSuccess) { delete e; return ENV_E_HIP; }

  const size_t state_bytes = (size_t)e->fields * (size_t)n_envs * 4;
  if (hipMalloc(reinterpret_cast<void**>(&e->state), state_bytes) != hipSuccess) {
    (void)hipGetLastError(); delete e; return ENV_E_ALLOC;
  }
  e->state_alloc = e->state;
  static_assert(sizeof(DeviceStats) == 128, "one cache line per copy of the statistics");
  if (hipMalloc(reinterpret_cast<void**>(&e->stats), STATS_STRIPES * sizeof(DeviceStats) + sizeof(StepCounter)) !=
      hipSuccess) {
    (void)hipGetLastError(); (void)hipFree(e->state); delete e; return ENV_E_ALLOC;
  }
  if (kind == ENV_PONG_PIXELS && pixel_pipe_create(e->pipe, n_envs, c.pixel_update == ENV_PIXELS_DELTA,
                                                     c.step_counter == ENV_STEP_COUNTER_DEVICE && c.pixel_layout == ENV_PIXELS_SLOT_MAJOR &&
                                                         c.pixel_update == ENV_PIXELS_FULL) != hipSuccess) {
    (void)hipGetLastError(); (void)hipFree(e->state); (void)hipFree(e->stats); delete e;
    return ENV_E_ALLOC;
  }
  e->counter = reinterpret_cast<StepCounter*>(e->stats + STATS_STRIPES);
  if (kind == ENV_PONG && n_envs >= PACED_MIN_ENVS && n_envs <= PACED_MAX_ENVS) {
    // one allocation: the trial statistics behind the trial state
    const size_t sb = (state_bytes + 255) & ~(size_t)255;
    if (hipMalloc(reinterpret_cast<void**>(&e->trial_state), sb + STATS_STRIPES * sizeof(DeviceStats)) != hipSuccess) {
      (void)hipGetLastError(); (void)hipFree(e->state); (void)hipFree(e->stats); delete e;
      return ENV_E_ALLOC;
    }
    e->trial_stats = reinterpret_cast<DeviceStats*>(reinterpret_cast<char*>(e->trial_state) + sb);
  }
  const EmptyStats z;
  if (hipMemsetAsync(e->state, 0, state_bytes, e->stream) != hipSuccess ||
      hipMemsetAsync(e->counter, 0, sizeof(StepCounter), e->stream) != hipSuccess ||
      hipMemcpyAsync(e->stats, z.stripes, sizeof z.stripes, hipMemcpyHostToDevice, e->stream) != hipSuccess ||
      hipStreamSynchronize(e->stream) != hipSuccess) {
    (void)hipGetLastError(); (void)hipFree(e->state); (void)hipFree(e->stats); (void)hipFree(e->trial_state);
    pixel_pipe_destroy(e->pipe); delete e;
    return ENV_E_HIP;
  }
  *out = e;
  return ENV_OK;
}

void env_destroy(env_t* e) {
  if (!e) return;
  (void)hipStreamSynchronize(e->stream);
  (void)hipFree(e->state_alloc);
  (void)hipFree(e->stats);
  (void)hipFree(e->trial_state);
  step_resident_release(e->resident);
  pixel_pipe_destroy(e->pipe);
  delete e;
}

int env_reset(env_t* e, void* obs_dev) {
  if (!e) return ENV_E_ARG;
  if (!on_own_device(e)) return ENV_E_STATE;
  hipError_t err;
  const StepCounter* counter = e->device_counter ? e->counter : nullptr;
  if (e->kind == ENV_PONG_PIXELS && obs_dev) {
    if (!device_range_ok(e, obs_dev, (size_t)e->n * 4 * FRAME_BYTES, 16)) return ENV_E_ARG;
    err = launch_pixel_reset(e->state, e->n, e->seed, e->step, counter, static_cast<uint8_t*>(obs_dev),
                             e->cfg.pixel_layout == ENV_PIXELS_SLOT_MAJOR, e->pipe.blocks[0], e->stream);
    pixel_pipe_invalidate(e->pipe);
    if (err == hipSuccess) err = pixel_counted_forget(e->pipe, e->stream);
    if (err == hipSuccess && e->cfg.pixel_update == ENV_PIXELS_DELTA)
      err = pixel_update_after_reset(e->pipe, e->state, e->n, e->step, counter,
                                     static_cast<const uint8_t*>(obs_dev), e->stream);
  } else if (e->kind == ENV_BODY) {
    if (obs_dev && !device_range_ok(e, obs_dev, (size_t)e->n * BODY_OBS * sizeof(float), 4))
      return ENV_E_ARG;
    err = launch_body_reset(e->state, e->n, e->seed, e->step, counter, static_cast<float*>(obs_dev), e->stream);
  } else if (e->kind == ENV_CARTPOLE) {
    if (obs_dev && !device_range_ok(e, obs_dev, (size_t)e->n * CARTPOLE_OBS * sizeof(float), 16))
      return ENV_E_ARG;
    err = launch_cartpole_reset(e->state, e->n, e->seed, e->step, counter, static_cast<float*>(obs_dev),
                                e->stream);
  } else {
    if (obs_dev && !device_range_ok(e, obs_dev, (size_t)e->n * PONG_OBS * sizeof(float), 16))
      return ENV_E_ARG;
    err = launch_pong_reset(e->state, e->n, e->seed, e->step, counter,
                            e->kind == ENV_PONG ? static_cast<float*>(obs_dev) : nullptr,
                            e->cfg.obs_scaling == ENV_OBS_NORMALIZED, e->stream);
    if (e->kind == ENV_PONG_PIXELS) {
      pixel_pipe_invalidate(e->pipe);
      if (err == hipSuccess) err = pixel_counted_forget(e->pipe, e->stream);
      // new episodes, no observation buffer written: what it holds is stale
      if (err == hipSuccess) err = pixel_update_forget(e->pipe, e->stream);
    }
  }
  if (err != hipSuccess) return ENV_E_HIP;
  e->was_reset = true;
  return ENV_OK;
}

int env_step(env_t* e, const void* actions_dev, void* obs_dev, float* reward_dev, uint8_t* done_dev) {
  return run(e, 1, true, actions_dev, obs_dev, reward_dev, done_dev);
}

int env_rollout(env_t* e, int32_t T, const void* actions_dev, void* obs_dev, float* reward_dev,
                uint8_t* done_dev) {
  return run(e, T, false, actions_dev, obs_dev, reward_dev, done_dev);
}

int env_stats(env_t* e, env_stats_t* host_out, int reset_counters) {
  if (!e || !host_out) return ENV_E_ARG;
  if (!on_own_device(e)) return ENV_E_STATE;
  static_assert(STATS_STRIPES * sizeof(DeviceStats) <= 64 * 1024, "the copies are read into a stack buffer");
  DeviceStats stripes[STATS_STRIPES];
  if (hipMemcpyAsync(stripes, e->stats, sizeof stripes, hipMemcpyDeviceToHost, e->stream) != hipSuccess ||
      hipStreamSynchronize(e->stream) != hipSuccess)
    return ENV_E_HIP;
  DeviceStats d = empty_stats();
  for (const DeviceStats& s : stripes) {
    d.episodes += s.episodes;
    d.length_sum += s.length_sum;
    d.return_sum_i += s.return_sum_i;
    d.return_sum_f += s.return_sum_f;
    d.nonfinite += s.nonfinite;
    d.return_min_key = s.return_min_key < d.return_min_key ? s.return_min_key : d.return_min_key;
    d.return_max_key = s.return_max_key > d.return_max_key ? s.return_max_key : d.return_max_key;
  }
  host_out->episodes = (int64_t)d.episodes;
  host_out->length_sum = (int64_t)d.length_sum;
  host_out->nonfinite = (int64_t)d.nonfinite;
  const bool any = d.episodes > 0;
  if (e->kind == ENV_BODY) {
    host_out->return_sum = d.return_sum_f;
    host_out->return_min = any ? (double)key_to_float(d.return_min_key) : INFINITY;
    host_out->return_max = any ? (double)key_to_float(d.return_max_key) : -INFINITY;
  } else {
    host_out->return_sum = (double)d.return_sum_i;
    host_out->return_min = any ? (double)d.return_min_key : INFINITY;
    host_out->return_max = any ? (double)d.return_max_key : -INFINITY;
  }
  if (reset_counters) {
    const EmptyStats z;
    if (hipMemcpyAsync(e->stats, z.stripes, sizeof z.stripes, hipMemcpyHostToDevice, e->stream) != hipSuccess ||
        hipStreamSynchronize(e->stream) != hipSuccess)
      return ENV_E_HIP;
  }
  return ENV_OK;
}

size_t env_state_bytes(const env_t* e) {
  return e ? 8 + (size_t)4 * (size_t)e->fields * (size_t)e->n : 0;
}

int env_get_state(env_t* e, void* host_buf, size_t bytes) {
  if (!e || !host_buf || bytes != env_state_bytes(e)) return ENV_E_ARG;
  if (!on_own_device(e)) return ENV_E_STATE;
  std::memcpy(host_buf, &e->step, 8);
  if (e->device_counter) {
    uint64_t s = 0;
    if (read_device_step(e, &s) != ENV_OK) return ENV_E_HIP;
    std::memcpy(host_buf, &s, 8);
  }
  if (hipMemcpyAsync(static_cast<char*>(host_buf) + 8, e->state, bytes - 8, hipMemcpyDeviceToHost,
                     e->stream) != hipSuccess ||
      hipStreamSynchronize(e->stream) != hipSuccess)
    return ENV_E_HIP;
  return ENV_OK;
}

int env_set_state(env_t* e, const void* host_buf, size_t bytes) {
  if (!e || !host_buf || bytes != env_state_bytes(e)) return ENV_E_ARG;
  if (!on_own_device(e)) return ENV_E_STATE;
  const char* fields = static_cast<const char*>(host_buf) + 8;
  // Pong: a negative zero in a float field (the game never produces one) is stored as +0, so that
  // the step's sign-bit tests and the comparisons they stand for agree on every state.
  std::vector<uint32_t> fixed;
  if (e->kind == ENV_PONG || e->kind == ENV_PONG_PIXELS) {
    const size_t words = (size_t)PONG_FLOAT_FIELDS * (size_t)e->n;
    bool any = false;
    for (size_t k = 0; k < words && !any; ++k) {
      uint32_t w;
      std::memcpy(&w, fields + 4 * k, 4);
      any = w == 0x80000000u;
    }
    if (any) {
      try { fixed.resize((bytes - 8) / 4); } catch (const std::bad_alloc&) { return ENV_E_ALLOC; }
      std::memcpy(fixed.data(), fields, bytes - 8);
      for (size_t k = 0; k < words; ++k)
        if (fixed[k] == 0x80000000u) fixed[k] = 0u;
      fields = reinterpret_cast<const char*>(fixed.data());
    }
  }
  if (hipMemcpyAsync(e->state, fields, bytes - 8, hipMemcpyHostToDevice, e->stream) != hipSuccess ||
      hipStreamSynchronize(e->stream) != hipSuccess)
    return ENV_E_HIP;
  std::memcpy(&e->step, host_buf, 8);
  if (e->device_counter) {
    const StepCounter c = {e->step, 0u, 0u};
    if (hipMemcpyAsync(e->counter, &c, sizeof c, hipMemcpyHostToDevice, e->stream) != hipSuccess ||
        hipStreamSynchronize(e->stream) != hipSuccess)
      return ENV_E_HIP;
  }
  e->was_reset = true;
  if (e->kind == ENV_PONG_PIXELS) {
    pixel_pipe_invalidate(e->pipe);
    if (pixel_counted_forget(e->pipe, e->stream) != hipSuccess) return ENV_E_HIP;
    // the observation buffer is not part of the state: it no longer matches
    if (pixel_update_forget(e->pipe, e->stream) != hipSuccess) return ENV_E_HIP;
  }
  return ENV_OK;
}

int env_obs_dim(int kind) {
  switch (kind) {
    case ENV_PONG: return PONG_OBS;
    case ENV_PONG_PIXELS: return 4 * FRAME_BYTES;
    case ENV_BODY: return BODY_OBS;
    case ENV_CARTPOLE: return CARTPOLE_OBS;
  }
  return ENV_E_ARG;
}

int env_action_dim(int kind) {
  switch (kind) {
    case ENV_PONG: case ENV_PONG_PIXELS: case ENV_CARTPOLE: return 1;
    case ENV_BODY: return BODY_ACT;
  }
  return ENV_E_ARG;
}

int64_t env_num_envs(const env_t* e) { return e ? e->n : 0; }
uint64_t env_step_count(const env_t* e) {
  if (!e) return 0;
  if (!e->device_counter) return e->step;
  uint64_t s = 0;
  return read_device_step(e, &s) == ENV_OK ? s : UINT64_MAX;
}

int env_set_stream(env_t* e, void* hip_stream) {
  if (!e) return ENV_E_ARG;
  e->stream = static_cast<hipStream_t>(hip_stream);
  return ENV_OK;
}

const char* env_strerror(int code) {
  switch (code) {
    case ENV_OK: return "ok";
    case ENV_E_ARG: return "bad argument (NULL, size, alignment or not device memory)";
    case ENV_E_ALLOC: return "device allocation failed";
    case ENV_E_HIP: return "HIP runtime call or kernel launch failed";
    case ENV_E_STATE:
      return "wrong state for this call (env_reset / env_set_state not called yet, the stream is "
             "capturing and the handle keeps its step counter on the host, or the current device is "
             "not the handle's)";
    case ENV_E_UNSUPPORTED: return "not supported for this environment kind";
    case ENV_E_TOO_LARGE: return "more environments than env_step_pixels_noalloc's fixed scratch array holds";
  }
  return "unknown status";
}

// How many ring steps of a delta-update handle rewrote only changed pixels, and how many fell back
// to a full write of the slot.
int mi355env_pixel_update_counts(const void* handle, int64_t* delta_steps, int64_t* full_steps) {
  const env_t* e = static_cast<const env_t*>(handle);
  if (!e || !delta_steps || !full_steps || e->kind != ENV_PONG_PIXELS) return ENV_E_ARG;
  return pixel_update_counts(const_cast<env_t*>(e)->pipe, e->device_counter, delta_steps, full_steps, e->stream) ==
                 hipSuccess
             ? ENV_OK
             : ENV_E_HIP;
}

// Measurement knob, not part of the documented boundary: launch shape of the pixel kernels.
int mi355env_tune_pixels(int envs_per_wave, int streaming) {
  return set_pixel_tuning(envs_per_wave, streaming) ? ENV_OK : ENV_E_ARG;
}

int mi355env_tune_plane_path(int on) { return set_plane_path(on) ? ENV_OK : ENV_E_ARG; }

int mi355env_tune_rollout(int threads_per_block, int xcd_remap) {
  return set_rollout_block(threads_per_block, xcd_remap) ? ENV_OK : ENV_E_ARG;
}

// Steps per chunk of the Pong rollout's main loop: 2, 4 or 8; 0 = chosen from N.
int mi355env_tune_rollout_chunk(int steps) { return set_rollout_chunk(steps) ? ENV_OK : ENV_E_ARG; }

// Pong rollout with a second wavefront per 64 environments drawing the Philox blocks: 0 = chosen
// from N and T, 1 = never, 2 = whenever the launch has in-kernel actions and raw observations.
int mi355env_tune_rollout_split(int mode) { return set_rollout_split(mode) ? ENV_OK : ENV_E_ARG; }

// Pong rollout pacing: the write rate (GB/s) the paced loop holds the launch to; forces that loop
// for any N.  0 = chosen from N, -1 = never paced.
int mi355env_tune_rollout_pace(int gb_per_s) { return set_rollout_pace(gb_per_s) ? ENV_OK : ENV_E_ARG; }

// 1 = whether the Pong rollout is paced, and at which rate, is measured once per device and batch
// size (default), 0 = taken from the launcher's table.
int mi355env_tune_measure_pace(int on) { return set_measure_pace(on) ? ENV_OK : ENV_E_ARG; }

// What was measured for n environments on the current device: GB/s, -1 = not paced, 0 = nothing yet.
int mi355env_pace_choice(int64_t n) { return pong_pace_choice(n); }

// Pong env_step: 1 = the dedicated step kernel (default), 0 = the rollout kernel with T = 1.
int mi355env_tune_step_kernel(int on) { return set_step_kernel(on) ? ENV_OK : ENV_E_ARG; }
unsigned long long mi355env_resident_step_launches(void) { return resident_step_launches(); }

// Cart-pole rollout with a second wavefront per 64 environments drawing the Philox blocks: 0 = chosen
// from N and T, 1 = never, 2 = whenever the launch has in-kernel actions.
int mi355env_tune_cartpole_split(int mode) { return set_cartpole_split(mode) ? ENV_OK : ENV_E_ARG; }

// 0 = direct observation stores, 1 = paged through LDS wherever a workgroup is full, 2 = by N.
int mi355env_tune_paged_stores(int mode) { return set_paged_stores(mode) ? ENV_OK : ENV_E_ARG; }

// Pixel env_rollout: 0 = one launch, 1 = staged and rendered a chunk of steps at a time, 2 = by N.
int mi355env_tune_frame_trajectory(int mode) { return set_traj_mode(mode) ? ENV_OK : ENV_E_ARG; }

}  // extern "C"
