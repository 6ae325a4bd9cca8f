// Planar articulated body: launch descriptors (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "stats.hpp"
#include "step_counter.hpp"

namespace envk {

constexpr int BODY_DOF = 9;      // x, z, pitch, 3 back-leg joints, 3 front-leg joints
constexpr int BODY_ACT = 6;
constexpr int BODY_OBS = 17;     // q[1:9], v[0:9]
constexpr int BODY_FIELDS = 20;  // q[9] v[9] ep_ret ep_len
constexpr float BODY_DEFAULT_ARMATURE = 0.1f;
constexpr float BODY_DEFAULT_JOINT_DAMPING = 3.0f;
constexpr float BODY_DEFAULT_FRICTION_MU = 0.4f;

struct BodyLaunch {
  uint32_t* state;       // SoA [20][n]
  int64_t n;
  uint64_t seed;
  uint64_t step0;        // used when counter == nullptr
  StepCounter* counter;  // device-resident step counter, or nullptr
  int32_t ticket;        // set by the launcher: the launch advances `counter` itself (small grids)
  int32_t envs_per_wave; // set by the launcher: environments (lane pairs) a wavefront takes, at most 32
  int32_t T;
  int32_t max_episode_steps;
  float armature, joint_damping, friction_mu;
  int32_t newton;        // contact model: 0 penalty spring + limit projection, 1 Newton on the soft-constraint QP
  int32_t f32;           // arithmetic inside a step: 0 float64 (default), 1 float32
  const float* actions;  // [T,n,6] or nullptr
  float* obs;            // [T,n,17]
  float* reward;         // [T,n]
  uint8_t* done;         // [T,n]
  DeviceStats* stats;
};

hipError_t launch_body_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                             const StepCounter* counter, float* obs, hipStream_t stream);
hipError_t launch_body_rollout(const BodyLaunch& a, hipStream_t stream);

}  // namespace envk
