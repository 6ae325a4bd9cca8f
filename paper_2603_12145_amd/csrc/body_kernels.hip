// Planar articulated body ("HalfCheetah-like", paper App. A.1: forward kinematics, mass matrix,
// bias forces, contact Jacobians, Cholesky; first solver revision = penalty spring): reset and the
// fused T-step rollout (T = 1 is env_step).  Two lanes per environment (one per leg), everything in
// registers.
//
// Model: q = (x, z, theta, b1, b2, b3, f1, f2, f3); torso of length 1 with the hips at its ends;
// each leg a chain thigh / shin / foot of uniform rods hanging along d(phi) = (sin phi, -cos phi),
// phi = theta + joint angles down the chain.  Per substep (5 per step, h = 0.01):
//   M v* = M v + h (Q_g - bias + gear * a - damping * v_joint + contact),
//   joints at a limit that still move outwards are removed (rows / columns -> identity, right-hand
//   side 0) and the system is solved again (M-orthogonal projection), q += h v+, joints clipped.
//
// Formulation used here (hand-derived for this tree, not a generic link loop):
//  * every Jacobian column of a leg point is a partial sum of the three link vectors
//    E_k = L_k (cos phi_k, sin phi_k), plus H = +-(1/2) t_perp for the pitch column, so the 9x9 mass
//    matrix is assembled from six centre-of-mass vectors per leg and a handful of dot products;
//  * the two legs couple only through the root, so with the ordering (back joints, front joints,
//    root) the Cholesky factor has no fill between the legs: two 3x3 factorisations, two 3x3
//    triangular solves with three right-hand sides, one 3x3 Schur complement;
//  * that structure is also the work split: lane 2i carries the root and the back leg of
//    environment i, lane 2i+1 the root and the front leg; each builds and factors its own leg block,
//    the root's mass, right-hand side and Schur complement are sums of the two lanes' parts (one
//    DPP quad permutation per 32-bit half), and both lanes solve the same 3x3 root system;
//  * sin / cos of the six joint angles (always in [-1, 1]) come from a polynomial without range
//    reduction, the link angles from angle addition on top of one sincos of the pitch.
//
// Second contact model (solver = Newton; the paper's final solver revision for this case study,
// App. A.1: an acceleration-space quadratic programme solved by Newton's method with Cholesky
// factorisations).  The substep's acceleration minimises
//     1/2 (a - a0)^T M (a - a0) + sum_i D_i / 2 * min(0, J_i a - aref_i)^2,
// rows i = the two friction-pyramid edges J_z +- mu J_x of every contact point below the ground
// (aref = -b J v - k z - dJ/dt qdot, k = 1/tc^2, b = 2/tc, tc = 0.02) and one row per joint sitting
// at a limit (aref = -b J v).  Newton on the active set with unit steps: S = rows with negative
// residual at the current a; a <- (M + sum_S D J^T J)^-1 (M a0 + sum_S D aref J); stop when S repeats
// (at most 8 passes).  A contact row of a leg touches only the root and that leg's joints, so
// M + sum D J^T J keeps the block structure of M and goes through the same block Cholesky; rows are
// never stored: each pass rebuilds them from the link vectors (8 multiply-adds per leg).  A
// wavefront leaves the loop when no lane's active set changed; a lane whose set is already stable
// re-solves the same system and gets the same numbers.
//
// Arithmetic is float64 inside a step by default: the 9x9 system has a condition number of order
// 10^2, which in float32 leaves a per-step error of about 10^-6..10^-5 of the state, the same size
// as the agreement asked of this kernel.  MI355X issues float64 FMAs at the rate of unpacked
// float32, so the price is registers (and the quarter-rate reciprocal square root), not issue
// slots.  State, observations and rewards are float32 in memory; the state is rounded to float32
// at the end of every step, so a T-step launch equals T one-step launches bit for bit.
// The same text is compiled a second time in float32 (the precision the paper's case study names,
// App. A.1), selected per handle: body_impl.inc holds the arithmetic, this file the two
// instantiations and the launchers.
#include "body_kernels.hpp"
#include "philox.hpp"

#pragma clang fp contract(fast)

namespace envk {

namespace {

#define LIT(x) ((real)(x))
// Newton steps behind the float64 reciprocal square root estimate.  The estimate is good to about
// 2^-23, one step leaves about 2^-45 -- nine orders of magnitude under the rounding of the float32
// state the step ends in -- and a second step (full precision) changed no output of 24576 single
// steps against the oracle while costing 4 % of the launch (N = 8192 x T = 1000: 10.09 against
// 9.73 ms).  Build with -DBODY_RSQ_STEPS=2 for the fully converged form.
#ifndef BODY_RSQ_STEPS
#define BODY_RSQ_STEPS 1
#endif

namespace f64 {
#define BODY_REAL double
#ifndef BODY_F64_WAVES
#define BODY_F64_WAVES 2
#endif
#define BODY_OCCUPANCY __attribute__((amdgpu_waves_per_eu(BODY_F64_WAVES, BODY_F64_WAVES)))
#include "body_impl.inc"
#undef BODY_REAL
#undef BODY_OCCUPANCY
}  // namespace f64

// The float64 text once more for launches of at most one wavefront per SIMD (1024 wavefronts): no
// register cap.  The Newton model then keeps its loop invariants in registers (313) instead of
// 244 bytes of scratch per lane, which is worth 6 % of a fused launch at N = 8192 (18.6 -> 17.5 ms
// per 1000 steps) and 15 % of a single step (30.7 -> 26.3 us: the spills and reloads of the
// prologue are paid at every launch).  With two wavefronts per SIMD the capped build wins
// (N = 262144 x T = 100: 14.7 against 17.1 ms).  Same arithmetic in the same order: same bits.
namespace f64_alone {
#define BODY_REAL double
#define BODY_OCCUPANCY __attribute__((amdgpu_waves_per_eu(1, 1)))
#include "body_impl.inc"
#undef BODY_REAL
#undef BODY_OCCUPANCY
}  // namespace f64_alone

namespace f32 {
#define BODY_REAL float
#ifndef BODY_F32_WAVES
#define BODY_F32_WAVES 4
#endif
#define BODY_OCCUPANCY __attribute__((amdgpu_waves_per_eu(BODY_F32_WAVES, BODY_F32_WAVES)))
#include "body_impl.inc"
#undef BODY_REAL
#undef BODY_OCCUPANCY
}  // namespace f32

#undef LIT

}  // namespace

hipError_t launch_body_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                             const StepCounter* counter, float* obs, hipStream_t stream) {
  hipLaunchKernelGGL(f64::body_reset_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, state, n,
                     seed, step, counter, obs);
  return hipGetLastError();
}

hipError_t launch_body_rollout(const BodyLaunch& a, hipStream_t stream) {
  BodyLaunch a2 = a;
  // A wavefront of the Newton model runs as many passes as its slowest environment needs.  When
  // the batch leaves SIMDs empty anyway, fewer environments per wavefront (the other lanes idle)
  // mean a smaller maximum: N = 8192 x T = 400 takes 8.46 ms with 32 environments per wavefront,
  // 8.00 with 16, 7.53 with 8 (12.1 with 4: too many wavefronts per SIMD by then); N = 16384:
  // 4.31 / 4.13 / 6.74.  The penalty model gains nothing (its second solve is needed by some
  // environment of almost any group) and keeps 32.
  a2.envs_per_wave = !a.newton ? 32 : a.n <= 8192 ? 8 : a.n <= 16384 ? 16 : 32;
  const dim3 grid((unsigned)((a.n + a2.envs_per_wave - 1) / a2.envs_per_wave));
  a2.ticket = grid.x <= TICKET_MAX_BLOCKS;
  const dim3 block(64);
  if (a.f32) {
    if (a.newton && a.n >= 32768) hipLaunchKernelGGL((f32::body_rollout_kernel<true, true>), grid, block, 0, stream, a2);
    else if (a.newton) hipLaunchKernelGGL((f32::body_rollout_kernel<true, false>), grid, block, 0, stream, a2);
    else hipLaunchKernelGGL((f32::body_rollout_kernel<false, false>), grid, block, 0, stream, a2);
  } else if (a.newton && grid.x <= 1024u) {          // at most one wavefront per SIMD
    if (a.n >= 32768) hipLaunchKernelGGL((f64_alone::body_rollout_kernel<true, true>), grid, block, 0, stream, a2);
    else hipLaunchKernelGGL((f64_alone::body_rollout_kernel<true, false>), grid, block, 0, stream, a2);
  } else {
    if (a.newton && a.n >= 32768) hipLaunchKernelGGL((f64::body_rollout_kernel<true, true>), grid, block, 0, stream, a2);
    else if (a.newton) hipLaunchKernelGGL((f64::body_rollout_kernel<true, false>), grid, block, 0, stream, a2);
    else hipLaunchKernelGGL((f64::body_rollout_kernel<false, false>), grid, block, 0, stream, a2);
  }
  const hipError_t err = hipGetLastError();
  return err != hipSuccess ? err : advance_step_counter_behind(a.counter, a.T, grid.x, stream);
}

}  // namespace envk
