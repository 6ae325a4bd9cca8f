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
// Arithmetic is float64 inside a step: the 9x9 system has a condition number of order 10^2, which
// in float32 leaves a per-step error of about 10^-6..10^-5 of the state, the same size as the
// agreement asked of this kernel.  MI355X issues float64 FMAs at the rate of unpacked float32, so
// the price is registers, not time.  State, observations and rewards are float32 in memory; the
// state is rounded to float32 at the end of every step, so a T-step launch equals T one-step
// launches bit for bit.
#include "body_kernels.hpp"
#include "philox.hpp"

#pragma clang fp contract(fast)

namespace envk {

namespace {

typedef double real;

constexpr int WAVE = 64;
constexpr real L1 = 0.29, L2 = 0.30, L3 = 0.19;
constexpr real M1 = 1.5, M2 = 1.2, M3 = 0.9, MT = 6.4;
constexpr real MLEG = M1 + M2 + M3, MTOT = MT + 2 * MLEG;
constexpr real I1 = M1 * L1 * L1 / 12, I2 = M2 * L2 * L2 / 12, I3 = M3 * L3 * L3 / 12, IT = MT / 12;
constexpr real GRAVITY = 9.81, CONTACT_K = 1e4, CONTACT_C = 100.0, STEP_H = 0.01, GEAR = 120.0;
constexpr float Z0 = 0.8f;
constexpr int SUBSTEPS = 5;

struct Vec2 { real x, z; };
__device__ __forceinline__ Vec2 operator+(Vec2 a, Vec2 b) { return {a.x + b.x, a.z + b.z}; }
__device__ __forceinline__ Vec2 operator-(Vec2 a, Vec2 b) { return {a.x - b.x, a.z - b.z}; }
__device__ __forceinline__ Vec2 operator*(real s, Vec2 a) { return {s * a.x, s * a.z}; }
__device__ __forceinline__ real dot(Vec2 a, Vec2 b) { return a.x * b.x + a.z * b.z; }

// sin and cos on [-1, 1] (joint angles are clipped to that range): Taylor series to x^19 / x^18,
// truncation error below 1e-17.
__device__ __forceinline__ void sincos_unit(real x, real& s, real& c) {
  const real x2 = x * x;
  real ps = -1.0 / 121645100408832000.0;            // -1/19!
  ps = ps * x2 + 1.0 / 355687428096000.0;           //  1/17!
  ps = ps * x2 - 1.0 / 1307674368000.0;             // -1/15!
  ps = ps * x2 + 1.0 / 6227020800.0;                //  1/13!
  ps = ps * x2 - 1.0 / 39916800.0;                  // -1/11!
  ps = ps * x2 + 1.0 / 362880.0;                    //  1/9!
  ps = ps * x2 - 1.0 / 5040.0;                      // -1/7!
  ps = ps * x2 + 1.0 / 120.0;                       //  1/5!
  ps = ps * x2 - 1.0 / 6.0;                         // -1/3!
  s = x + x * x2 * ps;
  real pc = 1.0 / 6402373705728000.0;               //  1/18!
  pc = pc * x2 - 1.0 / 20922789888000.0;            // -1/16!
  pc = pc * x2 + 1.0 / 87178291200.0;               //  1/14!
  pc = pc * x2 - 1.0 / 479001600.0;                 // -1/12!
  pc = pc * x2 + 1.0 / 3628800.0;                   //  1/10!
  pc = pc * x2 - 1.0 / 40320.0;                     // -1/8!
  pc = pc * x2 + 1.0 / 720.0;                       //  1/6!
  pc = pc * x2 - 1.0 / 24.0;                        // -1/4!
  pc = pc * x2 + 0.5;                               //  1/2!
  c = 1.0 - x2 * pc;
}

// sin and cos of the pitch, which is not confined to an interval: reduce by multiples of pi/2 with a
// two-part constant (exact to ~1e-16 for the |x| < 1e4 a tumbling body can reach), evaluate the
// unit-interval polynomials on the remainder (|r| <= pi/4) and undo the quadrant.  About half the
// instructions of the general library routine, which carries a large-argument path.
__device__ __forceinline__ void sincos_any(real x, real& s, real& c) {
  const real k = __builtin_rint(x * 0.63661977236758134308);              // x / (pi/2)
  real r = __builtin_fma(-k, 1.57079632679489655800e+00, x);               // pi/2, leading 53 bits
  r = __builtin_fma(-k, 6.12323399573676603587e-17, r);                    // ... and the next 53
  real sr, cr;
  sincos_unit(r, sr, cr);
  const int q = (int)k & 3;
  const real s0 = (q & 1) ? cr : sr, c0 = (q & 1) ? sr : cr;
  s = (q & 2) ? -s0 : s0;
  c = ((q + 1) & 2) ? -c0 : c0;
}

// 1 / sqrt(s) to full precision: hardware estimate plus two Newton steps.
__device__ __forceinline__ real inv_sqrt(real s) {
  real y = __builtin_amdgcn_rsq(s);
  y = y * (1.5 - 0.5 * s * y * y);
  y = y * (1.5 - 0.5 * s * y * y);
  return y;
}

struct Leg {                 // everything one leg contributes, for one substep
  Vec2 E1, E2, E3;           // L_k (cos phi_k, sin phi_k)
  Vec2 H;                    // +-(1/2) t_perp
  real w1, w2, w3;           // link angular rates
  real A[6];                 // joint block of M: 00 01 02 11 12 22
  real C[3][3];              // C[root coord x,z,theta][joint]
  real mthth;                // this leg's part of M[theta][theta]
  Vec2 Pth;                  // this leg's part of (M[x][theta], M[z][theta])
  real rhs[3];               // generalised force on the joints (everything but M qddot)
  real rhs_x, rhs_z, rhs_th; // ... and this leg's part of the root rows
};

struct Params {
  real armature, damping, mu;
  real d_contact, d_limit, k_ref, b_ref;   // Newton model: 1 / regularisation, reference spring and damper
};

constexpr real NEWTON_TIME_CONST = 0.02, NEWTON_REG_CONTACT = 0.02, NEWTON_REG_LIMIT = 0.5;
constexpr int NEWTON_MAX_PASSES = 8;

struct LegRows {             // Newton model: what the contact rows of one leg need besides the link vectors
  uint32_t below;            // bit k: point k (hip, knee, ankle, toe) is under the ground, its rows exist
  real aref[4][2];           // reference acceleration of the +mu and the -mu edge
};

// Kinematics, mass-matrix blocks, bias, gravity and contact of one leg.
// sign = -1 back, +1 front; (st, ct) = sin / cos pitch; jq, jv = the leg's joint angles and rates.
template <bool NEWTON>
__device__ __forceinline__ void leg_terms(Leg& g, LegRows& rows, const real sign, const real st, const real ct,
                                          const real z, const real vx, const real vz, const real vth,
                                          const real* jq, const real* jv, const Params& P) {
  // link angles by angle addition
  real sj, cj;
  sincos_unit(jq[0], sj, cj);
  const real s1 = st * cj + ct * sj, c1 = ct * cj - st * sj;
  sincos_unit(jq[1], sj, cj);
  const real s2 = s1 * cj + c1 * sj, c2 = c1 * cj - s1 * sj;
  sincos_unit(jq[2], sj, cj);
  const real s3 = s2 * cj + c2 * sj, c3 = c2 * cj - s2 * sj;
  g.w1 = vth + jv[0]; g.w2 = g.w1 + jv[1]; g.w3 = g.w2 + jv[2];
  g.E1 = {L1 * c1, L1 * s1}; g.E2 = {L2 * c2, L2 * s2}; g.E3 = {L3 * c3, L3 * s3};
  g.H = {-0.5 * sign * st, 0.5 * sign * ct};

  // centre-of-mass Jacobian columns: thigh A; shin B0, B1; foot C0, C1, C2
  const Vec2 A = 0.5 * g.E1;
  const Vec2 B1 = 0.5 * g.E2, B0 = g.E1 + B1;
  const Vec2 C2 = 0.5 * g.E3, C1 = g.E2 + C2, C0 = g.E1 + C1;
  g.A[0] = M1 * dot(A, A) + M2 * dot(B0, B0) + M3 * dot(C0, C0) + (I1 + I2 + I3);
  g.A[1] = M2 * dot(B0, B1) + M3 * dot(C0, C1) + (I2 + I3);
  g.A[2] = M3 * dot(C0, C2) + I3;
  g.A[3] = M2 * dot(B1, B1) + M3 * dot(C1, C1) + (I2 + I3);
  g.A[4] = M3 * dot(C1, C2) + I3;
  g.A[5] = M3 * dot(C2, C2) + I3;
  const Vec2 P0 = M1 * A + M2 * B0 + M3 * C0, P1 = M2 * B1 + M3 * C1, P2 = M3 * C2;
  g.C[0][0] = P0.x; g.C[0][1] = P1.x; g.C[0][2] = P2.x;
  g.C[1][0] = P0.z; g.C[1][1] = P1.z; g.C[1][2] = P2.z;
  g.C[2][0] = dot(g.H, P0) + g.A[0]; g.C[2][1] = dot(g.H, P1) + g.A[1]; g.C[2][2] = dot(g.H, P2) + g.A[2];
  g.Pth = MLEG * g.H + P0;
  g.mthth = MLEG * 0.25 + 2.0 * dot(g.H, P0) + g.A[0];
  g.A[0] += P.armature; g.A[3] += P.armature; g.A[5] += P.armature;

  // velocity-product accelerations of the three centres of mass (centripetal terms only)
  const Vec2 Hk = {-0.5 * sign * ct * vth * vth, -0.5 * sign * st * vth * vth};
  const Vec2 D1 = {L1 * s1 * g.w1 * g.w1, -L1 * c1 * g.w1 * g.w1};
  const Vec2 D2 = {L2 * s2 * g.w2 * g.w2, -L2 * c2 * g.w2 * g.w2};
  const Vec2 D3 = {L3 * s3 * g.w3 * g.w3, -L3 * c3 * g.w3 * g.w3};
  const Vec2 k1 = Hk - 0.5 * D1, k2 = Hk - D1 - 0.5 * D2, k3 = Hk - D1 - D2 - 0.5 * D3;
  const real h0 = M1 * dot(A, k1) + M2 * dot(B0, k2) + M3 * dot(C0, k3);
  const real h1 = M2 * dot(B1, k2) + M3 * dot(C1, k3);
  const real h2 = M3 * dot(C2, k3);
  const Vec2 K = M1 * k1 + M2 * k2 + M3 * k3;

  // ground contact at hip, knee, ankle, toe: normal spring-damper without adhesion, friction
  // c * vx clipped to +-mu * fn
  const real z_hip = z + 0.5 * sign * st;
  const real z_knee = z_hip - L1 * c1, z_ank = z_knee - L2 * c2, z_toe = z_ank - L3 * c3;
  const Vec2 v_hip = Vec2{vx, vz} + vth * g.H;
  const Vec2 v_knee = v_hip + g.w1 * g.E1, v_ank = v_knee + g.w2 * g.E2, v_toe = v_ank + g.w3 * g.E3;
  auto force = [&](real zp, Vec2 vp) -> Vec2 {
    if (NEWTON) return Vec2{0.0, 0.0};           // contact enters through the constraint rows instead
    real fn = -CONTACT_K * zp - CONTACT_C * vp.z;
    fn = (zp < 0.0 && fn > 0.0) ? fn : 0.0;
    real want = CONTACT_C * vp.x;
    const real cap = P.mu * fn;
    want = want > cap ? cap : want;
    want = want < -cap ? -cap : want;
    return {-want, fn};
  };
  const Vec2 S3 = force(z_toe, v_toe);
  const Vec2 S2 = S3 + force(z_ank, v_ank);
  const Vec2 S1 = S2 + force(z_knee, v_knee);
  const Vec2 S0 = S1 + force(z_hip, v_hip);
  const real c2f = dot(g.E3, S3), c1f = dot(g.E2, S2) + c2f, c0f = dot(g.E1, S1) + c1f;
  if (NEWTON) {
    // velocity-product accelerations of the four points: the centre-of-mass ones with whole links
    const Vec2 a_knee = Hk - D1, a_ank = a_knee - D2, a_toe = a_ank - D3;
    const real zs[4] = {z_hip, z_knee, z_ank, z_toe};
    const Vec2 vs[4] = {v_hip, v_knee, v_ank, v_toe};
    const Vec2 as[4] = {Hk, a_knee, a_ank, a_toe};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      rows.below = (k == 0 ? 0u : rows.below) | (zs[k] < 0.0 ? 1u << k : 0u);
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const real smu = e == 0 ? P.mu : -P.mu;
        rows.aref[k][e] = -P.b_ref * (vs[k].z + smu * vs[k].x) - P.k_ref * zs[k] - (as[k].z + smu * as[k].x);
      }
    }
  }

  // right-hand sides: gravity (-g times the z row of M) - bias + contact; torque and damping are
  // added by the caller
  g.rhs[0] = -GRAVITY * g.C[1][0] - h0 + c0f;
  g.rhs[1] = -GRAVITY * g.C[1][1] - h1 + c1f;
  g.rhs[2] = -GRAVITY * g.C[1][2] - h2 + c2f;
  g.rhs_x = -K.x + S0.x;
  g.rhs_z = -K.z + S0.z;
  g.rhs_th = -GRAVITY * g.Pth.z - (dot(g.H, K) + h0) + dot(g.H, S0) + c0f;
}

struct LegFactor {           // Cholesky factor of a leg block and Y = L^-1 C^T
  real i00, l10, l20, i11, l21, i22;    // iXX = 1 / lXX
  real Y[3][3];                          // Y[k][root coord]
};

// keep[j] = false removes joint j (row and column of the identity, no coupling to the root).
template <class Block>   // anything with A[6] and C[3][3]
__device__ __forceinline__ void factor_leg(LegFactor& f, const Block& g, const bool keep[3]) {
  const real a00 = keep[0] ? g.A[0] : 1.0;
  const real a01 = (keep[0] && keep[1]) ? g.A[1] : 0.0;
  const real a02 = (keep[0] && keep[2]) ? g.A[2] : 0.0;
  const real a11 = keep[1] ? g.A[3] : 1.0;
  const real a12 = (keep[1] && keep[2]) ? g.A[4] : 0.0;
  const real a22 = keep[2] ? g.A[5] : 1.0;
  f.i00 = inv_sqrt(a00);
  f.l10 = a01 * f.i00;
  f.l20 = a02 * f.i00;
  f.i11 = inv_sqrt(a11 - f.l10 * f.l10);
  f.l21 = (a12 - f.l20 * f.l10) * f.i11;
  f.i22 = inv_sqrt(a22 - f.l20 * f.l20 - f.l21 * f.l21);
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    const real c0 = keep[0] ? g.C[r][0] : 0.0, c1 = keep[1] ? g.C[r][1] : 0.0, c2 = keep[2] ? g.C[r][2] : 0.0;
    f.Y[0][r] = c0 * f.i00;
    f.Y[1][r] = (c1 - f.l10 * f.Y[0][r]) * f.i11;
    f.Y[2][r] = (c2 - f.l20 * f.Y[0][r] - f.l21 * f.Y[1][r]) * f.i22;
  }
}

__device__ __forceinline__ void forward_leg(const LegFactor& f, const real b[3], real y[3]) {
  y[0] = b[0] * f.i00;
  y[1] = (b[1] - f.l10 * y[0]) * f.i11;
  y[2] = (b[2] - f.l20 * y[0] - f.l21 * y[1]) * f.i22;
}

__device__ __forceinline__ void backward_leg(const LegFactor& f, const real y[3], const real xr[3], real x[3]) {
  real t[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) t[k] = y[k] - (f.Y[k][0] * xr[0] + f.Y[k][1] * xr[1] + f.Y[k][2] * xr[2]);
  x[2] = t[2] * f.i22;
  x[1] = (t[1] - f.l21 * x[2]) * f.i11;
  x[0] = (t[0] - f.l10 * x[1] - f.l20 * x[2]) * f.i00;
}

struct RootBlock { real xx, xz, xth, zz, zth, thth; };   // symmetric 3x3 over (x, z, pitch)

struct BodyLane {
  real q[9], v[9];
  float ep_ret;
  int ep_len;
};


// ---- Newton contact model ---------------------------------------------------------------------------

struct LegBlock { real A[6]; real C[3][3]; };

template <int N> struct Depth { static constexpr int value = N; };

// Calls fn(depth tag, point k, edge e, smu, theta entry, joint entries u[3]) for the eight contact
// rows of a leg.  Row = (smu, 1, t | u0, u1, u2) over (x, z, theta | the leg's joints): the dot
// products of the pyramid edge n = (smu, 1) with the Jacobian columns, which are partial sums of
// the link vectors.
template <class F>
__device__ __forceinline__ void for_each_contact_row(const Leg& g, const real mu, F&& fn) {
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const real smu = e == 0 ? mu : -mu;
    const real h = g.H.z + smu * g.H.x;
    const real e1 = g.E1.z + smu * g.E1.x, e2 = g.E2.z + smu * g.E2.x, e3 = g.E3.z + smu * g.E3.x;
    const real u0[3] = {0.0, 0.0, 0.0};
    fn(Depth<0>{}, 0, e, smu, h, u0);
    const real u1[3] = {e1, 0.0, 0.0};
    fn(Depth<1>{}, 1, e, smu, h + e1, u1);
    const real u2[3] = {e1 + e2, e2, 0.0};
    fn(Depth<2>{}, 2, e, smu, h + u2[0], u2);
    const real u3[3] = {u2[0] + e3, e2 + e3, e3};
    fn(Depth<3>{}, 3, e, smu, h + u3[0], u3);
  }
}

// Bits 0..7 of the result: contact rows of this leg with a negative residual at acceleration
// (ar = root part, aj = this leg's joints); bits 8..10: its joints' limit rows.
__device__ __forceinline__ uint32_t leg_active_set(const Leg& g, const LegRows& rows, const real* jq,
                                                   const real* jv, const real ar[3], const real aj[3],
                                                   const Params& P) {
  uint32_t set = 0;
  for_each_contact_row(g, P.mu, [&](auto depth, int k, int e, real smu, real t, const real* u) {
    real r = smu * ar[0] + ar[1] + t * ar[2] - rows.aref[k][e];
#pragma unroll
    for (int m = 0; m < decltype(depth)::value; ++m) r += u[m] * aj[m];
    set |= ((rows.below >> k & 1u) && r < 0.0) ? (1u << (2 * k + e)) : 0u;
  });
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    const real sgn = jq[m] >= 1.0 ? -1.0 : (jq[m] <= -1.0 ? 1.0 : 0.0);
    const real r = sgn * aj[m] + P.b_ref * sgn * jv[m];          // s a - aref, aref = -b s v
    set |= (sgn != 0.0 && r < 0.0) ? (1u << (8 + m)) : 0u;
  }
  return set;
}

// Adds D J^T J of the active rows to the leg's blocks and the root block, D aref J to the right-hand
// sides.
// SKIP_IDLE_ROWS: leave out a row that is active in no lane of the wavefront (it adds zeros).  The
// eight wave-uniform branches cost a lone wavefront on its SIMD more than they save (they cut the
// pass into blocks the scheduler cannot interleave: 21.8 against 21.4 ms at N = 8192) and pay once
// two wavefronts share a SIMD (14.4 against 15.4 ms at N = 262144), so the launcher picks by N.
template <bool SKIP_IDLE_ROWS>
__device__ __forceinline__ void leg_add_rows(const Leg& g, const LegRows& rows, const real* jq, const real* jv,
                                             const uint32_t set, const Params& P, LegBlock& B, RootBlock& R,
                                             real g_root[3], real g_leg[3]) {
  const int sym[3][3] = {{0, 1, 2}, {1, 3, 4}, {2, 4, 5}};
  for_each_contact_row(g, P.mu, [&](auto depth, int k, int e, real smu, real t, const real* u) {
    if (SKIP_IDLE_ROWS && __ballot(set >> (2 * k + e) & 1u) == 0ull) return;
    const real w = (set >> (2 * k + e) & 1u) ? P.d_contact : 0.0;
    const real aw = w * rows.aref[k][e];
    const real ws = w * smu, wt = w * t;
    R.xx += ws * smu; R.xz += ws; R.xth += ws * t; R.zz += w; R.zth += wt; R.thth += wt * t;
    g_root[0] += aw * smu; g_root[1] += aw; g_root[2] += aw * t;
#pragma unroll
    for (int m = 0; m < decltype(depth)::value; ++m) {
      const real wu = w * u[m];
      B.C[0][m] += wu * smu; B.C[1][m] += wu; B.C[2][m] += wu * t;
      g_leg[m] += aw * u[m];
#pragma unroll
      for (int c = m; c < decltype(depth)::value; ++c) B.A[sym[m][c]] += wu * u[c];
    }
  });
  const int diag[3] = {0, 3, 5};
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    const real sgn = jq[m] >= 1.0 ? -1.0 : (jq[m] <= -1.0 ? 1.0 : 0.0);
    const real w = (set >> (8 + m) & 1u) ? P.d_limit : 0.0;
    B.A[diag[m]] += w;                                            // s^2 = 1
    g_leg[m] += w * (-P.b_ref * sgn * jv[m]) * sgn;
  }
}


// Initial state: q0 = (0, 0.8, 0, ...) + U[-0.1, 0.1), v0 = 0.1 N(0, 1); uniforms from reset streams
// 16..18 in word order, normals from Box-Muller pairs of streams 19..21, all in float32.
__device__ __forceinline__ void body_initial(BodyLane& s, uint64_t seed, uint32_t env, uint64_t step) {
#pragma clang fp contract(off)   // base + (-0.1 + 0.2 u): separately rounded multiply and adds
  uint32_t w[6][4];
#pragma unroll
  for (int b = 0; b < 6; ++b) {
    const Draw4 d = philox_draw(seed, env, step, 16u + (uint32_t)b);
    w[b][0] = d.w0; w[b][1] = d.w1; w[b][2] = d.w2; w[b][3] = d.w3;
  }
#pragma unroll
  for (int j = 0; j < 9; ++j) {
    const float noise = -0.1f + 0.2f * unit_float(w[j / 4][j % 4]);
    s.q[j] = (real)((j == 1 ? Z0 : 0.0f) + noise);
  }
#pragma unroll
  for (int pair = 0; pair < 5; ++pair) {
    const float u1 = unit_float_nonzero(w[3 + pair / 2][2 * (pair % 2)]);
    const float u2 = unit_float(w[3 + pair / 2][2 * (pair % 2) + 1]);
    const float radius = sqrtf(-2.0f * logf(u1));
    const float angle = 6.283185307179586f * u2;
    s.v[2 * pair] = (real)(0.1f * (radius * cosf(angle)));
    if (2 * pair + 1 < 9) s.v[2 * pair + 1] = (real)(0.1f * (radius * sinf(angle)));
  }
  s.ep_ret = 0.0f;
  s.ep_len = 0;
}

__device__ __forceinline__ void body_store(uint32_t* __restrict__ state, int64_t n, int64_t i, const BodyLane& s) {
#pragma unroll
  for (int j = 0; j < 9; ++j) {
    state[(int64_t)j * n + i] = __float_as_uint((float)s.q[j]);
    state[(int64_t)(9 + j) * n + i] = __float_as_uint((float)s.v[j]);
  }
  state[18 * n + i] = __float_as_uint(s.ep_ret);
  state[19 * n + i] = (uint32_t)s.ep_len;
}

__device__ __forceinline__ void body_observe(float* __restrict__ o, const BodyLane& s) {
#pragma unroll
  for (int j = 1; j < 9; ++j) o[j - 1] = (float)s.q[j];
#pragma unroll
  for (int j = 0; j < 9; ++j) o[8 + j] = (float)s.v[j];
}

__device__ __forceinline__ bool finite32(float x) { return (__float_as_uint(x) & 0x7f800000u) != 0x7f800000u; }

__global__ __launch_bounds__(256) void body_reset_kernel(uint32_t* __restrict__ state, int64_t n, uint64_t seed,
                                                         uint64_t host_step,
                                                         const StepCounter* __restrict__ counter,
                                                         float* __restrict__ obs) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint64_t step = read_step(counter, host_step);
  BodyLane s;
  body_initial(s, seed, (uint32_t)i, step);
  body_store(state, n, i, s);
  if (obs) body_observe(obs + i * BODY_OBS, s);
}

// ---- two lanes per environment ---------------------------------------------------------------------
// Lane 2i holds the root and the back leg of environment i, lane 2i+1 the root and the front leg.
// Each lane builds its own leg's terms and factor; whatever the 3x3 root system needs from both legs
// (mass, right-hand side, Schur complement) is the sum of a lane's part and its neighbour's, fetched
// with one DPP quad permutation per 32-bit half; the root system itself is solved twice, once per
// lane, on identical numbers (x + y and y + x round alike).  Per lane this is about 0.6 of the
// instructions a single lane per environment would need, which is what counts when a launch has
// fewer wavefronts than the device has SIMDs (N = 8192: 1.7x faster with the penalty model, 2.0x with
// the Newton model), and it costs nothing at large N (fewer registers, two wavefronts per SIMD).

__device__ __forceinline__ real pair_other(real x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xF, 0xF, true);      // quad_perm [1, 0, 3, 2]
  hi = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ real pair_sum(real x) { return x + pair_other(x); }
__device__ __forceinline__ int pair_other_int(int x) { return __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, true); }

struct PairLane {
  real qr[3], vr[3];        // x, z, pitch and their rates (the same numbers in both lanes)
  real jq[3], jv[3];        // this lane's leg
  float ep_ret;
  int ep_len;
};

// Solve the 9x9 system of one environment across its two lanes.  B = this lane's leg blocks, R = the
// whole root block, b_root = the whole root right-hand side, b_leg = this leg's.
template <class Block>
__device__ __forceinline__ void solve_pair(const Block& B, const RootBlock& R, const bool keep[3],
                                           const real b_root[3], const real b_leg[3], real x_root[3],
                                           real x_leg[3]) {
  LegFactor f;
  factor_leg(f, B, keep);
  real bl[3], y[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) bl[k] = keep[k] ? b_leg[k] : 0.0;
  forward_leg(f, bl, y);
  real s[3][3] = {{R.xx, R.xz, R.xth}, {R.xz, R.zz, R.zth}, {R.xth, R.zth, R.thth}};
  real br[3];
#pragma unroll
  for (int r = 0; r < 3; ++r) {
#pragma unroll
    for (int c = 0; c <= r; ++c) {
      real acc = 0.0;
#pragma unroll
      for (int k = 0; k < 3; ++k) acc += f.Y[k][r] * f.Y[k][c];
      s[r][c] -= pair_sum(acc);
    }
    real acc = 0.0;
#pragma unroll
    for (int k = 0; k < 3; ++k) acc += f.Y[k][r] * y[k];
    br[r] = b_root[r] - pair_sum(acc);
  }
  const real i00 = inv_sqrt(s[0][0]);
  const real l10 = s[1][0] * i00, l20 = s[2][0] * i00;
  const real i11 = inv_sqrt(s[1][1] - l10 * l10);
  const real l21 = (s[2][1] - l20 * l10) * i11;
  const real i22 = inv_sqrt(s[2][2] - l20 * l20 - l21 * l21);
  const real y0 = br[0] * i00;
  const real y1 = (br[1] - l10 * y0) * i11;
  const real y2 = (br[2] - l20 * y0 - l21 * y1) * i22;
  x_root[2] = y2 * i22;
  x_root[1] = (y1 - l21 * x_root[2]) * i11;
  x_root[0] = (y0 - l10 * x_root[1] - l20 * x_root[2]) * i00;
  backward_leg(f, y, x_root, x_leg);
}

// One substep in place, penalty contact model.  sign: -1 back leg, +1 front leg; a[3]: this leg's
// clipped actions.
__device__ __forceinline__ void pair_substep(PairLane& s, const real sign, const real a[3], const Params& P) {
  real st, ct;
  sincos_any(s.qr[2], st, ct);
  Leg g;
  LegRows unused;
  leg_terms<false>(g, unused, sign, st, ct, s.qr[1], s.vr[0], s.vr[1], s.vr[2], s.jq, s.jv, P);
  const real mxth = pair_sum(g.Pth.x), mzth = pair_sum(g.Pth.z);
  const real mthth = IT + pair_sum(g.mthth);
  const RootBlock R = {MTOT, 0.0, mxth, MTOT, mzth, mthth};

  // b = M v + h * rhs
  const real vx = s.vr[0], vz = s.vr[1], vth = s.vr[2];
  real cx = 0.0, cz = 0.0, cth = 0.0;
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    cx += g.C[0][m] * s.jv[m];
    cz += g.C[1][m] * s.jv[m];
    cth += g.C[2][m] * s.jv[m];
  }
  real b_root[3], b_leg[3];
  b_root[0] = MTOT * vx + mxth * vth + pair_sum(cx) + STEP_H * pair_sum(g.rhs_x);
  b_root[1] = MTOT * vz + mzth * vth + pair_sum(cz) + STEP_H * (-GRAVITY * MTOT + pair_sum(g.rhs_z));
  b_root[2] = mxth * vx + mzth * vz + mthth * vth + pair_sum(cth) + STEP_H * pair_sum(g.rhs_th);
  const int sym[3][3] = {{0, 1, 2}, {1, 3, 4}, {2, 4, 5}};
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    real mv = g.C[0][m] * vx + g.C[1][m] * vz + g.C[2][m] * vth;
#pragma unroll
    for (int k = 0; k < 3; ++k) mv += g.A[sym[m][k]] * s.jv[k];
    b_leg[m] = mv + STEP_H * (g.rhs[m] + GEAR * a[m] - P.damping * s.jv[m]);
  }

  const bool all[3] = {true, true, true};
  real x_root[3], x_leg[3];
  solve_pair(g, R, all, b_root, b_leg, x_root, x_leg);
  bool keep[3];
#pragma unroll
  for (int m = 0; m < 3; ++m)
    keep[m] = !((s.jq[m] >= 1.0 && x_leg[m] > 0.0) || (s.jq[m] <= -1.0 && x_leg[m] < 0.0));
  // the wavefront skips the second solve only when no lane has a joint to freeze; an environment
  // with nothing to freeze gets the same numbers again
  if (__ballot(!(keep[0] && keep[1] && keep[2])) != 0ull) solve_pair(g, R, keep, b_root, b_leg, x_root, x_leg);

#pragma unroll
  for (int m = 0; m < 3; ++m) {
    s.vr[m] = x_root[m];
    s.jv[m] = x_leg[m];
    s.qr[m] = s.qr[m] + STEP_H * s.vr[m];
    const real q = s.jq[m] + STEP_H * s.jv[m];
    s.jq[m] = q < -1.0 ? -1.0 : (q > 1.0 ? 1.0 : q);
  }
}

// One substep in place, Newton contact model.
template <bool SKIP_IDLE_ROWS>
__device__ __forceinline__ void pair_substep_newton(PairLane& s, const real sign, const real a[3],
                                                    const Params& P) {
  real st, ct;
  sincos_any(s.qr[2], st, ct);
  Leg g;
  LegRows rows;
  leg_terms<true>(g, rows, sign, st, ct, s.qr[1], s.vr[0], s.vr[1], s.vr[2], s.jq, s.jv, P);
  const RootBlock R0 = {MTOT, 0.0, pair_sum(g.Pth.x), MTOT, pair_sum(g.Pth.z), IT + pair_sum(g.mthth)};
  real f_root[3], f_leg[3];
  f_root[0] = pair_sum(g.rhs_x);
  f_root[1] = -GRAVITY * MTOT + pair_sum(g.rhs_z);
  f_root[2] = pair_sum(g.rhs_th);
#pragma unroll
  for (int m = 0; m < 3; ++m) f_leg[m] = g.rhs[m] + GEAR * a[m] - P.damping * s.jv[m];
  const bool all[3] = {true, true, true};
  real x_root[3], x_leg[3];
  solve_pair(g, R0, all, f_root, f_leg, x_root, x_leg);

  uint32_t prev = 0;
  for (int pass = 0; pass < NEWTON_MAX_PASSES; ++pass) {
    const uint32_t set = leg_active_set(g, rows, s.jq, s.jv, x_root, x_leg, P);
    if (__ballot(set != prev) == 0ull) break;
    LegBlock B;
#pragma unroll
    for (int k = 0; k < 6; ++k) B.A[k] = g.A[k];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int c = 0; c < 3; ++c) B.C[r][c] = g.C[r][c];
    RootBlock dR = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
    real dg_root[3] = {0.0, 0.0, 0.0}, g_leg[3] = {f_leg[0], f_leg[1], f_leg[2]};
    leg_add_rows<SKIP_IDLE_ROWS>(g, rows, s.jq, s.jv, set, P, B, dR, dg_root, g_leg);
    const RootBlock R = {R0.xx + pair_sum(dR.xx), R0.xz + pair_sum(dR.xz), R0.xth + pair_sum(dR.xth),
                         R0.zz + pair_sum(dR.zz), R0.zth + pair_sum(dR.zth), R0.thth + pair_sum(dR.thth)};
    real g_root[3];
#pragma unroll
    for (int m = 0; m < 3; ++m) g_root[m] = f_root[m] + pair_sum(dg_root[m]);
    solve_pair(B, R, all, g_root, g_leg, x_root, x_leg);
    prev = set;
  }

#pragma unroll
  for (int m = 0; m < 3; ++m) {
    s.vr[m] = s.vr[m] + STEP_H * x_root[m];
    s.jv[m] = s.jv[m] + STEP_H * x_leg[m];
    s.qr[m] = s.qr[m] + STEP_H * s.vr[m];
    const real q = s.jq[m] + STEP_H * s.jv[m];
    s.jq[m] = q < -1.0 ? -1.0 : (q > 1.0 ? 1.0 : q);
  }
}

__device__ __forceinline__ void pair_from_full(PairLane& p, const BodyLane& s, const int side) {
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    p.qr[m] = s.q[m]; p.vr[m] = s.v[m];
    p.jq[m] = side ? s.q[6 + m] : s.q[3 + m];
    p.jv[m] = side ? s.v[6 + m] : s.v[3 + m];
  }
  p.ep_ret = s.ep_ret; p.ep_len = s.ep_len;
}

template <bool NEWTON, bool SKIP_IDLE_ROWS>
__global__ __launch_bounds__(WAVE) __attribute__((amdgpu_waves_per_eu(2, 2))) void body_rollout_kernel(BodyLaunch a) {
  a.step0 = launch_first_step(a.counter, a.step0, a.T, a.ticket != 0);
  const int64_t n = a.n;
  const int side = threadIdx.x & 1;
  const real sign = side ? 1.0 : -1.0;
  const int64_t i = (int64_t)blockIdx.x * a.envs_per_wave + (threadIdx.x >> 1);
  const bool live = (int)(threadIdx.x >> 1) < a.envs_per_wave && i < n;
  // idle lane pairs shadow the wavefront's first environment: they add nothing to its ballots
  const int64_t ic = live ? i : (int64_t)blockIdx.x * a.envs_per_wave;
  const Params P = {(real)a.armature, (real)a.joint_damping, (real)a.friction_mu,
                    1.0 / NEWTON_REG_CONTACT, 1.0 / NEWTON_REG_LIMIT,
                    1.0 / (NEWTON_TIME_CONST * NEWTON_TIME_CONST), 2.0 / NEWTON_TIME_CONST};
  const int jbase = 3 + 3 * side;                  // first joint field of this lane's leg
  PairLane s;
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    s.qr[m] = (real)__uint_as_float(a.state[(int64_t)m * n + ic]);
    s.vr[m] = (real)__uint_as_float(a.state[(int64_t)(9 + m) * n + ic]);
    s.jq[m] = (real)__uint_as_float(a.state[(int64_t)(jbase + m) * n + ic]);
    s.jv[m] = (real)__uint_as_float(a.state[(int64_t)(9 + jbase + m) * n + ic]);
  }
  s.ep_ret = __uint_as_float(a.state[18 * n + ic]);
  s.ep_len = (int)a.state[19 * n + ic];
  LaneEpisodes le;
  const bool writer = live && side == 0;           // one lane per environment reports and counts

  for (int32_t t = 0; t < a.T; ++t) {
    const uint64_t step = a.step0 + (uint64_t)t;
    real act[3];
    if (a.actions) {
      const float* src = a.actions + ((int64_t)t * n + ic) * BODY_ACT + 3 * side;
#pragma unroll
      for (int m = 0; m < 3; ++m) act[m] = (real)src[m];
    } else {
      const Draw4 d0 = philox_draw(a.seed, (uint32_t)ic, step, 0u);
      const Draw4 d1 = philox_draw(a.seed, (uint32_t)ic, step, 1u);
      act[0] = (real)(-1.0f + 2.0f * unit_float(side ? d0.w3 : d0.w0));
      act[1] = (real)(-1.0f + 2.0f * unit_float(side ? d1.w0 : d0.w1));
      act[2] = (real)(-1.0f + 2.0f * unit_float(side ? d1.w1 : d0.w2));
    }
    real cost = 0.0;
#pragma unroll
    for (int m = 0; m < 3; ++m) {
      act[m] = act[m] < -1.0 ? -1.0 : (act[m] > 1.0 ? 1.0 : act[m]);
      cost += act[m] * act[m];
    }
    cost = pair_sum(cost);
    real vx_sum = 0.0;
    for (int sub = 0; sub < SUBSTEPS; ++sub) {
      if (NEWTON) pair_substep_newton<SKIP_IDLE_ROWS>(s, sign, act, P);
      else pair_substep(s, sign, act, P);
      vx_sum += s.vr[0];
    }
    float reward = (float)(vx_sum / (real)SUBSTEPS - 0.1 * cost);
    // the state lives in memory as float32: round here so that T fused steps equal T launches
    bool ok = finite32(reward);
#pragma unroll
    for (int m = 0; m < 3; ++m) {
      const float a0 = (float)s.qr[m], a1 = (float)s.vr[m], a2 = (float)s.jq[m], a3 = (float)s.jv[m];
      ok = ok && finite32(a0) && finite32(a1) && finite32(a2) && finite32(a3);
      s.qr[m] = (real)a0; s.vr[m] = (real)a1; s.jq[m] = (real)a2; s.jv[m] = (real)a3;
    }
    ok = ok && (pair_other_int(ok ? 1 : 0) != 0);     // both legs of the environment
    bool done = false;
    if (!ok) {                       // left the finite range: count it, start over
      reward = 0.0f;
      done = true;
      if (writer) le.nonfinite += 1;
      BodyLane fresh;
      body_initial(fresh, a.seed, (uint32_t)ic, step + 1);
      pair_from_full(s, fresh, side);
    } else {
      s.ep_ret += reward;
      s.ep_len += 1;
      if (s.ep_len >= a.max_episode_steps) {
        done = true;
        if (writer) {
          le.count += 1; le.length_sum += s.ep_len; le.ret_sum_f += s.ep_ret;
          const int key = float_order_key(s.ep_ret);
          le.min_key = min(le.min_key, key); le.max_key = max(le.max_key, key);
        }
        BodyLane fresh;
        body_initial(fresh, a.seed, (uint32_t)ic, step + 1);
        pair_from_full(s, fresh, side);
      }
    }
    if (live) {
      float* o = a.obs + ((int64_t)t * n + i) * BODY_OBS;
      // obs = (z, pitch, back joints, front joints | vx, vz, vpitch, back rates, front rates)
#pragma unroll
      for (int m = 0; m < 3; ++m) {
        o[2 + 3 * side + m] = (float)s.jq[m];
        o[11 + 3 * side + m] = (float)s.jv[m];
      }
      if (side == 0) {
        o[0] = (float)s.qr[1]; o[1] = (float)s.qr[2];
        o[8] = (float)s.vr[0]; o[9] = (float)s.vr[1]; o[10] = (float)s.vr[2];
        a.reward[(int64_t)t * n + i] = reward;
        a.done[(int64_t)t * n + i] = done ? 1 : 0;
      }
    }
  }
  if (live) {
#pragma unroll
    for (int m = 0; m < 3; ++m) {
      a.state[(int64_t)(jbase + m) * n + i] = __float_as_uint((float)s.jq[m]);
      a.state[(int64_t)(9 + jbase + m) * n + i] = __float_as_uint((float)s.jv[m]);
    }
    if (side == 0) {
#pragma unroll
      for (int m = 0; m < 3; ++m) {
        a.state[(int64_t)m * n + i] = __float_as_uint((float)s.qr[m]);
        a.state[(int64_t)(9 + m) * n + i] = __float_as_uint((float)s.vr[m]);
      }
      a.state[18 * n + i] = __float_as_uint(s.ep_ret);
      a.state[19 * n + i] = (uint32_t)s.ep_len;
    }
  }
  flush_wave_stats<true>(a.stats, le);
}

}  // namespace

hipError_t launch_body_reset(uint32_t* state, int64_t n, uint64_t seed, uint64_t step,
                             const StepCounter* counter, float* obs, hipStream_t stream) {
  hipLaunchKernelGGL(body_reset_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, state, n,
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
  if (a.newton && a.n >= 32768) hipLaunchKernelGGL((body_rollout_kernel<true, true>), grid, dim3(WAVE), 0, stream, a2);
  else if (a.newton) hipLaunchKernelGGL((body_rollout_kernel<true, false>), grid, dim3(WAVE), 0, stream, a2);
  else hipLaunchKernelGGL((body_rollout_kernel<false, false>), grid, dim3(WAVE), 0, stream, a2);
  const hipError_t err = hipGetLastError();
  return err != hipSuccess ? err : advance_step_counter_behind(a.counter, a.T, grid.x, stream);
}

}  // namespace envk
