// Planar articulated body ("HalfCheetah-like", paper App. A.1: forward kinematics, mass matrix,
// bias forces, contact Jacobians, Cholesky; first solver revision = penalty spring): reset and the
// fused T-step rollout (T = 1 is env_step).  One lane per environment, everything in registers.
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
  real z[4];                 // height of hip, knee, ankle, toe (rows exist iff < 0)
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
      rows.z[k] = zs[k];
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

// Solve the 9x9 system with the joints in `keep` (others: v = 0).  R = root block
// (Mtot, Mtot, m_xth, m_zth, m_thth); b = right-hand side (root 3, back 3, front 3).
struct RootBlock { real xx, xz, xth, zz, zth, thth; };

template <class Block>
__device__ __forceinline__ void solve_system(const Block& gb, const Block& gf, const RootBlock& R,
                                             const bool keep_b[3], const bool keep_f[3],
                                             const real b_root[3], const real b_back[3], const real b_front[3],
                                             real x_root[3], real x_back[3], real x_front[3]) {
  LegFactor fb, ff;
  factor_leg(fb, gb, keep_b);
  factor_leg(ff, gf, keep_f);
  real bb[3], bf[3], yb[3], yf[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) { bb[k] = keep_b[k] ? b_back[k] : 0.0; bf[k] = keep_f[k] ? b_front[k] : 0.0; }
  forward_leg(fb, bb, yb);
  forward_leg(ff, bf, yf);
  // Schur complement of the root block (symmetric 3x3: xx xz xth zz zth thth)
  real s[3][3] = {{R.xx, R.xz, R.xth}, {R.xz, R.zz, R.zth}, {R.xth, R.zth, R.thth}};
  real br[3];
#pragma unroll
  for (int r = 0; r < 3; ++r) {
#pragma unroll
    for (int c = 0; c <= r; ++c) {
      real acc = 0.0;
#pragma unroll
      for (int k = 0; k < 3; ++k) acc += fb.Y[k][r] * fb.Y[k][c] + ff.Y[k][r] * ff.Y[k][c];
      s[r][c] -= acc;
    }
    real acc = 0.0;
#pragma unroll
    for (int k = 0; k < 3; ++k) acc += fb.Y[k][r] * yb[k] + ff.Y[k][r] * yf[k];
    br[r] = b_root[r] - acc;
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
  backward_leg(fb, yb, x_root, x_back);
  backward_leg(ff, yf, x_root, x_front);
}

struct BodyLane {
  real q[9], v[9];
  float ep_ret;
  int ep_len;
};

// One substep in place.  a[6]: clipped actions.
__device__ __forceinline__ void body_substep(BodyLane& s, const real a[6], const Params& P) {
  real st, ct;
  sincos(s.q[2], &st, &ct);
  Leg gb, gf;
  LegRows unused;
  leg_terms<false>(gb, unused, -1.0, st, ct, s.q[1], s.v[0], s.v[1], s.v[2], &s.q[3], &s.v[3], P);
  leg_terms<false>(gf, unused, +1.0, st, ct, s.q[1], s.v[0], s.v[1], s.v[2], &s.q[6], &s.v[6], P);
  const real mxth = gb.Pth.x + gf.Pth.x, mzth = gb.Pth.z + gf.Pth.z;
  const real mthth = IT + gb.mthth + gf.mthth;
  const RootBlock R = {MTOT, 0.0, mxth, MTOT, mzth, mthth};

  // b = M v + h * rhs
  real b_root[3], b_back[3], b_front[3];
  const real vx = s.v[0], vz = s.v[1], vth = s.v[2];
  real mv_x = MTOT * vx + mxth * vth, mv_z = MTOT * vz + mzth * vth;
  real mv_th = mxth * vx + mzth * vz + mthth * vth;
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    mv_x += gb.C[0][m] * s.v[3 + m] + gf.C[0][m] * s.v[6 + m];
    mv_z += gb.C[1][m] * s.v[3 + m] + gf.C[1][m] * s.v[6 + m];
    mv_th += gb.C[2][m] * s.v[3 + m] + gf.C[2][m] * s.v[6 + m];
  }
  b_root[0] = mv_x + STEP_H * (gb.rhs_x + gf.rhs_x);
  b_root[1] = mv_z + STEP_H * (-GRAVITY * MTOT + gb.rhs_z + gf.rhs_z);
  b_root[2] = mv_th + STEP_H * (gb.rhs_th + gf.rhs_th);
  const int sym[3][3] = {{0, 1, 2}, {1, 3, 4}, {2, 4, 5}};
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    real mb = gb.C[0][m] * vx + gb.C[1][m] * vz + gb.C[2][m] * vth;
    real mf = gf.C[0][m] * vx + gf.C[1][m] * vz + gf.C[2][m] * vth;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
      mb += gb.A[sym[m][k]] * s.v[3 + k];
      mf += gf.A[sym[m][k]] * s.v[6 + k];
    }
    b_back[m] = mb + STEP_H * (gb.rhs[m] + GEAR * a[m] - P.damping * s.v[3 + m]);
    b_front[m] = mf + STEP_H * (gf.rhs[m] + GEAR * a[3 + m] - P.damping * s.v[6 + m]);
  }

  // unconstrained velocity, then the joints to freeze, then the projected velocity
  const bool all[3] = {true, true, true};
  real x_root[3], x_back[3], x_front[3];
  solve_system(gb, gf, R, all, all, b_root, b_back, b_front, x_root, x_back, x_front);
  bool keep_b[3], keep_f[3];
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    keep_b[m] = !((s.q[3 + m] >= 1.0 && x_back[m] > 0.0) || (s.q[3 + m] <= -1.0 && x_back[m] < 0.0));
    keep_f[m] = !((s.q[6 + m] >= 1.0 && x_front[m] > 0.0) || (s.q[6 + m] <= -1.0 && x_front[m] < 0.0));
  }
  // lanes with nothing to freeze get the same numbers again; the wavefront skips the second solve
  // only when no lane needs it
  const bool any_frozen = !(keep_b[0] && keep_b[1] && keep_b[2] && keep_f[0] && keep_f[1] && keep_f[2]);
  if (__ballot(any_frozen) != 0ull)
    solve_system(gb, gf, R, keep_b, keep_f, b_root, b_back, b_front, x_root, x_back, x_front);

#pragma unroll
  for (int m = 0; m < 3; ++m) {
    s.v[m] = x_root[m]; s.v[3 + m] = x_back[m]; s.v[6 + m] = x_front[m];
  }
#pragma unroll
  for (int j = 0; j < 9; ++j) s.q[j] = s.q[j] + STEP_H * s.v[j];
#pragma unroll
  for (int j = 3; j < 9; ++j) s.q[j] = s.q[j] < -1.0 ? -1.0 : (s.q[j] > 1.0 ? 1.0 : s.q[j]);
}


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
    set |= (rows.z[k] < 0.0 && r < 0.0) ? (1u << (2 * k + e)) : 0u;
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
__device__ __forceinline__ void leg_add_rows(const Leg& g, const LegRows& rows, const real* jq, const real* jv,
                                             const uint32_t set, const Params& P, LegBlock& B, RootBlock& R,
                                             real g_root[3], real g_leg[3]) {
  const int sym[3][3] = {{0, 1, 2}, {1, 3, 4}, {2, 4, 5}};
  for_each_contact_row(g, P.mu, [&](auto depth, int k, int e, real smu, real t, const real* u) {
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

// One substep in place, Newton contact model.  a[6]: clipped actions.
__device__ __forceinline__ void body_substep_newton(BodyLane& s, const real a[6], const Params& P) {
  real st, ct;
  sincos(s.q[2], &st, &ct);
  Leg gb, gf;
  LegRows rb, rf;
  leg_terms<true>(gb, rb, -1.0, st, ct, s.q[1], s.v[0], s.v[1], s.v[2], &s.q[3], &s.v[3], P);
  leg_terms<true>(gf, rf, +1.0, st, ct, s.q[1], s.v[0], s.v[1], s.v[2], &s.q[6], &s.v[6], P);
  const RootBlock R0 = {MTOT, 0.0, gb.Pth.x + gf.Pth.x, MTOT, gb.Pth.z + gf.Pth.z, IT + gb.mthth + gf.mthth};

  // generalised force without constraints: f = M a0
  real f_root[3], f_back[3], f_front[3];
  f_root[0] = gb.rhs_x + gf.rhs_x;
  f_root[1] = -GRAVITY * MTOT + gb.rhs_z + gf.rhs_z;
  f_root[2] = gb.rhs_th + gf.rhs_th;
#pragma unroll
  for (int m = 0; m < 3; ++m) {
    f_back[m] = gb.rhs[m] + GEAR * a[m] - P.damping * s.v[3 + m];
    f_front[m] = gf.rhs[m] + GEAR * a[3 + m] - P.damping * s.v[6 + m];
  }
  const bool all[3] = {true, true, true};
  real x_root[3], x_back[3], x_front[3];
  solve_system(gb, gf, R0, all, all, f_root, f_back, f_front, x_root, x_back, x_front);

  uint32_t prev = 0;
  for (int pass = 0; pass < NEWTON_MAX_PASSES; ++pass) {
    const uint32_t set = leg_active_set(gb, rb, &s.q[3], &s.v[3], x_root, x_back, P) |
                         (leg_active_set(gf, rf, &s.q[6], &s.v[6], x_root, x_front, P) << 16);
    // pass 0 compares with the empty set: no row active = the unconstrained acceleration stands
    if (__ballot(set != prev) == 0ull) break;
    LegBlock Bb, Bf;
#pragma unroll
    for (int k = 0; k < 6; ++k) { Bb.A[k] = gb.A[k]; Bf.A[k] = gf.A[k]; }
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int c = 0; c < 3; ++c) { Bb.C[r][c] = gb.C[r][c]; Bf.C[r][c] = gf.C[r][c]; }
    RootBlock R = R0;
    real g_root[3], g_back[3], g_front[3];
#pragma unroll
    for (int m = 0; m < 3; ++m) { g_root[m] = f_root[m]; g_back[m] = f_back[m]; g_front[m] = f_front[m]; }
    leg_add_rows(gb, rb, &s.q[3], &s.v[3], set & 0xffffu, P, Bb, R, g_root, g_back);
    leg_add_rows(gf, rf, &s.q[6], &s.v[6], set >> 16, P, Bf, R, g_root, g_front);
    solve_system(Bb, Bf, R, all, all, g_root, g_back, g_front, x_root, x_back, x_front);
    prev = set;
  }

#pragma unroll
  for (int m = 0; m < 3; ++m) {
    s.v[m] = s.v[m] + STEP_H * x_root[m];
    s.v[3 + m] = s.v[3 + m] + STEP_H * x_back[m];
    s.v[6 + m] = s.v[6 + m] + STEP_H * x_front[m];
  }
#pragma unroll
  for (int j = 0; j < 9; ++j) s.q[j] = s.q[j] + STEP_H * s.v[j];
#pragma unroll
  for (int j = 3; j < 9; ++j) s.q[j] = s.q[j] < -1.0 ? -1.0 : (s.q[j] > 1.0 ? 1.0 : s.q[j]);
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

__device__ __forceinline__ BodyLane body_load(const uint32_t* __restrict__ state, int64_t n, int64_t i) {
  BodyLane s;
#pragma unroll
  for (int j = 0; j < 9; ++j) {
    s.q[j] = (real)__uint_as_float(state[(int64_t)j * n + i]);
    s.v[j] = (real)__uint_as_float(state[(int64_t)(9 + j) * n + i]);
  }
  s.ep_ret = __uint_as_float(state[18 * n + i]);
  s.ep_len = (int)state[19 * n + i];
  return s;
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

template <bool NEWTON>
__global__ __launch_bounds__(WAVE) void body_rollout_kernel(BodyLaunch a) {
  a.step0 = launch_first_step(a.counter, a.step0, a.T);
  const int64_t n = a.n;
  const int64_t i = (int64_t)blockIdx.x * WAVE + threadIdx.x;
  const bool live = i < n;
  const int64_t ic = live ? i : n - 1;             // idle lanes shadow the last environment
  const Params P = {(real)a.armature, (real)a.joint_damping, (real)a.friction_mu,
                    1.0 / NEWTON_REG_CONTACT, 1.0 / NEWTON_REG_LIMIT,
                    1.0 / (NEWTON_TIME_CONST * NEWTON_TIME_CONST), 2.0 / NEWTON_TIME_CONST};
  BodyLane s = body_load(a.state, n, ic);
  LaneEpisodes le;

  for (int32_t t = 0; t < a.T; ++t) {
    const uint64_t step = a.step0 + (uint64_t)t;
    real act[6];
    if (a.actions) {
      const float* src = a.actions + ((int64_t)t * n + ic) * BODY_ACT;
#pragma unroll
      for (int j = 0; j < 6; ++j) act[j] = (real)src[j];
    } else {
      const Draw4 d0 = philox_draw(a.seed, (uint32_t)ic, step, 0u);
      const Draw4 d1 = philox_draw(a.seed, (uint32_t)ic, step, 1u);
      act[0] = (real)(-1.0f + 2.0f * unit_float(d0.w0)); act[1] = (real)(-1.0f + 2.0f * unit_float(d0.w1));
      act[2] = (real)(-1.0f + 2.0f * unit_float(d0.w2)); act[3] = (real)(-1.0f + 2.0f * unit_float(d0.w3));
      act[4] = (real)(-1.0f + 2.0f * unit_float(d1.w0)); act[5] = (real)(-1.0f + 2.0f * unit_float(d1.w1));
    }
    real cost = 0.0;
#pragma unroll
    for (int j = 0; j < 6; ++j) {
      act[j] = act[j] < -1.0 ? -1.0 : (act[j] > 1.0 ? 1.0 : act[j]);
      cost += act[j] * act[j];
    }
    real vx_sum = 0.0;
    for (int sub = 0; sub < SUBSTEPS; ++sub) {
      if (NEWTON) body_substep_newton(s, act, P);
      else body_substep(s, act, P);
      vx_sum += s.v[0];
    }
    float reward = (float)(vx_sum / (real)SUBSTEPS - 0.1 * cost);
    // the state lives in memory as float32: round here so that T fused steps equal T launches
    bool ok = finite32(reward);
#pragma unroll
    for (int j = 0; j < 9; ++j) {
      const float qf = (float)s.q[j], vf = (float)s.v[j];
      ok = ok && finite32(qf) && finite32(vf);
      s.q[j] = (real)qf; s.v[j] = (real)vf;
    }
    bool done = false;
    if (!ok) {                       // left the finite range: count it, start over
      reward = 0.0f;
      done = true;
      if (live) le.nonfinite += 1;
      body_initial(s, a.seed, (uint32_t)ic, step + 1);
    } else {
      s.ep_ret += reward;
      s.ep_len += 1;
      if (s.ep_len >= a.max_episode_steps) {
        done = true;
        if (live) {
          le.count += 1; le.length_sum += s.ep_len; le.ret_sum_f += s.ep_ret;
          const int key = float_order_key(s.ep_ret);
          le.min_key = min(le.min_key, key); le.max_key = max(le.max_key, key);
        }
        body_initial(s, a.seed, (uint32_t)ic, step + 1);
      }
    }
    if (live) {
      body_observe(a.obs + ((int64_t)t * n + i) * BODY_OBS, s);
      a.reward[(int64_t)t * n + i] = reward;
      a.done[(int64_t)t * n + i] = done ? 1 : 0;
    }
  }
  if (live) body_store(a.state, n, i, s);
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
  const dim3 grid((unsigned)((a.n + WAVE - 1) / WAVE));
  if (a.newton) hipLaunchKernelGGL(body_rollout_kernel<true>, grid, dim3(WAVE), 0, stream, a);
  else hipLaunchKernelGGL(body_rollout_kernel<false>, grid, dim3(WAVE), 0, stream, a);
  return hipGetLastError();
}

}  // namespace envk
