// TEST INFRASTRUCTURE — CPU oracle. Not part of the product path; shares no code with the HIP library.
//
// Planar articulated body ("HalfCheetah-like"): 7 rigid links, 9 degrees of freedom, 6 actuated
// hinges, penalty ground contact.  The paper's case study (App. A.1 "HalfCheetah JAX": forward
// kinematics, mass matrix, bias forces, contact Jacobians, float32; first solver revision =
// penalty spring) names the ingredients; the numbers are the benchmark configuration's.
//
// The equations of motion are built the slow, obviously-right way (projection onto generalised
// coordinates): for every link i with centre of mass p_i(q), translational Jacobian J_i and
// angular Jacobian A_i,
//     M   = sum_i  m_i J_i^T J_i + I_i A_i^T A_i          (+ armature on the joint diagonal)
//     h   = sum_i  m_i J_i^T (dJ_i/dt qdot)               (A_i is constant in the plane)
//     Q_g = sum_i  J_i^T (0, -m_i g)
//     M qddot + h = Q_g + tau + sum_p J_p^T F_p.
//
// Model conventions (fixed here; the configuration gives only lengths, masses, gains):
//   q = (x, z, theta, b1, b2, b3, f1, f2, f3); (x, z) torso centre, theta torso pitch (CCW),
//   torso axis t = (cos theta, sin theta), back hip = c - t/2, front hip = c + t/2;
//   leg link k has absolute angle phi = theta + (joint angles down its chain) and points along
//   d(phi) = (sin phi, -cos phi) (straight down at 0); links are uniform thin rods
//   (centre of mass at the midpoint, I = m L^2 / 12); contact points = 2 hips, 2 knees, 2 ankles,
//   2 toes; gravity 9.81.
//
// One environment step = 5 substeps of h = 0.01 (semi-implicit Euler):
//   1. assemble M, h, Q_g, contact forces at (q, v);
//   2. v* = v + h M^-1 rhs                      (Cholesky)
//   3. joint limits +-1 rad: S = joints sitting at a limit and still moving outwards under v*;
//      v+ = M-orthogonal projection of v* onto {v_S = 0}: solve M_FF v_F = (M v + h rhs)_F;
//   4. q+ = q + h v+, joint angles clipped to [-1, 1].
//
// Second contact model (solver = 1), after the paper's final solver revision for this case study
// (App. A.1, "HalfCheetah JAX": a quadratic programme over accelerations, solved by Newton's method
// with Cholesky factorisations; the paper gives no formulas, so everything below is this
// repository's reading):
// the substep's acceleration a minimises the strictly convex, piecewise quadratic
//     c(a) = 1/2 (a - a0)^T M (a - a0)  +  sum_i  D_i / 2 * min(0, J_i a - aref_i)^2 ,
// a0 = M^-1 (Q_g + tau - h) being the acceleration without constraints (Gauss' principle with soft
// one-sided constraints).  Rows i, in this order:
//   * contact point p = 0..7 below the ground (z_p < 0): two rows, the edges of the friction
//     pyramid, J = J_z + mu J_x then J_z - mu J_x, row acceleration J a + (dJ/dt qdot), wanted
//     >= -b (J v) - k z_p, i.e. aref = -b (J v) - k z_p - (dJ/dt qdot);  D = 1 / reg_contact;
//   * joint j = 3..8 sitting at +1 (row -e_j) or -1 (row +e_j): aref = -b (J v);  D = 1 / reg_limit;
//   k = 1 / tc^2, b = 2 / tc (critically damped reference, tc = time_const = 0.02 s = 2 h).
// Solved by Newton's method on the active set (unit steps: the cost is quadratic on each set):
//   a <- a0;  repeat at most newton_iters times: S = {i : J_i a - aref_i < 0}; stop if S is the set
//   of the previous pass; a <- (M + sum_S D_i J_i^T J_i)^-1 (M a0 + sum_S D_i aref_i J_i)  (Cholesky).
// Then v+ = v + h a, q+ = q + h v+, joint angles clipped to [-1, 1] as before.  The constraint
// forces depend on the acceleration being solved for (implicit), which is what removes the
// stiffness limit of the explicit penalty spring.
//
// Everything is templated on the scalar type.  float64 serves the invariants and is the parity
// target of the single-step comparison (stepping from a float32 state; `round_state_f32` rounds the
// state back to the storage format after every step); float32 serves the long-rollout statistics
// and shows what float32 arithmetic alone would cost.  Build with -ffp-contract=off.
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

extern "C" {
void oracle_draw_block(uint64_t seed, uint32_t env, uint64_t step, uint32_t stream, uint32_t out[4]);
float oracle_u01(uint32_t w);
void oracle_normal_pair(uint32_t wa, uint32_t wb, float out[2]);
}

namespace {

const int NQ = 9, NLINK = 7, NPOINT = 8, NACT = 6;

// A point rigidly attached to the tree: c + hip_sign/2 * t(theta) + sum_k w[k] * d(phi_leg,k).
struct PointDesc { int leg; double hip_sign; double w[3]; };   // leg: -1 torso, 0 back, 1 front

const double L_THIGH = 0.29, L_SHIN = 0.30, L_FOOT = 0.19, L_TORSO = 1.0;
const double LINK_MASS[NLINK] = {6.4, 1.5, 1.2, 0.9, 1.5, 1.2, 0.9};
const double LINK_LEN[NLINK] = {L_TORSO, L_THIGH, L_SHIN, L_FOOT, L_THIGH, L_SHIN, L_FOOT};
// centres of mass: torso, back thigh/shin/foot, front thigh/shin/foot
const PointDesc LINK_COM[NLINK] = {
    {-1, 0.0, {0, 0, 0}},
    {0, -1.0, {L_THIGH / 2, 0, 0}}, {0, -1.0, {L_THIGH, L_SHIN / 2, 0}}, {0, -1.0, {L_THIGH, L_SHIN, L_FOOT / 2}},
    {1, +1.0, {L_THIGH / 2, 0, 0}}, {1, +1.0, {L_THIGH, L_SHIN / 2, 0}}, {1, +1.0, {L_THIGH, L_SHIN, L_FOOT / 2}}};
// how many joints of its leg rotate the link (torso: none)
const int LINK_DEPTH[NLINK] = {0, 1, 2, 3, 1, 2, 3};
// contact points: back hip, knee, ankle, toe; front hip, knee, ankle, toe
const PointDesc CONTACT[NPOINT] = {
    {0, -1.0, {0, 0, 0}}, {0, -1.0, {L_THIGH, 0, 0}}, {0, -1.0, {L_THIGH, L_SHIN, 0}}, {0, -1.0, {L_THIGH, L_SHIN, L_FOOT}},
    {1, +1.0, {0, 0, 0}}, {1, +1.0, {L_THIGH, 0, 0}}, {1, +1.0, {L_THIGH, L_SHIN, 0}}, {1, +1.0, {L_THIGH, L_SHIN, L_FOOT}}};

template <class R>
struct Params {
  R armature, joint_damping, friction_mu;
  R gravity, contact_k, contact_c, h, gear, z0;
  int substeps, max_episode_steps;
  int round_state_f32;   // round q, v, episode return to float32 after every step (the storage format)
  int solver;            // 0 penalty spring + limit projection, 1 Newton on the soft-constraint QP
  int newton_iters;
  R time_const, reg_contact, reg_limit;
};

template <class R>
struct Kin {        // position, Jacobian (2 x 9), velocity and dJ/dt qdot of one point
  R pos[2], J[2][NQ], vel[2], jdqd[2];
};

// Kinematics of one described point at (q, v).
template <class R>
void point_kinematics(const PointDesc& d, const R* q, const R* v, Kin<R>* k) {
  const R th = q[2];
  const R tx = std::cos(th), tz = std::sin(th);          // torso axis t; t_perp = (-tz, tx)
  for (int a = 0; a < 2; ++a) for (int j = 0; j < NQ; ++j) k->J[a][j] = 0;
  k->J[0][0] = 1; k->J[1][1] = 1;
  const R hs = (R)(d.hip_sign * 0.5 * L_TORSO);
  k->pos[0] = q[0] + hs * tx;
  k->pos[1] = q[1] + hs * tz;
  k->J[0][2] = hs * (-tz);
  k->J[1][2] = hs * tx;
  k->jdqd[0] = hs * (-tx) * v[2] * v[2];
  k->jdqd[1] = hs * (-tz) * v[2] * v[2];
  if (d.leg >= 0) {
    const int j0 = 3 + 3 * d.leg;                        // first joint coordinate of this leg
    R phi = th, phid = v[2];
    for (int s = 0; s < 3; ++s) {
      phi = phi + q[j0 + s];
      phid = phid + v[j0 + s];
      const R w = (R)d.w[s];
      if (w == 0) continue;
      const R sn = std::sin(phi), cs = std::cos(phi);    // d = (sn, -cs), e = dd/dphi = (cs, sn)
      k->pos[0] += w * sn;
      k->pos[1] += w * (-cs);
      // phi depends on theta and on joints 0..s of this leg
      k->J[0][2] += w * cs; k->J[1][2] += w * sn;
      for (int m = 0; m <= s; ++m) { k->J[0][j0 + m] += w * cs; k->J[1][j0 + m] += w * sn; }
      // d/dt (e phid) at qddot = 0 is de/dphi phid^2 = (-sn, cs) phid^2 = -d phid^2
      k->jdqd[0] += w * (-sn) * phid * phid;
      k->jdqd[1] += w * cs * phid * phid;
    }
  }
  for (int a = 0; a < 2; ++a) {
    R s = 0;
    for (int j = 0; j < NQ; ++j) s += k->J[a][j] * v[j];
    k->vel[a] = s;
  }
}

// Angular Jacobian of link i: omega_i = A_i . qdot (entries 0 or 1).
void angular_jacobian(int link, int A[NQ]) {
  for (int j = 0; j < NQ; ++j) A[j] = 0;
  A[2] = 1;
  if (link >= 1) {
    const int leg = (link - 1) / 3, depth = LINK_DEPTH[link];
    for (int m = 0; m < depth; ++m) A[3 + 3 * leg + m] = 1;
  }
}

template <class R>
void mass_matrix(const Params<R>& P, const R* q, R M[NQ][NQ]) {
  R zero_v[NQ] = {0};
  for (int a = 0; a < NQ; ++a) for (int b = 0; b < NQ; ++b) M[a][b] = 0;
  for (int i = 0; i < NLINK; ++i) {
    Kin<R> k;
    point_kinematics(LINK_COM[i], q, zero_v, &k);
    int A[NQ];
    angular_jacobian(i, A);
    const R m = (R)LINK_MASS[i];
    const R I = (R)(LINK_MASS[i] * LINK_LEN[i] * LINK_LEN[i] / 12.0);
    for (int a = 0; a < NQ; ++a)
      for (int b = 0; b < NQ; ++b)
        M[a][b] += m * (k.J[0][a] * k.J[0][b] + k.J[1][a] * k.J[1][b]) + I * (R)(A[a] * A[b]);
  }
  for (int j = 3; j < NQ; ++j) M[j][j] += P.armature;
}

// bias (velocity-product) forces h and gravity generalised forces Q_g
template <class R>
void bias_and_gravity(const Params<R>& P, const R* q, const R* v, R h[NQ], R Qg[NQ]) {
  for (int j = 0; j < NQ; ++j) { h[j] = 0; Qg[j] = 0; }
  for (int i = 0; i < NLINK; ++i) {
    Kin<R> k;
    point_kinematics(LINK_COM[i], q, v, &k);
    const R m = (R)LINK_MASS[i];
    for (int j = 0; j < NQ; ++j) {
      h[j] += m * (k.J[0][j] * k.jdqd[0] + k.J[1][j] * k.jdqd[1]);
      Qg[j] += k.J[1][j] * (-m * P.gravity);
    }
  }
}

// Penalty ground contact at the 8 points: normal spring-damper without adhesion, regularised
// Coulomb friction.  Adds J_p^T F_p to Q; optionally reports the forces per point.
template <class R>
void contact_forces(const Params<R>& P, const R* q, const R* v, R Q[NQ], R* forces /* [8][2] or null */) {
  for (int p = 0; p < NPOINT; ++p) {
    Kin<R> k;
    point_kinematics(CONTACT[p], q, v, &k);
    R fn = 0, ft = 0;
    if (k.pos[1] < 0) {
      fn = -P.contact_k * k.pos[1] - P.contact_c * k.vel[1];
      if (fn < 0) fn = 0;
      R want = P.contact_c * k.vel[0];
      const R cap = P.friction_mu * fn;
      if (want > cap) want = cap;
      if (want < -cap) want = -cap;
      ft = -want;
    }
    if (forces) { forces[2 * p] = ft; forces[2 * p + 1] = fn; }
    for (int j = 0; j < NQ; ++j) Q[j] += k.J[0][j] * ft + k.J[1][j] * fn;
  }
}

// Solve A x = b for symmetric positive definite A (Cholesky, lower factor); returns false if a
// pivot is not positive.
template <class R>
bool cholesky_solve(const R A[NQ][NQ], const R b[NQ], R x[NQ]) {
  R L[NQ][NQ];
  for (int i = 0; i < NQ; ++i) {
    for (int j = 0; j <= i; ++j) {
      R s = A[i][j];
      for (int k = 0; k < j; ++k) s -= L[i][k] * L[j][k];
      if (i == j) {
        if (!(s > 0)) return false;
        L[i][i] = std::sqrt(s);
      } else {
        L[i][j] = s / L[j][j];
      }
    }
  }
  R y[NQ];
  for (int i = 0; i < NQ; ++i) {
    R s = b[i];
    for (int k = 0; k < i; ++k) s -= L[i][k] * y[k];
    y[i] = s / L[i][i];
  }
  for (int i = NQ - 1; i >= 0; --i) {
    R s = y[i];
    for (int k = i + 1; k < NQ; ++k) s -= L[k][i] * x[k];
    x[i] = s / L[i][i];
  }
  return true;
}

template <class R>
void clip_actions(const R* a_in, R a[NACT]) {
  for (int j = 0; j < NACT; ++j) {
    R x = a_in[j];
    if (x < -1) x = -1;
    if (x > 1) x = 1;
    a[j] = x;
  }
}

// ---- Newton contact solver (solver = 1) -----------------------------------------------------------
const int MAXROW = 2 * NPOINT + NACT;

template <class R>
struct Rows { int m; R J[MAXROW][NQ]; R aref[MAXROW]; R D[MAXROW]; };

// Constraint rows at (q, v), in the order stated in the header.
template <class R>
void constraint_rows(const Params<R>& P, const R* q, const R* v, Rows<R>* rows) {
  const R k = (R)1 / (P.time_const * P.time_const), b = (R)2 / P.time_const;
  rows->m = 0;
  for (int p = 0; p < NPOINT; ++p) {
    Kin<R> kin;
    point_kinematics(CONTACT[p], q, v, &kin);
    if (!(kin.pos[1] < 0)) continue;
    for (int e = 0; e < 2; ++e) {
      const R smu = e == 0 ? P.friction_mu : -P.friction_mu;
      const int i = rows->m++;
      R jv = 0;
      for (int j = 0; j < NQ; ++j) {
        rows->J[i][j] = kin.J[1][j] + smu * kin.J[0][j];
        jv += rows->J[i][j] * v[j];
      }
      rows->aref[i] = -b * jv - k * kin.pos[1] - (kin.jdqd[1] + smu * kin.jdqd[0]);
      rows->D[i] = (R)1 / P.reg_contact;
    }
  }
  for (int j = 3; j < NQ; ++j) {
    R sign = 0;
    if (q[j] >= 1) sign = -1;
    else if (q[j] <= -1) sign = 1;
    if (sign == 0) continue;
    const int i = rows->m++;
    for (int c = 0; c < NQ; ++c) rows->J[i][c] = 0;
    rows->J[i][j] = sign;
    rows->aref[i] = -b * (sign * v[j]);
    rows->D[i] = (R)1 / P.reg_limit;
  }
}

struct NewtonInfo { int rows, passes, converged; uint32_t active; };

// Minimise c(a); f = M a0 (the generalised force without constraints).  Returns false if a
// factorisation fails.
template <class R>
bool newton_solve(const Params<R>& P, const R M[NQ][NQ], const R f[NQ], const Rows<R>& rows, R a[NQ],
                  NewtonInfo* info) {
  if (!cholesky_solve(M, f, a)) return false;
  uint32_t prev = 0;
  int passes = 0, converged = rows.m == 0;
  for (int it = 0; it < P.newton_iters && rows.m > 0; ++it) {
    uint32_t set = 0;
    for (int i = 0; i < rows.m; ++i) {
      R r = -rows.aref[i];
      for (int j = 0; j < NQ; ++j) r += rows.J[i][j] * a[j];
      if (r < 0) set |= 1u << i;
    }
    if (it > 0 && set == prev) { converged = 1; break; }
    if (it == 0 && set == 0) { converged = 1; prev = 0; break; }
    R Hm[NQ][NQ], g[NQ];
    for (int x = 0; x < NQ; ++x) {
      g[x] = f[x];
      for (int y = 0; y < NQ; ++y) Hm[x][y] = M[x][y];
    }
    for (int i = 0; i < rows.m; ++i) {
      if (!(set & (1u << i))) continue;
      for (int x = 0; x < NQ; ++x) {
        g[x] += rows.D[i] * rows.aref[i] * rows.J[i][x];
        for (int y = 0; y < NQ; ++y) Hm[x][y] += rows.D[i] * rows.J[i][x] * rows.J[i][y];
      }
    }
    if (!cholesky_solve(Hm, g, a)) return false;
    prev = set;
    ++passes;
  }
  if (info) { info->rows = rows.m; info->passes = passes; info->converged = converged; info->active = prev; }
  return true;
}

template <class R>
void smooth_force(const Params<R>& P, const R* q, const R* v, const R a[NACT], R M[NQ][NQ], R f[NQ]) {
  R hb[NQ];
  mass_matrix(P, q, M);
  bias_and_gravity(P, q, v, hb, f);                    // f = Q_g
  for (int j = 0; j < NQ; ++j) f[j] -= hb[j];
  for (int j = 0; j < NACT; ++j) f[3 + j] += P.gear * a[j] - P.joint_damping * v[3 + j];
}

template <class R>
bool substep_newton(const Params<R>& P, R* q, R* v, const R a[NACT], NewtonInfo* info) {
  R M[NQ][NQ], f[NQ], acc[NQ];
  smooth_force(P, q, v, a, M, f);
  Rows<R> rows;
  constraint_rows(P, q, v, &rows);
  if (!newton_solve(P, M, f, rows, acc, info)) return false;
  for (int j = 0; j < NQ; ++j) { v[j] = v[j] + P.h * acc[j]; q[j] = q[j] + P.h * v[j]; }
  for (int j = 3; j < NQ; ++j) {
    if (q[j] < -1) q[j] = -1;
    if (q[j] > 1) q[j] = 1;
  }
  return true;
}

// One substep; a[] already clipped.  limit_mask_out (optional): bit j set if joint j was projected.
// margin_io (optional, penalty model): lowered to the distance of this substep's closest decision
// from its switching surface -- |z_p| of the eight contact points (the force law changes at z = 0),
// 1 - |q_j| of the joints not sitting at a limit (the projection applies from |q_j| = 1 on), and
// |v*_j| of the joints that are (projected or not by the sign of v*_j).
template <class R>
bool substep(const Params<R>& P, R* q, R* v, const R a[NACT], int* limit_mask_out, R* margin_io = nullptr) {
  if (P.solver == 1) {
    if (limit_mask_out) *limit_mask_out = 0;
    return substep_newton(P, q, v, a, (NewtonInfo*)nullptr);
  }
  R M[NQ][NQ], hb[NQ], rhs[NQ];
  mass_matrix(P, q, M);
  bias_and_gravity(P, q, v, hb, rhs);                  // rhs = Q_g
  for (int j = 0; j < NQ; ++j) rhs[j] -= hb[j];
  for (int j = 0; j < NACT; ++j) rhs[3 + j] += P.gear * a[j] - P.joint_damping * v[3 + j];
  contact_forces(P, q, v, rhs, (R*)nullptr);
  // b = M v + h rhs, so that M v* = b
  R b[NQ];
  for (int i = 0; i < NQ; ++i) {
    R s = 0;
    for (int j = 0; j < NQ; ++j) s += M[i][j] * v[j];
    b[i] = s + P.h * rhs[i];
  }
  R vs[NQ];
  if (!cholesky_solve(M, b, vs)) return false;
  if (margin_io) {
    R m = *margin_io;
    for (int p = 0; p < NPOINT; ++p) {
      Kin<R> k;
      point_kinematics(CONTACT[p], q, v, &k);
      m = std::fmin(m, std::fabs(k.pos[1]));
    }
    for (int j = 3; j < NQ; ++j)
      m = std::fmin(m, (q[j] >= 1 || q[j] <= -1) ? std::fabs(vs[j]) : (R)1 - std::fabs(q[j]));
    *margin_io = m;
  }
  int mask = 0;
  for (int j = 3; j < NQ; ++j)
    if ((q[j] >= 1 && vs[j] > 0) || (q[j] <= -1 && vs[j] < 0)) mask |= 1 << j;
  if (mask) {
    for (int j = 3; j < NQ; ++j) {
      if (!(mask & (1 << j))) continue;
      for (int k = 0; k < NQ; ++k) { M[j][k] = 0; M[k][j] = 0; }
      M[j][j] = 1;
      b[j] = 0;
    }
    if (!cholesky_solve(M, b, vs)) return false;
  }
  for (int j = 0; j < NQ; ++j) { v[j] = vs[j]; q[j] = q[j] + P.h * vs[j]; }
  for (int j = 3; j < NQ; ++j) {
    if (q[j] < -1) q[j] = -1;
    if (q[j] > 1) q[j] = 1;
  }
  if (limit_mask_out) *limit_mask_out = mask;
  return true;
}

// Total mechanical energy: kinetic (1/2 v^T M v, armature included) + potential above the ground.
template <class R>
R energy(const Params<R>& P, const R* q, const R* v) {
  R M[NQ][NQ];
  mass_matrix(P, q, M);
  R T = 0;
  for (int i = 0; i < NQ; ++i) for (int j = 0; j < NQ; ++j) T += v[i] * M[i][j] * v[j];
  T = T / 2;
  R V = 0;
  R zero_v[NQ] = {0};
  for (int i = 0; i < NLINK; ++i) {
    Kin<R> k;
    point_kinematics(LINK_COM[i], q, zero_v, &k);
    V += (R)LINK_MASS[i] * P.gravity * k.pos[1];
  }
  return T + V;
}

template <class R>
struct Env {
  R q[NQ], v[NQ];
  R ep_ret;
  int32_t ep_len;
};

template <class R>
bool state_finite(const Env<R>& e) {
  for (int j = 0; j < NQ; ++j)
    if (!std::isfinite(e.q[j]) || !std::isfinite(e.v[j])) return false;
  return true;
}

// Initial state: q0 = (0, z0, 0, ...) + U[-0.1, 0.1), v0 = 0.1 N(0, 1); draws from reset streams
// 16..18 (uniforms, word order) and 19..21 (Box-Muller pairs), all in float32.
template <class R>
void reset_env(const Params<R>& P, Env<R>* e, uint64_t seed, uint32_t env, uint64_t step) {
  uint32_t w[6][4];
  for (int b = 0; b < 6; ++b) oracle_draw_block(seed, env, step, 16u + (uint32_t)b, w[b]);
  for (int j = 0; j < NQ; ++j) {
    const float u = oracle_u01(w[j / 4][j % 4]);
    const float noise = -0.1f + 0.2f * u;
    const float base = (j == 1) ? (float)P.z0 : 0.0f;
    e->q[j] = (R)(base + noise);
  }
  for (int pair = 0; pair < 5; ++pair) {
    float n2[2];
    oracle_normal_pair(w[3 + pair / 2][2 * (pair % 2)], w[3 + pair / 2][2 * (pair % 2) + 1], n2);
    for (int m = 0; m < 2; ++m) {
      const int j = 2 * pair + m;
      if (j < NQ) e->v[j] = (R)(0.1f * n2[m]);
    }
  }
  e->ep_ret = 0;
  e->ep_len = 0;
}

template <class R>
void observe(const Env<R>& e, R obs[17]) {
  for (int j = 1; j < NQ; ++j) obs[j - 1] = e.q[j];
  for (int j = 0; j < NQ; ++j) obs[8 + j] = e.v[j];
}

struct StepInfo { int done; int nonfinite; double fin_ret; int fin_len; };

// One environment step: 5 substeps, reward = mean forward velocity - 0.1 |a|^2, truncation at
// max_episode_steps with auto-reset, re-initialisation if the state leaves the finite range.
template <class R>
R env_step(const Params<R>& P, Env<R>* e, const R a_in[NACT], uint64_t seed, uint32_t env,
           uint64_t step, StepInfo* info) {
  R a[NACT];
  clip_actions(a_in, a);
  R vx_sum = 0;
  bool ok = true;
  for (int s = 0; s < P.substeps && ok; ++s) {
    ok = substep(P, e->q, e->v, a, (int*)nullptr);
    vx_sum += e->v[0];
  }
  R cost = 0;
  for (int j = 0; j < NACT; ++j) cost += a[j] * a[j];
  R reward = vx_sum / (R)P.substeps - (R)0.1 * cost;
  info->done = 0; info->nonfinite = 0; info->fin_ret = 0; info->fin_len = 0;
  if (!ok || !state_finite(*e) || !std::isfinite(reward)) {
    info->nonfinite = 1;
    info->done = 1;
    reward = 0;
    info->fin_ret = (double)e->ep_ret; info->fin_len = e->ep_len + 1;
    reset_env(P, e, seed, env, step + 1);
    return reward;
  }
  e->ep_ret += reward;
  e->ep_len += 1;
  if (P.round_state_f32) {
    for (int j = 0; j < NQ; ++j) { e->q[j] = (R)(float)e->q[j]; e->v[j] = (R)(float)e->v[j]; }
    e->ep_ret = (R)(float)e->ep_ret;
    reward = (R)(float)reward;
  }
  if (e->ep_len >= P.max_episode_steps) {
    info->done = 1;
    info->fin_ret = (double)e->ep_ret; info->fin_len = e->ep_len;
    reset_env(P, e, seed, env, step + 1);
  }
  return reward;
}

template <class R>
void draw_actions(uint64_t seed, uint32_t env, uint64_t step, R a[NACT]) {
  uint32_t w0[4], w1[4];
  oracle_draw_block(seed, env, step, 0u, w0);
  oracle_draw_block(seed, env, step, 1u, w1);
  for (int j = 0; j < 4; ++j) a[j] = (R)(-1.0f + 2.0f * oracle_u01(w0[j]));
  a[4] = (R)(-1.0f + 2.0f * oracle_u01(w1[0]));
  a[5] = (R)(-1.0f + 2.0f * oracle_u01(w1[1]));
}

struct BodyStats { int64_t episodes; int64_t length_sum; double return_sum, return_min, return_max; int64_t nonfinite; };

template <class R>
struct Batch {
  int64_t n; uint64_t seed; uint64_t step;
  Params<R> P;
  std::vector<Env<R>> env;
  BodyStats stats;
};

void stats_clear(BodyStats* s) {
  s->episodes = 0; s->length_sum = 0; s->return_sum = 0; s->nonfinite = 0;
  s->return_min = INFINITY; s->return_max = -INFINITY;
}

template <class R>
Params<R> default_params() {
  Params<R> P;
  P.armature = (R)0.1; P.joint_damping = (R)3.0; P.friction_mu = (R)0.4;
  P.gravity = (R)9.81; P.contact_k = (R)1e4; P.contact_c = (R)100; P.h = (R)0.01; P.gear = (R)120;
  P.z0 = (R)0.8; P.substeps = 5; P.max_episode_steps = 1000; P.round_state_f32 = 0;
  P.solver = 0; P.newton_iters = 8; P.time_const = (R)0.02; P.reg_contact = (R)0.02; P.reg_limit = (R)0.5;
  return P;
}

template <class R>
void run_range(Batch<R>* B, int64_t lo, int64_t hi, int32_t T, const R* actions, R* obs, R* reward,
               uint8_t* done, BodyStats* st) {
  const int64_t n = B->n;
  for (int32_t t = 0; t < T; ++t) {
    const uint64_t s = B->step + (uint64_t)t;
    for (int64_t i = lo; i < hi; ++i) {
      R a[NACT];
      if (actions) for (int j = 0; j < NACT; ++j) a[j] = actions[((int64_t)t * n + i) * NACT + j];
      else draw_actions(B->seed, (uint32_t)i, s, a);
      StepInfo info;
      const R r = env_step(B->P, &B->env[(size_t)i], a, B->seed, (uint32_t)i, s, &info);
      if (info.nonfinite) st->nonfinite += 1;
      else if (info.done) {
        st->episodes += 1; st->length_sum += info.fin_len; st->return_sum += info.fin_ret;
        if (info.fin_ret < st->return_min) st->return_min = info.fin_ret;
        if (info.fin_ret > st->return_max) st->return_max = info.fin_ret;
      }
      if (obs) observe(B->env[(size_t)i], obs + ((int64_t)t * n + i) * 17);
      if (reward) reward[(int64_t)t * n + i] = r;
      if (done) done[(int64_t)t * n + i] = (uint8_t)info.done;
    }
  }
}

template <class R>
void rollout(Batch<R>* B, int32_t T, const R* actions, R* obs, R* reward, uint8_t* done, int nthreads) {
  if (nthreads <= 1) {
    run_range(B, (int64_t)0, B->n, T, actions, obs, reward, done, &B->stats);
  } else {
    std::vector<std::thread> pool;
    std::vector<BodyStats> part((size_t)nthreads);
    for (int k = 0; k < nthreads; ++k) {
      stats_clear(&part[(size_t)k]);
      const int64_t lo = B->n * k / nthreads, hi = B->n * (k + 1) / nthreads;
      pool.emplace_back(run_range<R>, B, lo, hi, T, actions, obs, reward, done, &part[(size_t)k]);
    }
    for (auto& th : pool) th.join();
    for (auto& p : part) {
      B->stats.episodes += p.episodes; B->stats.length_sum += p.length_sum;
      B->stats.return_sum += p.return_sum; B->stats.nonfinite += p.nonfinite;
      if (p.return_min < B->stats.return_min) B->stats.return_min = p.return_min;
      if (p.return_max > B->stats.return_max) B->stats.return_max = p.return_max;
    }
  }
  B->step += (uint64_t)T;
}

template <class R>
Batch<R>* create(int64_t n, uint64_t seed, const double* cfg /* armature, damping, mu, max_steps or null */) {
  Batch<R>* B = new Batch<R>();
  B->n = n; B->seed = seed; B->step = 0;
  B->P = default_params<R>();
  if (cfg) {
    B->P.armature = (R)cfg[0]; B->P.joint_damping = (R)cfg[1]; B->P.friction_mu = (R)cfg[2];
    B->P.max_episode_steps = (int)cfg[3];
  }
  B->env.resize((size_t)n);
  stats_clear(&B->stats);
  for (int64_t i = 0; i < n; ++i) reset_env(B->P, &B->env[(size_t)i], seed, (uint32_t)i, (uint64_t)0);
  return B;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// C entry points, one set per scalar type (suffix _f32 / _f64).
#define BODY_API(R, SFX)                                                                          \
  extern "C" {                                                                                    \
  void* oracle_body_create##SFX(int64_t n, uint64_t seed, const double* cfg) {                    \
    return create<R>(n, seed, cfg);                                                               \
  }                                                                                               \
  void oracle_body_destroy##SFX(void* h) { delete (Batch<R>*)h; }                                 \
  void oracle_body_set_params##SFX(void* h, const double* p /* 15: armature damping mu g k c h gear substeps round_state_f32 solver newton_iters time_const reg_contact reg_limit */) { \
    Batch<R>* B = (Batch<R>*)h;                                                                   \
    B->P.solver = (int)p[10]; B->P.newton_iters = (int)p[11]; B->P.time_const = (R)p[12];         \
    B->P.reg_contact = (R)p[13]; B->P.reg_limit = (R)p[14];                                       \
    B->P.armature = (R)p[0]; B->P.joint_damping = (R)p[1]; B->P.friction_mu = (R)p[2];            \
    B->P.gravity = (R)p[3]; B->P.contact_k = (R)p[4]; B->P.contact_c = (R)p[5]; B->P.h = (R)p[6]; \
    B->P.gear = (R)p[7]; B->P.substeps = (int)p[8]; B->P.round_state_f32 = (int)p[9];             \
  }                                                                                               \
  void oracle_body_reset##SFX(void* h, R* obs) {                                                  \
    Batch<R>* B = (Batch<R>*)h;                                                                   \
    for (int64_t i = 0; i < B->n; ++i) {                                                          \
      reset_env(B->P, &B->env[(size_t)i], B->seed, (uint32_t)i, B->step);                         \
      if (obs) observe(B->env[(size_t)i], obs + 17 * i);                                          \
    }                                                                                             \
  }                                                                                               \
  void oracle_body_rollout##SFX(void* h, int32_t T, const R* actions, R* obs, R* reward,          \
                                uint8_t* done, int32_t nthreads) {                                \
    rollout((Batch<R>*)h, T, actions, obs, reward, done, nthreads);                               \
  }                                                                                               \
  /* state as [n][20]: q[9] v[9] ep_ret ep_len(as scalar) */                                      \
  void oracle_body_get_state##SFX(void* h, R* out) {                                              \
    Batch<R>* B = (Batch<R>*)h;                                                                   \
    for (int64_t i = 0; i < B->n; ++i) {                                                          \
      const Env<R>& e = B->env[(size_t)i];                                                        \
      for (int j = 0; j < NQ; ++j) { out[20 * i + j] = e.q[j]; out[20 * i + 9 + j] = e.v[j]; }    \
      out[20 * i + 18] = e.ep_ret; out[20 * i + 19] = (R)e.ep_len;                                \
    }                                                                                             \
  }                                                                                               \
  void oracle_body_set_state##SFX(void* h, const R* in) {                                         \
    Batch<R>* B = (Batch<R>*)h;                                                                   \
    for (int64_t i = 0; i < B->n; ++i) {                                                          \
      Env<R>& e = B->env[(size_t)i];                                                              \
      for (int j = 0; j < NQ; ++j) { e.q[j] = in[20 * i + j]; e.v[j] = in[20 * i + 9 + j]; }      \
      e.ep_ret = in[20 * i + 18]; e.ep_len = (int32_t)in[20 * i + 19];                            \
    }                                                                                             \
  }                                                                                               \
  uint64_t oracle_body_step_count##SFX(void* h) { return ((Batch<R>*)h)->step; }                  \
  void oracle_body_set_step_count##SFX(void* h, uint64_t s) { ((Batch<R>*)h)->step = s; }         \
  void oracle_body_get_stats##SFX(void* h, BodyStats* out, int32_t clear) {                       \
    Batch<R>* B = (Batch<R>*)h; *out = B->stats; if (clear) stats_clear(&B->stats);               \
  }                                                                                               \
  /* component access for the pins; all use the batch's parameters */                             \
  void oracle_body_mass_matrix##SFX(void* h, const R* q, R* M81) {                                \
    R M[NQ][NQ]; mass_matrix(((Batch<R>*)h)->P, q, M); std::memcpy(M81, M, sizeof M);             \
  }                                                                                               \
  void oracle_body_bias_gravity##SFX(void* h, const R* q, const R* v, R* hb, R* Qg) {             \
    bias_and_gravity(((Batch<R>*)h)->P, q, v, hb, Qg);                                            \
  }                                                                                               \
  void oracle_body_contact##SFX(void* h, const R* q, const R* v, R* Q9, R* forces16) {            \
    for (int j = 0; j < NQ; ++j) Q9[j] = 0;                                                       \
    contact_forces(((Batch<R>*)h)->P, q, v, Q9, forces16);                                        \
  }                                                                                               \
  /* kind 0: link centre of mass `index` (0..6); kind 1: contact point `index` (0..7) */          \
  void oracle_body_point##SFX(int32_t kind, int32_t index, const R* q, const R* v, R* pos2,       \
                              R* J18, R* vel2, R* jdqd2) {                                        \
    Kin<R> k; point_kinematics(kind == 0 ? LINK_COM[index] : CONTACT[index], q, v, &k);           \
    pos2[0] = k.pos[0]; pos2[1] = k.pos[1]; std::memcpy(J18, k.J, sizeof k.J);                    \
    vel2[0] = k.vel[0]; vel2[1] = k.vel[1]; jdqd2[0] = k.jdqd[0]; jdqd2[1] = k.jdqd[1];           \
  }                                                                                               \
  double oracle_body_energy##SFX(void* h, const R* q, const R* v) {                               \
    return (double)energy(((Batch<R>*)h)->P, q, v);                                               \
  }                                                                                               \
  /* one substep in place on (q, v) with clipped actions a; returns the limit mask or -1 */       \
  int32_t oracle_body_substep##SFX(void* h, R* q, R* v, const R* a_in) {                          \
    R a[NACT]; clip_actions(a_in, a); int mask = 0;                                               \
    return substep(((Batch<R>*)h)->P, q, v, a, &mask) ? mask : -1;                                \
  }                                                                                               \
  /* Newton contact model, for the pins: rows at (q, v); returns their number */                  \
  int32_t oracle_body_newton_rows##SFX(void* h, const R* q, const R* v, R* J /* [22][9] */, R* aref, R* D) { \
    Rows<R> rows; constraint_rows(((Batch<R>*)h)->P, q, v, &rows);                                \
    std::memcpy(J, rows.J, sizeof rows.J); std::memcpy(aref, rows.aref, sizeof rows.aref);        \
    std::memcpy(D, rows.D, sizeof rows.D); return rows.m;                                         \
  }                                                                                               \
  /* acceleration of one substep at (q, v) under clipped actions; info4 = rows, passes, converged, active set */ \
  int32_t oracle_body_newton_accel##SFX(void* h, const R* q, const R* v, const R* a_in, R* acc9, R* f9, int32_t* info4) { \
    const Params<R>& P = ((Batch<R>*)h)->P;                                                       \
    R a[NACT]; clip_actions(a_in, a); R M[NQ][NQ]; smooth_force(P, q, v, a, M, f9);               \
    Rows<R> rows; constraint_rows(P, q, v, &rows); NewtonInfo info = {0, 0, 0, 0};                \
    const bool ok = newton_solve(P, M, f9, rows, acc9, &info);                                    \
    info4[0] = info.rows; info4[1] = info.passes; info4[2] = info.converged; info4[3] = (int32_t)info.active; \
    return ok ? 1 : 0;                                                                            \
  }                                                                                               \
  /* smallest distance of any decision of one env step (all substeps, penalty model) from its   */ \
  /* switching surface, stepping a copy of (q, v) under clipped actions; -1 if a solve fails      */ \
  double oracle_body_step_margin##SFX(void* h, const R* q_in, const R* v_in, const R* a_in) {     \
    const Params<R>& P = ((Batch<R>*)h)->P;                                                       \
    R q[NQ], v[NQ], a[NACT]; clip_actions(a_in, a);                                               \
    for (int j = 0; j < NQ; ++j) { q[j] = q_in[j]; v[j] = v_in[j]; }                              \
    R margin = (R)INFINITY;                                                                       \
    for (int s = 0; s < P.substeps; ++s)                                                          \
      if (!substep(P, q, v, a, (int*)nullptr, &margin)) return -1.0;                              \
    return (double)margin;                                                                        \
  }                                                                                               \
  int32_t oracle_body_solve##SFX(const R* A81, const R* b, R* x) {                                \
    R A[NQ][NQ]; std::memcpy(A, A81, sizeof A); return cholesky_solve(A, b, x) ? 1 : 0;           \
  }                                                                                               \
  void oracle_body_draw_actions##SFX(uint64_t seed, uint32_t env, uint64_t step, R* a6) {         \
    draw_actions(seed, env, step, a6);                                                            \
  }                                                                                               \
  }

BODY_API(float, _f32)
BODY_API(double, _f64)

extern "C" {
// link table for tests: mass, length of link i
void oracle_body_link(int32_t i, double* mass, double* length) { *mass = LINK_MASS[i]; *length = LINK_LEN[i]; }
}
