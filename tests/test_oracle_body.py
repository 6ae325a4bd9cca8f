"""Pins for the rigid-body oracle (CPU only): invariants, closed forms, finite-difference checks
and library cross-checks, mostly on the float64 instantiation."""
import math

import numpy as np
import pytest

from oracle.body_binding import Body, NQ

RNG = np.random.default_rng(2024)
M_TOT = 13.6
G = 9.81


@pytest.fixture(scope="module")
def b64():
    return Body(4, 1, np.float64)


def rand_q(scale=0.8):
    q = RNG.uniform(-scale, scale, NQ)
    q[1] = RNG.uniform(2.0, 3.0)          # well above the ground
    return q


def links(b):
    return [b.link(i) for i in range(7)]


def link_angle_rates(v):
    """omega of torso, back thigh/shin/foot, front thigh/shin/foot."""
    return [v[2], v[2] + v[3], v[2] + v[3] + v[4], v[2] + v[3] + v[4] + v[5],
            v[2] + v[6], v[2] + v[6] + v[7], v[2] + v[6] + v[7] + v[8]]


# ------------------------------------------------------------------ geometry and Jacobians

def test_rest_pose_geometry(b64):
    q = np.zeros(NQ); q[1] = 0.8
    # legs hang straight down from the torso ends; toes 0.78 below the hips
    toe_b = b64.point(1, 3, q)[0]; toe_f = b64.point(1, 7, q)[0]
    assert np.allclose(toe_b, [-0.5, 0.8 - 0.78]) and np.allclose(toe_f, [0.5, 0.8 - 0.78])
    assert np.allclose(b64.point(1, 0, q)[0], [-0.5, 0.8]) and np.allclose(b64.point(1, 4, q)[0], [0.5, 0.8])
    assert np.allclose(b64.point(1, 1, q)[0], [-0.5, 0.8 - 0.29])          # back knee
    assert np.allclose(b64.point(0, 2, q)[0], [-0.5, 0.8 - 0.29 - 0.15])   # back shin centre
    # pitch the torso by +90 degrees (CCW): front hip goes up, back hip down, legs point +x
    q[2] = math.pi / 2
    assert np.allclose(b64.point(1, 4, q)[0], [0.0, 1.3]) and np.allclose(b64.point(1, 0, q)[0], [0.0, 0.3])
    assert np.allclose(b64.point(1, 7, q)[0], [0.78, 1.3])
    # positive joint angle swings the leg forward (+x) from straight down
    q = np.zeros(NQ); q[1] = 0.8; q[3] = 0.3
    knee = b64.point(1, 1, q)[0]
    assert np.allclose(knee, [-0.5 + 0.29 * math.sin(0.3), 0.8 - 0.29 * math.cos(0.3)])


def test_jacobians_match_finite_differences(b64):
    eps = 1e-6
    for _ in range(5):
        q, v = rand_q(), RNG.normal(0, 2, NQ)
        for kind, count in ((0, 7), (1, 8)):
            for idx in range(count):
                pos, J, vel, jd = b64.point(kind, idx, q, v)
                Jfd = np.zeros((2, NQ))
                for j in range(NQ):
                    dq = np.zeros(NQ); dq[j] = eps
                    Jfd[:, j] = (b64.point(kind, idx, q + dq)[0] - b64.point(kind, idx, q - dq)[0]) / (2 * eps)
                assert np.abs(J - Jfd).max() < 1e-8
                assert np.allclose(vel, J @ v, atol=1e-12)
                # dJ/dt qdot = second derivative of the position along the straight line q + s v
                acc = (b64.point(kind, idx, q + eps * 100 * v)[0] - 2 * pos
                       + b64.point(kind, idx, q - eps * 100 * v)[0]) / (eps * 100) ** 2
                assert np.abs(jd - acc).max() < 1e-4 * max(1.0, np.abs(acc).max())


# ------------------------------------------------------------------ mass matrix, bias, gravity

def test_mass_matrix_structure(b64):
    for _ in range(20):
        q = rand_q(3.0)
        M = b64.mass_matrix(q)
        assert np.abs(M - M.T).max() < 1e-13
        assert np.linalg.eigvalsh(M).min() > 0.05
        assert abs(M[0, 0] - M_TOT) < 1e-12 and abs(M[1, 1] - M_TOT) < 1e-12 and abs(M[0, 1]) < 1e-13
        # the two legs do not couple directly
        assert np.abs(M[3:6, 6:9]).max() == 0.0


def test_composite_inertia_by_hand(b64):
    q = np.zeros(NQ); q[1] = 1.0
    b = Body(1, 1, np.float64, armature=0.0)
    M = b.mass_matrix(q)
    leg = 0.0
    for m, L, z in ((1.5, 0.29, 0.145), (1.2, 0.30, 0.29 + 0.15), (0.9, 0.19, 0.59 + 0.095)):
        leg += m * L * L / 12 + m * (0.25 + z * z)          # parallel axis about the torso centre
    want = 6.4 * 1.0 / 12 + 2 * leg
    assert abs(M[2, 2] - want) < 1e-12
    # foot joint alone: the foot about its ankle, m L^2 / 3
    assert abs(M[5, 5] - 0.9 * 0.19 ** 2 / 3) < 1e-12
    # armature adds to the six joint diagonals only
    M2 = b64.mass_matrix(q)
    D = M2 - M
    assert np.allclose(np.diag(D), [0, 0, 0] + [0.1] * 6) and np.abs(D - np.diag(np.diag(D))).max() == 0


def test_kinetic_energy_from_finite_difference_velocities(b64):
    eps = 1e-6
    b = Body(1, 1, np.float64, armature=0.0)
    for _ in range(5):
        q, v = rand_q(), RNG.normal(0, 2, NQ)
        T = 0.0
        om = link_angle_rates(v)
        for i, (m, L) in enumerate(links(b)):
            pdot = (b.point(0, i, q + eps * v)[0] - b.point(0, i, q - eps * v)[0]) / (2 * eps)
            T += 0.5 * m * pdot @ pdot + 0.5 * (m * L * L / 12) * om[i] ** 2
        assert abs(0.5 * v @ b.mass_matrix(q) @ v - T) < 1e-7 * max(1.0, T)


def test_bias_equals_christoffel_form_by_finite_differences(b64):
    # h = Mdot qdot - 1/2 d(qdot^T M qdot)/dq ; a sign error in the Coriolis terms fails this
    eps = 1e-6
    for _ in range(5):
        q, v = rand_q(), RNG.normal(0, 2, NQ)
        hb, _ = b64.bias_gravity(q, v)
        Mdot = (b64.mass_matrix(q + eps * v) - b64.mass_matrix(q - eps * v)) / (2 * eps)
        grad = np.zeros(NQ)
        for j in range(NQ):
            dq = np.zeros(NQ); dq[j] = eps
            grad[j] = (v @ b64.mass_matrix(q + dq) @ v - v @ b64.mass_matrix(q - dq) @ v) / (2 * eps)
        want = Mdot @ v - 0.5 * grad
        assert np.abs(hb - want).max() < 1e-6 * max(1.0, np.abs(want).max())
        assert np.abs(hb).max() > 0.1          # the check is not vacuous


def test_gravity_forces_are_minus_potential_gradient(b64):
    eps = 1e-6
    for _ in range(5):
        q = rand_q()
        _, Qg = b64.bias_gravity(q, np.zeros(NQ))
        grad = np.zeros(NQ)
        for j in range(NQ):
            dq = np.zeros(NQ); dq[j] = eps
            grad[j] = (b64.energy(q + dq, np.zeros(NQ)) - b64.energy(q - dq, np.zeros(NQ))) / (2 * eps)
        assert np.abs(Qg + grad).max() < 1e-7
        assert abs(Qg[1] + M_TOT * G) < 1e-12 and abs(Qg[0]) < 1e-13


def accelerations(b, q, v, tau):
    M = b.mass_matrix(q)
    hb, Qg = b.bias_gravity(q, v)
    return np.linalg.solve(M, Qg + tau - hb)


def test_centre_of_mass_falls_freely_whatever_the_joint_torques(b64):
    for _ in range(10):
        q, v = rand_q(), RNG.normal(0, 3, NQ)
        tau = np.zeros(NQ); tau[3:] = RNG.normal(0, 50, 6)
        a = accelerations(b64, q, v, tau)
        acc = np.zeros(2)
        for i, (m, _) in enumerate(links(b64)):
            _, J, _, jd = b64.point(0, i, q, v)
            acc += m * (J @ a + jd)
        assert np.abs(acc / M_TOT - [0, -G]).max() < 1e-11


def test_angular_momentum_balance_under_internal_torques(b64):
    # d/dt sum_i [ m_i r_i x rdot_i + I_i omega_i ] = sum_i r_i x (0, -m_i g): joint torques drop out
    for _ in range(10):
        q, v = rand_q(), RNG.normal(0, 3, NQ)
        tau = np.zeros(NQ); tau[3:] = RNG.normal(0, 50, 6)
        a = accelerations(Body(1, 1, np.float64, armature=0.0), q, v, tau)
        lhs = rhs = 0.0
        alpha = link_angle_rates(a)
        for i, (m, L) in enumerate(links(b64)):
            pos, J, vel, jd = b64.point(0, i, q, v)
            acc = J @ a + jd
            lhs += m * (pos[0] * acc[1] - pos[1] * acc[0]) + (m * L * L / 12) * alpha[i]
            rhs += pos[0] * (-m * G)
        assert abs(lhs - rhs) < 1e-9 * max(1.0, abs(rhs))


def test_power_balance(b64):
    # dE/dt along the computed acceleration equals the power of the joint torques
    b = Body(1, 1, np.float64, joint_damping=0.0)
    d = 1e-6
    for _ in range(5):
        q, v = rand_q(), RNG.normal(0, 2, NQ)
        tau = np.zeros(NQ); tau[3:] = RNG.normal(0, 20, 6)
        a = accelerations(b, q, v, tau)
        Ep = b.energy(q + d * v + 0.5 * d * d * a, v + d * a)
        Em = b.energy(q - d * v + 0.5 * d * d * a, v - d * a)
        assert abs((Ep - Em) / (2 * d) - tau @ v) < 1e-5 * max(1.0, abs(tau @ v))


# ------------------------------------------------------------------ integrator

def free_body(h, **kw):
    return Body(1, 1, np.float64, joint_damping=0.0, h=h, **kw)


def test_free_fall_energy_loss_closed_form():
    # semi-implicit Euler in free fall loses exactly M g^2 h^2 / 2 per substep
    for h in (0.01, 0.002):
        b = free_body(h)
        q = np.zeros(NQ); q[1] = 50.0; q[3:] = [0.3, -0.4, 0.2, -0.1, 0.5, -0.3]
        v = np.zeros(NQ); v[0] = 1.0; v[1] = 2.0
        for _ in range(20):
            E0 = b.energy(q, v)
            q, v, mask = b.substep(q, v, np.zeros(6))
            assert mask == 0
            assert abs((b.energy(q, v) - E0) + 0.5 * M_TOT * G * G * h * h) < 1e-9
        assert np.allclose(q[3:], [0.3, -0.4, 0.2, -0.1, 0.5, -0.3], atol=1e-12)   # rigid translation


def drift_per_step(h, steps=40):
    b = free_body(h)
    q = np.zeros(NQ); q[1] = 50.0; q[3:] = [0.2, -0.3, 0.1, -0.2, 0.3, -0.1]
    v = np.array([0.5, 0.0, 0.7, 1.5, -2.0, 1.0, -1.5, 2.0, -1.0])
    E0 = b.energy(q, v)
    worst = 0.0
    for _ in range(steps):
        q2, v2, mask = b.substep(q, v, np.zeros(6))
        assert mask == 0
        worst = max(worst, abs(b.energy(q2, v2) - b.energy(q, v)) / abs(E0))
        q, v = q2, v2
    return worst


def test_energy_drift_is_second_order_and_small_at_small_h():
    d1, d2, d3 = drift_per_step(1e-3), drift_per_step(5e-4), drift_per_step(2.5e-4)
    assert d3 < 1e-6                                  # zero torque, no contact, damping off
    assert 3.3 < d1 / d2 < 4.7 and 3.3 < d2 / d3 < 4.7   # halving h quarters the per-step drift


def test_substep_equals_library_solve_of_the_assembled_system(b64):
    # L2 composition: v+ from the oracle's substep equals numpy's solve of M v = M v0 + h rhs
    for _ in range(10):
        q = rand_q(0.6); q[1] = RNG.uniform(0.3, 0.9)         # low enough for contacts
        v = RNG.normal(0, 2, NQ)
        a = RNG.uniform(-1.5, 1.5, 6)
        M = b64.mass_matrix(q)
        hb, Qg = b64.bias_gravity(q, v)
        Qc, _ = b64.contact(q, v)
        rhs = Qg - hb + Qc
        rhs[3:] += 120.0 * np.clip(a, -1, 1) - 3.0 * v[3:]
        vstar = np.linalg.solve(M, M @ v + 0.01 * rhs)
        q2, v2, mask = b64.substep(q, v, a)
        assert mask == 0 and np.all(np.abs(q[3:]) < 1)
        assert np.abs(v2 - vstar).max() < 1e-9 * max(1.0, np.abs(vstar).max())
        assert np.allclose(q2, q + 0.01 * v2, atol=1e-13)


def test_joint_limit_projection(b64):
    hits = 0
    for trial in range(40):
        q = rand_q(0.6); q[1] = 3.0
        v = RNG.normal(0, 3, NQ)
        a = RNG.uniform(-1, 1, 6)
        at_limit = RNG.random(6) < 0.5
        q[3:][at_limit] = np.where(RNG.random(at_limit.sum()) < 0.5, 1.0, -1.0)
        M = b64.mass_matrix(q)
        hb, Qg = b64.bias_gravity(q, v)
        rhs = Qg - hb
        rhs[3:] += 120.0 * a - 3.0 * v[3:]
        bvec = M @ v + 0.01 * rhs
        vstar = np.linalg.solve(M, bvec)
        S = [j for j in range(3, NQ) if (q[j] >= 1 and vstar[j] > 0) or (q[j] <= -1 and vstar[j] < 0)]
        q2, v2, mask = b64.substep(q, v, a)
        assert mask == sum(1 << j for j in S)
        F = [j for j in range(NQ) if j not in S]
        want = np.zeros(NQ)
        want[F] = np.linalg.solve(M[np.ix_(F, F)], bvec[F])
        assert np.abs(v2 - want).max() < 1e-9 * max(1.0, np.abs(want).max())
        assert np.all(v2[S] == 0.0)
        assert np.all(np.abs(q2[3:]) <= 1.0)
        # M-orthogonal projection: kinetic energy never increases
        assert v2 @ M @ v2 <= vstar @ M @ vstar * (1 + 1e-12)
        hits += len(S)
    assert hits > 20


def test_cholesky_solver_against_lapack(b64):
    for dt, tol in ((np.float64, 1e-11), (np.float32, 2e-4)):
        b = Body(1, 1, dt)
        for _ in range(10):
            A = RNG.normal(size=(NQ, NQ)); A = A @ A.T + NQ * np.eye(NQ)
            rhs = RNG.normal(size=NQ)
            x, ok = b.solve(A, rhs)
            assert ok and np.abs(x - np.linalg.solve(A, rhs)).max() < tol
        _, ok = b.solve(-np.eye(NQ), np.ones(NQ))
        assert not ok


# ------------------------------------------------------------------ contact

def test_contact_force_law_signs(b64):
    q = np.zeros(NQ); q[1] = 0.78 - 0.01           # both toes 1 cm inside the ground, at rest
    Q, F = b64.contact(q, np.zeros(NQ))
    assert np.allclose(F[3], [0, 100.0]) and np.allclose(F[7], [0, 100.0])      # k * penetration
    assert np.all(F[[0, 1, 2, 4, 5, 6]] == 0)
    assert abs(Q[1] - 200.0) < 1e-9 and abs(Q[0]) < 1e-12
    # moving down adds damping force, moving up fast enough removes the force (no adhesion)
    v = np.zeros(NQ); v[1] = -0.5
    assert np.allclose(b64.contact(q, v)[1][3], [0, 100.0 + 50.0])
    v[1] = +2.0
    assert np.all(b64.contact(q, v)[1] == 0)
    # sliding forward: friction opposes, saturates at mu * F_n
    v = np.zeros(NQ); v[0] = 0.1
    assert np.allclose(b64.contact(q, v)[1][3], [-10.0, 100.0])       # c * vx = 10 < 0.4 * 100
    v[0] = -5.0
    assert np.allclose(b64.contact(q, v)[1][3], [+40.0, 100.0])       # capped at mu * F_n
    # above the ground nothing acts
    q[1] = 0.79
    assert np.all(b64.contact(q, np.zeros(NQ))[0] == 0)


def test_resting_body_is_carried_by_the_ground():
    # zero actions: the body sinks onto the ground and stays there (the explicit penalty contact
    # keeps a small chatter); averaged over time the normal forces carry the weight M g and the
    # tangential forces vanish (momentum balance of the whole body)
    b = Body(1, 3, np.float64, max_episode_steps=10 ** 8)
    b.reset()
    b.rollout(1500, actions=np.zeros((1500, 1, 6)))
    s = b.get_state()[0]
    q, v = s[:9].copy(), s[9:18].copy()
    assert q[1] < 0.3 and np.abs(v).max() < 0.2
    fn = ft = 0.0
    v_start = v.copy()
    steps = 2000
    for _ in range(steps):
        _, F = b.contact(q, v)
        fn += F[:, 1].sum(); ft += F[:, 0].sum()
        q, v, _ = b.substep(q, v, np.zeros(6))
    assert abs(fn / steps - M_TOT * G) < 0.01 * M_TOT * G
    assert abs(ft / steps) < 0.5
    assert np.abs(v - v_start).max() < 0.3


# ------------------------------------------------------------------ resets, actions, rollouts

def test_reset_distribution():
    n = 4000
    b = Body(n, 11, np.float32)
    obs = b.reset()
    s = b.get_state()
    q0, v0 = s[:, :9].astype(np.float64), s[:, 9:18].astype(np.float64)
    base = np.zeros(9); base[1] = 0.8
    d = q0 - base
    assert d.min() >= -0.1 - 1e-6 and d.max() <= 0.1 + 1e-6
    m = n * 9
    assert abs(d.mean()) < 4.5 * math.sqrt(0.2 ** 2 / 12 / m)
    assert abs(d.var() - 0.2 ** 2 / 12) < 4.5 * math.sqrt((0.2 ** 4 / 80 - (0.2 ** 2 / 12) ** 2) / m)
    assert abs(v0.mean()) < 4.5 * 0.1 / math.sqrt(m)
    assert abs(v0.var() - 0.01) < 4.5 * 0.01 * math.sqrt(2.0 / m)
    # every coordinate gets its own draw: columns are uncorrelated
    c = np.corrcoef(np.concatenate([d, v0], axis=1).T)
    assert np.abs(c - np.eye(18)).max() < 0.1
    assert np.array_equal(obs, np.concatenate([s[:, 1:9], s[:, 9:18]], axis=1))


def test_action_draws_and_clipping():
    b = Body(2, 5, np.float32)
    a = np.array([b.draw_actions(e, t) for e in range(2) for t in range(3000)], np.float64)
    assert a.min() >= -1 and a.max() < 1
    assert abs(a.mean()) < 4.5 * math.sqrt(1 / 3 / a.size)
    assert abs((a ** 2).mean() - 1 / 3) < 4.5 * math.sqrt((1 / 5 - 1 / 9) / a.size)
    # actions outside [-1, 1] act as the clipped value
    q = np.zeros(NQ); q[1] = 3.0
    b64 = Body(1, 1, np.float64)
    big = b64.substep(q, np.zeros(NQ), np.array([5, -5, 0.5, 2, -2, 0.0]))
    clipped = b64.substep(q, np.zeros(NQ), np.array([1, -1, 0.5, 1, -1, 0.0]))
    assert np.array_equal(big[1], clipped[1])


def test_reward_truncation_and_structure():
    n, T = 64, 260
    b = Body(n, 9, np.float32, max_episode_steps=100)
    b.reset()
    obs, rew, done = b.rollout(T)
    assert np.isfinite(obs).all() and np.isfinite(rew).all()
    assert np.array_equal(np.flatnonzero(done[:, 0]), [99, 199])
    assert np.all(done.sum(0) == 2)
    st = b.stats()
    assert st["episodes"] == 2 * n and st["length_sum"] == 200 * n and st["nonfinite"] == 0
    # reward = mean forward velocity over the substeps - 0.1 |a|^2, action part recomputed here
    acts = np.array([[b.draw_actions(e, t) for e in range(n)] for t in range(T)], np.float64)
    cost = 0.1 * (acts ** 2).sum(-1)
    fwd = rew.astype(np.float64) + cost
    # the last substep's velocity is in the observation; the mean over 5 substeps stays close to it
    live = done == 0
    assert np.abs(fwd[live] - obs[..., 8][live]).mean() < 0.5
    ret = np.add.reduceat(rew.astype(np.float64), [0, 100], axis=0)[:2].sum()
    assert abs(st["return_sum"] - rew[:200].astype(np.float64).sum()) < 1e-2
    # N-independence and split rollouts
    c = Body(8, 9, np.float32, max_episode_steps=100); c.reset()
    o1, r1, d1 = c.rollout(130)
    o2, r2, d2 = c.rollout(130)
    assert np.array_equal(np.concatenate([o1, o2]), obs[:, :8])
    assert np.array_equal(np.concatenate([r1, r2]), rew[:, :8])
    d = Body(8, 9, np.float32, max_episode_steps=100); d.reset()
    o3, _, _ = d.rollout(T, nthreads=3)
    assert np.array_equal(o3, obs[:, :8])


def test_float32_and_float64_agree_on_single_steps_away_from_events():
    n = 256
    a = Body(n, 21, np.float64); a.reset()
    a.rollout(37, nthreads=4)                      # states from all phases of motion
    s = a.get_state()
    b32 = Body(n, 21, np.float32); b32.set_state(s.astype(np.float32)); b32.step_count = 37
    a.set_state(s.astype(np.float32).astype(np.float64))
    o64, r64, _ = a.rollout(1)
    o32, r32, _ = b32.rollout(1)
    err = np.abs(o32[0].astype(np.float64) - o64[0]) / np.maximum(np.abs(o64[0]), 1.0)
    frac_ok = (err.max(axis=1) < 1e-4).mean()
    assert frac_ok > 0.95                          # the rest toggled a contact or a limit
    assert np.median(err.max(axis=1)) < 2e-5


def test_thousand_step_rollouts_are_bounded_and_returns_have_the_expected_scale():
    n = 512
    b = Body(n, 4, np.float32); b.reset()
    _, rew, done = b.rollout(1000, nthreads=8, want_obs=False)
    st = b.stats()
    assert st["nonfinite"] == 0 and st["episodes"] == n and np.all(done[-1] == 1)
    ret = rew.astype(np.float64).sum(0)
    se = ret.std() / math.sqrt(n)
    # action cost alone is -200 in expectation; the forward part is small for random actions
    assert abs(ret.mean() + 200) < 15 and ret.std() < 120
    assert abs(st["return_sum"] / n - ret.mean()) < 1e-2 and se < 6


# ------------------------------------------------------------------ reward, action words, guards

def test_reward_is_mean_of_the_five_substep_velocities_minus_action_cost():
    """Benchmark configuration: reward = forward velocity - 0.1 |a|^2, with frame skip 5.  The forward
    term is the mean of the five post-update x velocities, which equals (x_after - x_before) / (5 h)
    because every substep moves x by h times its new velocity; both forms are checked, the first
    through the single-substep entry point, the second from the states alone."""
    n = 48
    b = Body(n, 13, np.float64); b.reset()
    b.rollout(23, nthreads=4)                                   # legs on the ground, joints at limits
    s0 = b.get_state()
    acts = RNG.uniform(-1.6, 1.6, (1, n, 6))                    # some beyond the clip
    _, rew, done = b.rollout(1, acts)
    s1 = b.get_state()
    assert not done.any()
    clipped = np.clip(acts[0], -1, 1)
    cost = 0.1 * (clipped ** 2).sum(-1)
    # (1) from the states: x advanced by h * (sum of the five new velocities)
    fwd_from_x = (s1[:, 0] - s0[:, 0]) / (5 * 0.01)
    assert np.abs(rew[0] - (fwd_from_x - cost)).max() < 1e-11
    # (2) five single substeps, averaging the post-update x velocity of each
    last_vs_mean = 0.0
    for e in range(n):
        q, v = s0[e, :9].copy(), s0[e, 9:18].copy()
        vx = []
        for _ in range(5):
            q, v, mask = b.substep(q, v, acts[0, e])
            assert mask >= 0
            vx.append(v[0])
        want = sum(vx) / 5 - cost[e]
        assert abs(rew[0, e] - want) <= 4 * np.spacing(abs(want)) + 1e-15
        assert np.array_equal(q, s1[e, :9]) and np.array_equal(v, s1[e, 9:18])
        last_vs_mean = max(last_vs_mean, abs(vx[-1] - sum(vx) / 5))
    # the case can tell the mean from the last substep's velocity
    assert last_vs_mean > 1e-2
    # episode return accumulates exactly this reward
    assert np.allclose(s1[:, 18] - s0[:, 18], rew[0], rtol=0, atol=1e-12)
    assert np.array_equal(s1[:, 19], s0[:, 19] + 1)


def test_action_words_stream_by_stream():
    """Actions 0..3 are words 0..3 of the per-step block of stream 0, actions 4 and 5 words 0 and 1
    of stream 1; a = -1 + 2 u with u = (w >> 8) * 2^-24, all in float32."""
    from oracle import oracle as orc
    table = [(0, 0), (0, 1), (0, 2), (0, 3), (1, 0), (1, 1)]      # action j <- (stream, word)
    seed = 0x1234567_89abcdef
    b = Body(1, seed, np.float32)
    seen = set()
    for env, step in [(0, 0), (1, 0), (0, 1), (7, 12345), (4095, 2 ** 32 + 5), (2 ** 31 + 3, 999)]:
        a = b.draw_actions(env, step)
        blocks = {s: orc.draw_block(seed, env, step, s) for s in (0, 1)}
        for j, (stream, word) in enumerate(table):
            w = blocks[stream][word]
            u = np.float32(w >> 8) * np.float32(2.0 ** -24)
            want = np.float32(-1.0) + np.float32(2.0) * u
            assert a[j] == want and a.dtype == np.float32, (env, step, j)
            seen.add(w)
    assert len(seen) == 36                                        # no word serves two actions
    # the rollout uses exactly these draws: external actions equal to them give the same step
    n = 5
    c = Body(n, 77, np.float64); c.reset()
    d = Body(n, 77, np.float64); d.reset()
    acts = np.array([[c.draw_actions(e, t) for e in range(n)] for t in range(3)])
    oc, rc, _ = c.rollout(3)
    od, rd, _ = d.rollout(3, acts)
    assert np.array_equal(oc, od) and np.array_equal(rc, rd)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_a_state_outside_the_finite_range_is_counted_and_reinitialised(dtype):
    """A state that leaves the finite range ends the step with done = 1 and reward 0, is counted as
    non-finite (not as an episode) and is re-initialised from the reset streams at step + 1."""
    n, start = 6, 41
    b = Body(n, 19, dtype); b.reset()
    b.rollout(start)
    s = b.get_state()
    bad = {1: (4, np.nan), 3: (11, np.inf), 4: (0, -np.inf)}      # env -> (component, value)
    for e, (j, val) in bad.items():
        s[e, j] = val
    b.set_state(s)
    b.stats(clear=True)
    obs, rew, done = b.rollout(1)
    st = b.stats()
    after = b.get_state()
    fresh = Body(n, 19, dtype); fresh.step_count = start + 1
    fresh_obs = fresh.reset()
    fresh_state = fresh.get_state()
    for e in range(n):
        if e in bad:
            assert done[0, e] == 1 and rew[0, e] == 0
            assert np.array_equal(after[e], fresh_state[e])       # q, v, return 0, length 0
            assert np.array_equal(obs[0, e], fresh_obs[e])
        else:
            assert done[0, e] == 0 and np.isfinite(rew[0, e]) and rew[0, e] != 0
            assert after[e, 19] == s[e, 19] + 1
    assert st["nonfinite"] == 3 and st["episodes"] == 0 and st["length_sum"] == 0
    assert st["return_sum"] == 0
    assert np.isfinite(after).all() and np.isfinite(obs).all() and np.isfinite(rew).all()
    # the other environments are untouched by their neighbours' fate
    ref = Body(n, 19, dtype); ref.reset(); ref.rollout(start)
    o2, r2, _ = ref.rollout(1)
    good = [e for e in range(n) if e not in bad]
    assert np.array_equal(o2[0, good], obs[0, good]) and np.array_equal(r2[0, good], rew[0, good])


def test_rounding_the_state_to_the_storage_format():
    """round_state_f32: after every step q, v, the episode return and the reward are rounded to
    float32 (the format the state is kept in); nothing else changes."""
    n = 40
    a = Body(n, 23, np.float64); a.reset(); a.rollout(30, nthreads=4)
    s = a.get_state().astype(np.float32).astype(np.float64)
    plain = Body(n, 23, np.float64); plain.set_state(s); plain.step_count = 30
    rounded = Body(n, 23, np.float64, round_state_f32=1); rounded.set_state(s); rounded.step_count = 30
    o_p, r_p, _ = plain.rollout(1)
    o_r, r_r, _ = rounded.rollout(1)
    sp, sr = plain.get_state(), rounded.get_state()
    f32 = lambda x: x.astype(np.float32).astype(np.float64)
    assert np.array_equal(sr[:, :18], f32(sp[:, :18]))
    assert np.array_equal(sr[:, 18], f32(sp[:, 18])) and np.array_equal(sr[:, 19], sp[:, 19])
    assert np.array_equal(r_r, f32(r_p)) and np.array_equal(o_r, f32(o_p))
    assert not np.array_equal(sr[:, :18], sp[:, :18])             # the rounding is visible
    # second step: starts from the rounded state, so it equals a fresh step from that state
    again = Body(n, 23, np.float64, round_state_f32=1); again.set_state(sr); again.step_count = 31
    o2, r2, _ = rounded.rollout(1)
    o3, r3, _ = again.rollout(1)
    assert np.array_equal(o2, o3) and np.array_equal(r2, r3)
    # off by default
    assert Body(1, 1, np.float64).params["round_state_f32"] == 0


def test_decision_margin_of_a_step():
    """The margin reported for a step is the distance of its closest decision from a switching
    surface: a contact point at height zero, a joint reaching its limit, a limit joint at rest."""
    b = Body(1, 3, np.float64, substeps=1)
    zero = np.zeros(6)
    q = np.zeros(NQ); q[1] = 2.0; v = np.zeros(NQ)
    # high above the ground, joints centred: the nearest surface is a joint limit, 1 away
    assert abs(b.step_margin(q, v, zero) - 1.0) < 1e-12
    q[4] = 0.75
    assert abs(b.step_margin(q, v, zero) - 0.25) < 1e-12
    # toes 1e-7 above the ground: that is the margin
    q = np.zeros(NQ); q[1] = 0.78 + 1e-7
    assert abs(b.step_margin(q, v, zero) - 1e-7) < 1e-12
    q[1] = 0.78 - 3e-9
    assert abs(b.step_margin(q, v, zero) - 3e-9) < 1e-12
    # a joint at its limit: the margin is |v*| of that joint, the velocity the free solve gives it
    q = np.zeros(NQ); q[1] = 2.0; q[5] = 1.0
    a = np.array([0.0, 0.0, 0.03, 0.0, 0.0, 0.0])
    _, v_after, mask = Body(1, 3, np.float64, substeps=1).substep(q, v, a)
    assert mask & (1 << 5)                                       # pushed outwards: projected, v = 0
    free = Body(1, 3, np.float64, substeps=1)
    q_in = q.copy(); q_in[5] = 0.999999                          # same state just inside: the free velocity
    _, v_free, mask2 = free.substep(q_in, v, a)
    assert mask2 == 0
    m = b.step_margin(q, v, a)
    assert abs(m - abs(v_free[5])) < 1e-4 * abs(v_free[5]) and 1e-3 < m < 0.9
    # all five substeps are covered: a body moving down crosses z = 0 in a later substep
    b5 = Body(1, 3, np.float64)
    q = np.zeros(NQ); q[1] = 0.78 + 0.02; v = np.zeros(NQ); v[1] = -1.0
    assert b5.step_margin(q, v, zero) < 0.012                    # first substep alone would report 0.02
