"""Pins for the second contact model of the rigid-body oracle (solver = 1: Newton's method on the
soft-constraint quadratic programme in acceleration space; paper App. A.1, "HalfCheetah JAX").
CPU only, float64 instantiation.  What fixes the result here is mathematics, not the paper (which
prints no formulas): the solution of a strictly convex programme is unique, so it can be checked
by its optimality conditions, by exhaustive search over active sets, and in the form of the
regularised linear complementarity problem the same conditions spell out."""
import itertools
import math

import numpy as np
import pytest

from oracle.body_binding import Body, NQ

RNG = np.random.default_rng(77)
M_TOT, G = 13.6, 9.81
TC = 0.02
K_REF, B_REF = 1.0 / TC ** 2, 2.0 / TC


@pytest.fixture(scope="module")
def nb():
    return Body(4, 1, np.float64, solver=1)


def states_in_contact(count, seed=5, warm=(3, 40)):
    """(q, v, action) triples taken from Newton-mode rollouts: contacts and joint limits active."""
    o = Body(64, seed, np.float64, solver=1)
    o.reset()
    out = []
    t = 0
    for w in warm:
        o.rollout(w, nthreads=4, want_obs=False)
        t += w
        s = o.get_state()
        for i in range(64):
            out.append((s[i, :9].copy(), s[i, 9:18].copy(), np.clip(o.draw_actions(i, t), -1, 1)))
    RNG.shuffle(out)
    return out[:count]


def cost(a, M, f, J, aref, D):
    a0 = np.linalg.solve(M, f)
    r = J @ a - aref if len(D) else np.zeros(0)
    return 0.5 * (a - a0) @ M @ (a - a0) + 0.5 * np.sum(D * np.minimum(r, 0.0) ** 2)


def test_rows_are_second_derivatives_of_the_gap_functions(nb):
    """J a - aref = g'' + b g' + k z for a contact edge g = z_p +- mu x_p along q(t) = q + v t + a t^2/2
    (derivatives by central differences of the forward kinematics), = s (a_j + b v_j) for a joint
    sitting at a limit with outward normal -s."""
    mu = 0.4
    checked_contact = checked_limit = 0
    for q, v, _ in states_in_contact(40):
        J, aref, D = nb.newton_rows(q, v)
        a = RNG.normal(0, 30, NQ)
        dt = 1e-4
        row = 0
        for p in range(8):
            z = nb.point(1, p, q)[0][1]
            if not z < 0:
                continue
            pos = [nb.point(1, p, q + v * s + 0.5 * a * s * s)[0] for s in (-dt, 0.0, dt)]
            for sign in (+1.0, -1.0):
                g = [x[1] + sign * mu * x[0] for x in pos]
                g1 = (g[2] - g[0]) / (2 * dt)
                g2 = (g[2] - 2 * g[1] + g[0]) / dt ** 2
                want = g2 + B_REF * g1 + K_REF * z
                got = J[row] @ a - aref[row]
                assert abs(got - want) < 2e-4 * max(1.0, abs(want)), (p, sign, got, want)
                assert D[row] == 1.0 / 0.02
                row += 1
                checked_contact += 1
        for j in range(3, 9):
            if abs(q[j]) >= 1:
                s = -math.copysign(1.0, q[j])
                assert np.array_equal(J[row], s * np.eye(NQ)[j])
                assert math.isclose(J[row] @ a - aref[row], s * (a[j] + B_REF * v[j]), rel_tol=1e-12, abs_tol=1e-9)
                assert D[row] == 1.0 / 0.5
                row += 1
                checked_limit += 1
        assert row == len(D)
    assert checked_contact >= 20 and checked_limit >= 20


def test_solution_is_stationary_and_solves_the_regularised_lcp(nb):
    """Optimality: M a - f = sum_i lambda_i J_i with lambda_i = D_i max(0, aref_i - J_i a).  The same
    statement as a complementarity problem in w = J a - aref + R lambda: lambda >= 0, w >= 0,
    lambda . w = 0 — and the pyramid edges give a normal force >= 0 and |tangential| <= mu normal."""
    seen_rows = 0
    for q, v, act in states_in_contact(80):
        acc, f, (m, passes, converged, active) = nb.newton_accel(q, v, act)
        assert converged == 1 and passes <= 8
        M = nb.mass_matrix(q)
        J, aref, D = nb.newton_rows(q, v)
        assert len(D) == m
        if m == 0:
            assert np.allclose(M @ acc, f, rtol=1e-11, atol=1e-9)
            continue
        r = J @ acc - aref
        lam = D * np.maximum(0.0, -r)
        resid = M @ acc - f - J.T @ lam
        assert np.abs(resid).max() < 1e-8 * max(1.0, np.abs(f).max()), np.abs(resid).max()
        w = r + lam / D
        assert (lam >= 0).all() and (w >= -1e-9 * max(1.0, np.abs(aref).max())).all()
        assert abs(lam @ w) < 1e-7 * max(1.0, lam @ lam)
        assert [bool(active >> i & 1) for i in range(m)] == list(r < 0)
        # friction pyramid per contact point (rows come in +mu / -mu pairs, contacts first)
        n_contact = sum(1 for p in range(8) if nb.point(1, p, q)[0][1] < 0)
        for c in range(n_contact):
            lp, lm = lam[2 * c], lam[2 * c + 1]
            normal, tangential = lp + lm, 0.4 * (lp - lm)
            assert normal >= 0 and abs(tangential) <= 0.4 * normal + 1e-12
        seen_rows += m
    assert seen_rows > 100


def test_exhaustive_active_set_search_finds_the_same_unique_solution(nb):
    """For every subset S of the rows solve the equality-constrained quadratic; exactly the subsets
    that reproduce themselves (row i in S iff its residual is negative) are solutions, they all
    give the same acceleration (strict convexity), and it is the solver's."""
    done = 0
    for q, v, act in states_in_contact(60, seed=9):
        J, aref, D = nb.newton_rows(q, v)
        m = len(D)
        if m == 0 or m > 10:
            continue
        acc, f, _ = nb.newton_accel(q, v, act)
        M = nb.mass_matrix(q)
        sols = []
        for bits in itertools.product((False, True), repeat=m):
            S = np.array(bits)
            H = M + (J[S].T * D[S]) @ J[S]
            a = np.linalg.solve(H, f + J[S].T @ (D[S] * aref[S]))
            r = J @ a - aref
            if np.array_equal(r < 0, S):
                sols.append(a)
        assert len(sols) >= 1
        for a in sols:
            assert np.allclose(a, acc, rtol=1e-9, atol=1e-8 * max(1.0, np.abs(acc).max()))
        done += 1
    assert done >= 25


def test_solution_is_the_global_minimum(nb):
    for q, v, act in states_in_contact(30, seed=11):
        acc, f, _ = nb.newton_accel(q, v, act)
        M = nb.mass_matrix(q)
        J, aref, D = nb.newton_rows(q, v)
        c0 = cost(acc, M, f, J, aref, D)
        a_free = np.linalg.solve(M, f)
        assert c0 <= cost(a_free, M, f, J, aref, D) + 1e-9
        for scale in (1e-3, 1e-1, 10.0):
            for _ in range(20):
                assert cost(acc + RNG.normal(0, scale, NQ), M, f, J, aref, D) >= c0 - 1e-9 * max(1.0, c0)


def test_without_rows_the_step_is_the_unconstrained_one_and_matches_the_penalty_model():
    """Airborne and inside the joint range both models are plain semi-implicit Euler on
    M a = Q_g + tau - h: the two substeps must agree to rounding."""
    new, old = Body(1, 0, np.float64, solver=1), Body(1, 0, np.float64)
    for _ in range(10):
        q = RNG.uniform(-0.8, 0.8, NQ); q[1] = RNG.uniform(2.0, 3.0)
        v = RNG.normal(0, 2, NQ)
        act = RNG.uniform(-1, 1, 6)
        assert len(new.newton_rows(q, v)[2]) == 0
        q1, v1, _ = new.substep(q, v, act)
        q2, v2, _ = old.substep(q, v, act)
        assert np.allclose(q1, q2, rtol=0, atol=1e-12) and np.allclose(v1, v2, rtol=0, atol=1e-10)


def test_body_dropped_on_the_ground_comes_to_rest_carrying_its_weight():
    """Zero actions, joints locked by a huge armature: the body is a rigid table on its two toes and
    settles completely (the penalty model keeps chattering here).  At rest the contact forces sum
    to the weight, no tangential force remains, and each toe sinks by weight / (2 toes * 2 edges *
    D * k), the static solution of the soft constraint."""
    o = Body(1, 3, np.float64, solver=1, armature=1e6, max_episode_steps=10 ** 8)
    q = np.zeros(NQ); q[1] = 0.79
    s = np.zeros((1, 20)); s[0, :9] = q
    o.set_state(s)
    zero = np.zeros((1, 1, 6))
    for _ in range(200):
        o.rollout(1, actions=zero)
    st = o.get_state()[0]
    q, v = st[:9], st[9:18]
    assert np.abs(v).max() < 1e-10 and abs(q[2]) < 1e-10
    acc, f, (m, _, conv, _) = o.newton_accel(q, v, np.zeros(6))
    assert conv == 1 and m == 4 and np.abs(acc).max() < 1e-9
    J, aref, D = o.newton_rows(q, v)
    lam = D * np.maximum(0.0, aref - J @ acc)
    normal = sum(lam[2 * c] + lam[2 * c + 1] for c in range(2))
    tangential = sum(0.4 * (lam[2 * c] - lam[2 * c + 1]) for c in range(2))
    assert math.isclose(normal, M_TOT * G, rel_tol=1e-9)
    assert abs(tangential) < 1e-9 * M_TOT * G
    depth = [-o.point(1, p, q)[0][1] for p in (3, 7)]
    want = M_TOT * G / (2 * 2 * 50.0 * K_REF)
    assert math.isclose(depth[0], want, rel_tol=1e-6) and math.isclose(depth[1], want, rel_tol=1e-6)
    assert all(o.point(1, p, q)[0][1] > 0 for p in (0, 1, 2, 4, 5, 6))


def test_long_rollouts_stay_finite_and_need_few_passes():
    o = Body(2048, 4, np.float64, solver=1)
    o.reset()
    obs, rew, done = o.rollout(1000, nthreads=8)
    st = o.stats()
    assert st["nonfinite"] == 0 and st["episodes"] == 2048 and np.isfinite(obs).all()
    mean = st["return_sum"] / st["episodes"]
    assert -215 < mean < -185                      # action cost alone is -200 in expectation
    assert np.abs(obs[..., 8:]).max() < 100 and obs[..., 0].max() < 3.0
    # a smaller joint regulariser than the penalty model needs (0.1) is enough here
    o2 = Body(512, 4, np.float64, solver=1, armature=0.02)
    o2.reset()
    o2.rollout(1000, nthreads=8, want_obs=False)
    assert o2.stats()["nonfinite"] == 0


def test_float32_instantiation_tracks_float64_for_one_step():
    a64 = Body(256, 6, np.float64, solver=1); a64.reset()
    a64.rollout(30, nthreads=4, want_obs=False)
    s = a64.get_state().astype(np.float32)
    a32 = Body(256, 6, np.float32, solver=1); a32.set_state(s); a32.step_count = 30
    a64.set_state(s.astype(np.float64))
    o32, _, _ = a32.rollout(1, nthreads=4)
    o64, _, _ = a64.rollout(1, nthreads=4)
    err = np.abs(o32[0].astype(np.float64) - o64[0]).max(axis=1) / np.maximum(np.abs(o64[0]).max(axis=1), 1.0)
    assert np.median(err) < 2e-5 and np.quantile(err, 0.9) < 1e-3
