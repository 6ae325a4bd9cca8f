"""Pins for the CartPole oracle (CPU only)."""
import math

import numpy as np

from oracle.cartpole_binding import CartPole, accel, sin_poly, cos_poly
from oracle import oracle as orc

MC, MP, L, G = 1.0, 0.1, 0.5, 9.8
M = MC + MP


def test_polynomials_match_libm_on_the_working_range():
    for x in np.linspace(-0.5, 0.5, 2001):
        x = float(np.float32(x))
        assert abs(sin_poly(x) - math.sin(x)) < 1.5e-7
        assert abs(cos_poly(x) - math.cos(x)) < 1.5e-7
    assert sin_poly(0.0) == 0.0 and cos_poly(0.0) == 1.0
    assert sin_poly(-0.2) == -sin_poly(0.2) and cos_poly(-0.2) == cos_poly(0.2)


def test_upright_closed_form():
    # theta = thetadot = 0: temp = F/M, thetaacc = -(F/M) / (l (4/3 - mp/M)), xacc = temp - mp l thetaacc / M
    for F in (10.0, -10.0):
        xa, ta = accel(0.0, 0.0, F)
        want_t = -(F / M) / (L * (4.0 / 3.0 - MP / M))
        want_x = F / M - MP * L * want_t / M
        assert abs(ta - want_t) < 2e-6 * abs(want_t) and abs(xa - want_x) < 2e-6 * abs(want_x)
    # pushing right accelerates the cart right and tips the pole left (negative angle)
    assert accel(0.0, 0.0, 10.0)[0] > 0 > accel(0.0, 0.0, 10.0)[1]


def test_equations_satisfy_the_lagrangian_form_and_power_balance():
    # the cart-pole equations of motion in matrix form (uniform pole of length 2l pivoting on the
    # cart):  [M, mp l c; mp l c, (4/3) mp l^2] [xacc; thacc] = [F + mp l thd^2 s; mp g l s]
    # and dE/dt = F xdot for E = 1/2 M xd^2 + mp l xd thd c + 2/3 mp l^2 thd^2 + mp g l c
    rng = np.random.default_rng(0)
    for _ in range(200):
        th, thd, xd = (float(np.float32(v)) for v in (rng.uniform(-0.21, 0.21), rng.uniform(-3, 3), rng.uniform(-3, 3)))
        F = 10.0 if rng.random() < 0.5 else -10.0
        xa, ta = accel(th, thd, F)
        s, c = math.sin(th), math.cos(th)
        r1 = M * xa + MP * L * c * ta - (F + MP * L * thd * thd * s)
        r2 = MP * L * c * xa + (4.0 / 3.0) * MP * L * L * ta - MP * G * L * s
        assert abs(r1) < 2e-5 and abs(r2) < 2e-5
        dE = M * xd * xa + MP * L * (xa * thd * c + xd * ta * c - xd * thd * thd * s) \
            + (4.0 / 3.0) * MP * L * L * thd * ta - MP * G * L * s * thd
        assert abs(dE - F * xd) < 1e-4 * max(1.0, abs(F * xd))


def test_euler_update_termination_truncation_and_reset():
    n, seed, T = 64, 5, 700
    c = CartPole(n, seed, max_steps=500)
    obs0 = c.reset()
    assert np.abs(obs0).max() <= 0.05 and np.abs(obs0).max() > 0.04
    for i in range(4):
        w = orc.draw_block(seed, i, 0, 16)
        want = [np.float32(-0.05) + np.float32(0.1) * np.float32((x >> 8) / 2 ** 24) for x in w]
        assert obs0[i].tolist() == [float(v) for v in want]
    obs, rew, done = c.rollout(T)
    prev = np.concatenate([obs0[None], obs[:-1]])
    assert np.all(rew == 1.0)
    live = done == 0
    # semi-explicit Euler of the benchmark: positions advance with the OLD velocities
    assert np.all(obs[..., 0][live] == (prev[..., 0] + np.float32(0.02) * prev[..., 1])[live])
    assert np.all(obs[..., 2][live] == (prev[..., 2] + np.float32(0.02) * prev[..., 3])[live])
    acts = np.array([[orc.draw_block(seed, i, t, 0)[0] >> 31 for i in range(n)] for t in range(T)])
    for t, i in [(0, 0), (3, 5), (40, 17)]:
        if done[t, i]:
            continue
        xa, ta = accel(float(prev[t, i, 2]), float(prev[t, i, 3]), 10.0 if acts[t, i] else -10.0)
        assert obs[t, i, 1] == np.float32(prev[t, i, 1]) + np.float32(0.02) * np.float32(xa)
        assert obs[t, i, 3] == np.float32(prev[t, i, 3]) + np.float32(0.02) * np.float32(ta)
    # live states are inside the bounds; after done the obs is a fresh initial state
    assert np.abs(obs[..., 0][live]).max() <= 2.4 and np.abs(obs[..., 2][live]).max() <= 0.20943951 + 1e-7
    assert np.abs(obs[done == 1]).max() <= 0.05
    st = c.stats()
    ends = int(done.sum())
    assert st["episodes"] == ends > 500
    assert 15 < st["length_sum"] / st["episodes"] < 30          # random policy: about 22 steps
    assert st["length_min"] >= 7
    # truncation: a tiny limit ends every episode at exactly that length
    d = CartPole(8, 1, max_steps=5); d.reset()
    _, _, dn = d.rollout(20)
    assert np.array_equal(np.flatnonzero(dn[:, 0]), [4, 9, 14, 19]) and d.stats()["length_max"] == 5


def test_structure_batch_independence_and_threads():
    a = CartPole(16, 9); a.reset()
    b = CartPole(200, 9); b.reset()
    oa, _, da = a.rollout(300)
    ob, _, db = b.rollout(300, nthreads=4)
    assert np.array_equal(oa, ob[:, :16]) and np.array_equal(da, db[:, :16])
    c = CartPole(16, 9); c.reset()
    o1, _, _ = c.rollout(120); o2, _, _ = c.rollout(180)
    assert np.array_equal(np.concatenate([o1, o2]), oa)
    acts = np.array([[orc.draw_block(9, i, t, 0)[0] >> 31 for i in range(16)] for t in range(300)], np.uint8)
    e = CartPole(16, 9); e.reset()
    oe, _, _ = e.rollout(300, actions=acts)
    assert np.array_equal(oe, oa)
    f = CartPole(16, 9); f.reset()
    of, _, _ = f.rollout(300, actions=np.where(acts == 1, 1, 7).astype(np.uint8))   # any code but 1 = left
    assert np.array_equal(of, oa)
