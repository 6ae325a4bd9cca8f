"""Pins for the oracle's Pong dynamics (CPU only): hand-traced single steps, invariants, closed
forms and structural properties.  Expected values in the hand-traced cases are worked out by hand
from the rules of the benchmark configuration, not produced by any implementation."""
import numpy as np
import pytest

from oracle import oracle as orc

f32 = np.float32


def S(**kw):
    base = dict(bx=79.0, by=104.0, vx=3.0, vy=0.0, pa=97.0, po=97.0, sa=0, so=0, ep_ret=0, ep_len=0)
    base.update(kw)
    return base


# ----------------------------------------------------------------------------- hand-traced steps

def test_trace_free_flight_no_event():
    # opponent: ball centre 105 == paddle centre 105 -> stays; ball (79,104)+(3,0.5)
    s, r, d, _, _ = orc.pong_step_one(S(vy=0.5), 0, -3.0, 1.0)
    assert (s["bx"], s["by"], s["vx"], s["vy"]) == (82.0, 104.5, 3.0, 0.5)
    assert (s["pa"], s["po"], s["sa"], s["so"]) == (97.0, 97.0, 0, 0)
    assert (r, d, s["ep_ret"], s["ep_len"]) == (0.0, 0, 0, 1)


def test_trace_top_wall_and_opponent_speed_limit():
    # by 1 - 1.5 = -0.5 -> mirrored to 0.5, vy 1.5; opponent wants -103, moves -3
    s, r, d, _, _ = orc.pong_step_one(S(bx=60.0, by=1.0, vx=-3.0, vy=-1.5), 0, 3.0, 0.0)
    assert (s["bx"], s["by"], s["vx"], s["vy"]) == (57.0, 0.5, -3.0, 1.5)
    assert s["po"] == 94.0 and r == 0.0 and d == 0


def test_trace_bottom_wall():
    # 207.5 + 1.25 = 208.75 > 208 -> 416 - 208.75 = 207.25, vy -1.25; opponent +3
    s, r, _, _, _ = orc.pong_step_one(S(bx=60.0, by=207.5, vx=3.0, vy=1.25), 0, 3.0, 0.0)
    assert (s["bx"], s["by"], s["vy"]) == (63.0, 207.25, -1.25)
    assert s["po"] == 100.0 and r == 0.0


def test_trace_agent_hit_offset_minus_three_uses_moved_paddle():
    # action 1 moves the paddle 104 -> 100 first.  Ball 136 -> 139: 141 >= 140 and 139 <= 144;
    # rows 104..106 vs paddle 100..116 overlap.  offset = (104+1) - (100+8) = -3.
    s, r, d, _, _ = orc.pong_step_one(S(bx=136.0, pa=104.0), 1, 3.0, 0.0)
    assert s["pa"] == 100.0
    assert (s["bx"], s["vx"]) == (138.0, -3.0)
    assert f32(s["vy"]) == f32(0.2) * f32(-3.0)
    assert f32(s["vy"]) == f32(-0.6)          # 0.2f * 3 rounds to the float nearest 0.6
    assert r == 0.0 and d == 0


def test_trace_agent_hit_edge_touch_counts():
    # ball bottom edge exactly on paddle top edge: by + 2 == pa -> hit (>=); offset = 99 - 108 = -9
    s, r, _, _, _ = orc.pong_step_one(S(bx=137.0, by=98.0, pa=100.0), 0, 3.0, 0.0)
    assert s["vx"] == -3.0 and s["bx"] == 138.0
    assert f32(s["vy"]) == f32(0.2) * f32(-9.0)
    # one unit higher: no contact, ball flies on
    s, r, _, _, _ = orc.pong_step_one(S(bx=137.0, by=97.0, pa=100.0), 0, 3.0, 0.0)
    assert s["vx"] == 3.0 and s["bx"] == 140.0 and r == 0.0


def test_trace_opponent_hit():
    # opponent 45 -> wants +4 (57-53), moves +3 -> 48; ball 22 -> 19: 19 <= 20 and 21 >= 16;
    # rows 56..58 vs 48..64; offset = 57 - 56 = 1 -> vy = 0.2f
    s, r, _, _, _ = orc.pong_step_one(S(bx=22.0, by=56.0, vx=-3.0, po=45.0), 0, 3.0, 0.0)
    assert s["po"] == 48.0
    assert (s["bx"], s["vx"]) == (20.0, 3.0)
    assert f32(s["vy"]) == f32(0.2)
    assert r == 0.0


def test_trace_agent_miss_scores_for_opponent_and_reserves():
    # paddle far away (150..166 vs ball rows 10..12).  157 -> 160; 162 > 160 -> reward -1.
    s, r, d, _, _ = orc.pong_step_one(S(bx=157.0, by=10.0, pa=150.0, ep_ret=-2, ep_len=40), 0,
                                      -3.0, 1.25)
    assert r == -1.0 and d == 0
    assert (s["sa"], s["so"]) == (0, 1)
    assert (s["bx"], s["by"], s["vx"], s["vy"]) == (79.0, 104.0, -3.0, 1.25)
    assert s["pa"] == 150.0          # paddles keep their place after a point
    assert s["po"] == 94.0           # opponent chased the old ball: -3
    assert (s["ep_ret"], s["ep_len"]) == (-3, 41)


def test_trace_right_edge_is_not_a_score_until_crossed():
    s, r, _, _, _ = orc.pong_step_one(S(bx=155.0, by=10.0, pa=150.0), 0, -3.0, 0.0)
    assert s["bx"] == 158.0 and r == 0.0          # 158 + 2 == 160: still in the field
    s, r, _, _, _ = orc.pong_step_one(s, 0, -3.0, 0.0)
    assert r == -1.0


def test_trace_agent_scores():
    # opponent paddle far below (150..166); ball 2 -> -1 < 0 -> reward +1
    s, r, d, _, _ = orc.pong_step_one(S(bx=2.0, by=10.0, vx=-3.0, po=153.0), 2, 3.0, -0.5)
    assert r == 1.0 and (s["sa"], s["so"]) == (1, 0) and d == 0
    assert (s["bx"], s["by"], s["vx"], s["vy"]) == (79.0, 104.0, 3.0, -0.5)
    assert s["pa"] == 101.0 and s["po"] == 150.0


def test_trace_twenty_first_point_ends_episode_and_resets():
    s, r, d, fr, fl = orc.pong_step_one(
        S(bx=157.0, by=10.0, pa=150.0, po=30.0, sa=4, so=20, ep_ret=-16, ep_len=900), 0, 3.0, 0.75)
    assert r == -1.0 and d == 1
    assert (fr, fl) == (-17, 901)
    assert (s["sa"], s["so"], s["pa"], s["po"]) == (0, 0, 97.0, 97.0)
    assert (s["bx"], s["by"], s["vx"], s["vy"]) == (79.0, 104.0, 3.0, 0.75)
    assert (s["ep_ret"], s["ep_len"]) == (0, 0)


def test_trace_paddle_clamps_and_unknown_action():
    s, *_ = orc.pong_step_one(S(pa=2.0), 1, 3.0, 0.0)
    assert s["pa"] == 0.0
    s, *_ = orc.pong_step_one(S(pa=192.0), 2, 3.0, 0.0)
    assert s["pa"] == 194.0
    s, *_ = orc.pong_step_one(S(pa=50.0), 7, 3.0, 0.0)
    assert s["pa"] == 50.0
    s, *_ = orc.pong_step_one(S(by=0.0, vy=0.0, po=1.0), 0, 3.0, 0.0)
    assert s["po"] == 0.0            # 1 - 3 clamped at the top
    s, *_ = orc.pong_step_one(S(by=208.0, vy=0.0, po=193.0), 0, 3.0, 0.0)
    assert s["po"] == 194.0


def test_trace_batch_of_four_matches_single_calls():
    # the batch driver applies the same transition with the step's Philox draws
    seed = 11
    p = orc.Pong(4, seed, max_score=21)
    e = p.envs()
    before = [{k: e[k][i].item() for k in e.dtype.names} for i in range(4)]
    L = orc.lib()
    obs, rew, done = p.step()
    for i in range(4):
        w = orc.draw_block(seed, i, 0, 0)
        s, r, d, _, _ = orc.pong_step_one(before[i], L.oracle_pong_action(w[0]),
                                          L.oracle_pong_serve_vx(w[1]), L.oracle_pong_serve_vy(w[2]))
        want = [s["bx"], s["by"], s["vx"], s["vy"], s["pa"], s["po"], s["sa"], s["so"]]
        assert obs[i].tolist() == [float(f32(x)) for x in want]
        assert rew[i] == r and done[i] == d


def test_reset_state():
    p = orc.Pong(8, 3)
    obs = p.reset()
    L = orc.lib()
    for i in range(8):
        w = orc.draw_block(3, i, 0, 16)
        assert obs[i].tolist() == [79.0, 104.0, L.oracle_pong_serve_vx(w[1]),
                                   L.oracle_pong_serve_vy(w[2]), 97.0, 97.0, 0.0, 0.0]


# ----------------------------------------------------------------------------- invariants

@pytest.fixture(scope="module", params=[(21, 3000), (2, 1500)])
def traj(request):
    max_score, T = request.param
    n = 192
    p = orc.Pong(n, 1234 + max_score, max_score=max_score)
    obs0 = p.reset()
    obs, rew, done = p.rollout(T)
    return dict(max_score=max_score, T=T, n=n, obs0=obs0, obs=obs, rew=rew, done=done,
                stats=p.stats())


def test_bounds(traj):
    o = traj["obs"]
    assert o[..., 4].min() >= 0 and o[..., 4].max() <= 194
    assert o[..., 5].min() >= 0 and o[..., 5].max() <= 194
    assert o[..., 1].min() >= 0 and o[..., 1].max() <= 208
    assert o[..., 0].min() >= 0 and o[..., 0].max() <= 158
    assert set(np.unique(np.abs(o[..., 2]))) == {3.0}
    assert np.abs(o[..., 3]).max() <= 2.0


def _prev(traj):
    return np.concatenate([traj["obs0"][None], traj["obs"][:-1]], axis=0)


def test_reflection_and_free_flight_steps(traj):
    o, p, rew = traj["obs"], _prev(traj), traj["rew"]
    quiet = (rew == 0) & (o[..., 2] == p[..., 2])          # no point, no paddle hit
    assert quiet.mean() > 0.9
    assert np.all(o[..., 0][quiet] == (p[..., 0] + p[..., 2])[quiet])
    raw = p[..., 1] + p[..., 3]                            # float32 add, as the step does
    top, bot = quiet & (raw < 0), quiet & (raw > 208)
    mid = quiet & ~(raw < 0) & ~(raw > 208)
    assert top.sum() > 5 and bot.sum() > 5          # walls are rarely reached: |vy| <= 2
    assert np.all(o[..., 1][mid] == raw[mid]) and np.all(o[..., 3][mid] == p[..., 3][mid])
    assert np.all(o[..., 1][top] == -raw[top]) and np.all(o[..., 3][top] == -p[..., 3][top])
    assert np.all(o[..., 1][bot] == (f32(416.0) - raw)[bot])
    assert np.all(o[..., 3][bot] == -p[..., 3][bot])


def test_paddle_hit_closed_form(traj):
    o, p, rew = traj["obs"], _prev(traj), traj["rew"]
    hit = (rew == 0) & (o[..., 2] == -p[..., 2])
    assert hit.sum() > 100
    agent = hit & (p[..., 2] > 0)
    opp = hit & (p[..., 2] < 0)
    assert agent.sum() > 10 and opp.sum() > 10
    assert np.all(o[..., 0][agent] == 138.0) and np.all(o[..., 0][opp] == 20.0)
    off_a = (o[..., 1] + f32(1)) - (o[..., 4] + f32(8))
    off_o = (o[..., 1] + f32(1)) - (o[..., 5] + f32(8))
    assert np.all(o[..., 3][agent] == (f32(0.2) * off_a)[agent])
    assert np.all(o[..., 3][opp] == (f32(0.2) * off_o)[opp])
    assert np.abs(off_a[agent]).max() <= 9 and np.abs(off_o[opp]).max() <= 9
    assert np.abs(o[..., 3][hit]).max() <= 1.8 + 1e-6


def test_score_bookkeeping(traj):
    o, p, rew, done = traj["obs"], _prev(traj), traj["rew"], traj["done"]
    ms = traj["max_score"]
    assert set(np.unique(rew)) <= {-1.0, 0.0, 1.0}
    assert set(np.unique(done)) <= {0, 1}
    sa, so, psa, pso = o[..., 6], o[..., 7], p[..., 6], p[..., 7]
    live = done == 0
    assert np.all((sa - psa)[live] == (rew == 1)[live])
    assert np.all((so - pso)[live] == (rew == -1)[live])
    # on the terminal transition the pre-reset score reached max_score and obs shows the new episode
    term = done == 1
    assert np.all(rew[term] != 0)
    reached = np.where(rew == 1, psa + 1, psa)[term] == ms
    reached |= np.where(rew == -1, pso + 1, pso)[term] == ms
    assert np.all(reached)
    assert np.all(sa[term] == 0) and np.all(so[term] == 0)
    assert np.all(o[..., 4][term] == 97) and np.all(o[..., 5][term] == 97)
    assert np.all(np.maximum(sa, so) < ms)
    # after every point the ball is re-served from the centre
    pt = rew != 0
    assert np.all(o[..., 0][pt] == 79) and np.all(o[..., 1][pt] == 104)
    # episode statistics recomputed from (reward, done) alone
    episodes = 0; ret_sum = 0; len_sum = 0; rmin, rmax = 10 ** 9, -10 ** 9
    for i in range(traj["n"]):
        ends = np.flatnonzero(done[:, i])
        start = 0
        for e_ in ends:
            ret = int(rew[start:e_ + 1, i].sum())
            episodes += 1; ret_sum += ret; len_sum += e_ + 1 - start
            rmin, rmax = min(rmin, ret), max(rmax, ret)
            # sum of rewards over the episode equals the final score difference
            fa = psa[e_, i] + (rew[e_, i] == 1); fo = pso[e_, i] + (rew[e_, i] == -1)
            assert ret == int(fa - fo)
            start = e_ + 1
    st = traj["stats"]
    if ms == 2:
        assert episodes > 1000
    assert st["episodes"] == episodes and st["return_sum"] == ret_sum
    assert st["length_sum"] == len_sum
    if episodes:
        assert st["return_min"] == rmin and st["return_max"] == rmax


def test_free_flight_closed_form_from_serve():
    # From a serve, until the first paddle/point event: bx = 79 + k vx exactly, and by is the
    # triangle-wave fold of 104 + k vy (period 416) to within accumulated rounding.
    p = orc.Pong(256, 77)
    obs0 = p.reset()
    obs, rew, done = p.rollout(24)
    vx0, vy0 = obs0[:, 2].astype(np.float64), obs0[:, 3].astype(np.float64)
    checked = 0
    for k in range(1, 19):                       # 79 +- 3k stays between the paddles for k <= 18
        o = obs[k - 1]
        assert np.all(o[:, 0] == 79 + k * vx0)
        y = (104 + k * vy0) % 416
        fold = np.where(y > 208, 416 - y, y)
        assert np.abs(o[:, 1] - fold).max() <= k * 2.0 ** -16
        checked += 1
    assert checked == 18


# ----------------------------------------------------------------------------- structural

def test_env_trajectory_independent_of_batch_size():
    a = orc.Pong(16, 5, max_score=3); a.reset()
    b = orc.Pong(300, 5, max_score=3); b.reset()
    oa, ra, da = a.rollout(800)
    ob, rb, db = b.rollout(800)
    assert np.array_equal(oa, ob[:, :16]) and np.array_equal(ra, rb[:, :16])
    assert np.array_equal(da, db[:, :16])
    assert da.sum() > 0


def test_step_by_step_equals_rollout_and_threads_equal_serial():
    a = orc.Pong(37, 8, max_score=2); a.reset()
    b = orc.Pong(37, 8, max_score=2); b.reset()
    c = orc.Pong(37, 8, max_score=2); c.reset()
    oa, ra, da = a.rollout(400)
    oc, rc, dc = c.rollout(400, nthreads=5)
    for t in range(400):
        o, r, d = b.step()
        assert np.array_equal(o, oa[t]) and np.array_equal(r, ra[t]) and np.array_equal(d, da[t])
    assert np.array_equal(oa, oc) and np.array_equal(ra, rc) and np.array_equal(da, dc)
    assert a.stats() == b.stats() == c.stats()
    assert a.step_count == b.step_count == c.step_count == 400


def test_save_restore_mid_rollout_is_invisible():
    a = orc.Pong(20, 9, max_score=2); a.reset()
    full = a.rollout(300)
    b = orc.Pong(20, 9, max_score=2); b.reset()
    first = b.rollout(150)
    snap, step = b.envs().copy(), b.step_count
    c2 = orc.Pong(20, 9, max_score=2)
    c2.envs()[:] = snap
    c2.step_count = step
    second = c2.rollout(150)
    for k in range(3):
        assert np.array_equal(full[k][:150], first[k])
        assert np.array_equal(full[k][150:], second[k])


def test_external_actions_equal_internal_draws():
    L = orc.lib()
    n, T, seed = 9, 200, 21
    acts = np.array([[L.oracle_pong_action(orc.draw_block(seed, i, t, 0)[0]) for i in range(n)]
                     for t in range(T)], np.uint8)
    a = orc.Pong(n, seed, max_score=2); a.reset()
    b = orc.Pong(n, seed, max_score=2); b.reset()
    ra = a.rollout(T)
    rb = b.rollout(T, actions=acts)
    for k in range(3):
        assert np.array_equal(ra[k], rb[k])
    # and a different action stream gives a different trajectory
    c = orc.Pong(n, seed, max_score=2); c.reset()
    rc = c.rollout(T, actions=np.zeros((T, n), np.uint8))
    assert not np.array_equal(ra[0], rc[0])
    assert np.all(rc[0][..., 4] == 97)            # "stay" never moves the agent paddle


def test_opponent_is_beatable_and_agent_random_play_loses():
    # sanity of the game's balance under uniform random actions: the agent loses most episodes,
    # the opponent still concedes points (so both reward signs occur)
    p = orc.Pong(128, 4); p.reset()
    _, rew, done = p.rollout(4000)
    assert (rew == 1).sum() > 0 and (rew == -1).sum() > (rew == 1).sum()
    st = p.stats()
    assert st["episodes"] > 100 and st["return_max"] < 0


def test_oracle_arithmetic_is_frozen_by_the_committed_digest():
    # tests/golden/pong_oracle_digest.txt is written by tests/golden/make_pong_digest.py from the
    # oracle alone; a change to the oracle's arithmetic must regenerate it on purpose
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_pong_digest",
                                                  os.path.join(here, "golden", "make_pong_digest.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    want = {}
    for line in open(os.path.join(here, "golden", "pong_oracle_digest.txt")):
        if "sha256=" in line:
            parts = dict(kv.split("=") for kv in line.split())
            want[int(parts["max_score"])] = parts
    for ms in (21, 2):
        d, obs, rew, done, st = mod.digest(ms)
        assert d == want[ms]["sha256"]
        assert st["episodes"] == int(want[ms]["episodes"])
        assert st["return_sum"] == int(want[ms]["return_sum"])


def test_normalised_observations_ranges_and_inverse():
    """Observation scaling at the source (paper App. B.1 item 8): same trajectories, each component
    mapped into [0,1] or [-1,1] by one float32 multiplication; extremes are reached exactly, and
    undoing the scaling in float64 returns the raw observation to within the two float32 roundings
    made (reciprocal, product): relative error <= 2 * 2^-24."""
    n, T = 256, 3000
    raw = orc.Pong(n, 31, max_score=3)
    nor = orc.Pong(n, 31, max_score=3, normalize=True)
    r0, n0 = raw.reset(), nor.reset()
    ro, rr, rd = raw.rollout(T, nthreads=4)
    no, nr, nd = nor.rollout(T, nthreads=4)
    assert np.array_equal(rr, nr) and np.array_equal(rd, nd)          # dynamics untouched
    for k in (0, 1, 4, 5, 6, 7):
        assert no[..., k].min() >= 0.0 and no[..., k].max() <= 1.0, k
    for k in (2, 3):
        assert no[..., k].min() >= -1.0 and no[..., k].max() <= 1.0, k
    assert set(np.unique(no[..., 2])) == {np.float32(-1.0), np.float32(1.0)}
    top = np.float32(194) * (np.float32(1) / np.float32(194))        # one ulp below 1: a product, not a quotient
    assert no[..., 4].max() == top and no[..., 4].min() == 0.0        # paddle clamps hit both ends
    assert no[..., 6].max() < 1.0 and no[..., 6].max() == np.float32(2) * (np.float32(1) / np.float32(3))
    ranges = np.array([158, 208, 3, 2, 194, 194, 3, 3], np.float64)
    back = no.astype(np.float64) * ranges
    assert (np.abs(back - ro) <= 2.0 ** -23 * np.abs(ro.astype(np.float64))).all()
    assert np.abs(back - ro).max() > 0.0                               # and the bound is not vacuous
    assert np.array_equal(n0[:, 4], np.full(n, np.float32(97) * (np.float32(1) / np.float32(194))))
    assert np.array_equal(r0[:, 2] * (np.float32(1) / np.float32(3)), n0[:, 2])
