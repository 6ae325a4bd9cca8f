"""GPU parity: Pong with vector observations, HIP path vs CPU oracle, bit for bit.
Every call goes through the C-ABI (paper_2603_12145_amd.binding is marshalling only)."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import oracle as orc                      # noqa: E402
from paper_2603_12145_amd import binding as b         # noqa: E402
from paper_2603_12145_amd import inputs               # noqa: E402
from gpu_helpers import assert_bit_equal, split_state, pong_state_fields, pong_blob  # noqa: E402

DEV = "cuda:0"


def bufs(T, n, obs_dim=8):
    return (torch.empty((T, n, obs_dim), dtype=torch.float32, device=DEV),
            torch.empty((T, n), dtype=torch.float32, device=DEV),
            torch.empty((T, n), dtype=torch.uint8, device=DEV))


def gpu_rollout(n, seed, T, max_score=21, actions=None, per_step=False):
    h = b.env_create(b.ENV_PONG, n, seed, {"max_score": max_score})
    try:
        obs0 = torch.empty((n, 8), dtype=torch.float32, device=DEV)
        b.env_reset(h, obs0)
        obs, rew, done = bufs(T, n)
        act = None if actions is None else torch.from_numpy(actions).to(DEV)
        if per_step:
            for t in range(T):
                b.env_step(h, None if act is None else act[t], obs[t], rew[t], done[t])
        else:
            b.env_rollout(h, T, act, obs, rew, done)
        torch.cuda.synchronize()
        out = dict(obs0=obs0.cpu().numpy(), obs=obs.cpu().numpy(), rew=rew.cpu().numpy(),
                   done=done.cpu().numpy(), stats=b.env_stats(h), state=b.env_get_state(h),
                   steps=b.env_step_count(h))
    finally:
        b.env_destroy(h)
    return out


def oracle_rollout(n, seed, T, max_score=21, actions=None, nthreads=8):
    p = orc.Pong(n, seed, max_score=max_score)
    obs0 = p.reset()
    obs, rew, done = p.rollout(T, actions=actions, nthreads=nthreads)
    return dict(obs0=obs0, obs=obs, rew=rew, done=done, stats=p.stats(),
                state=pong_state_fields(p.envs()), steps=p.step_count)


def compare(g, o, n, what):
    assert_bit_equal(g["obs0"], o["obs0"], what + " reset obs")
    assert_bit_equal(g["obs"], o["obs"], what + " obs")
    assert_bit_equal(g["rew"], o["rew"], what + " reward")
    assert_bit_equal(g["done"], o["done"], what + " done")
    step, fields = split_state(g["state"], n, 10)
    assert step == o["steps"] == g["steps"]
    assert_bit_equal(fields, o["state"], what + " final state")
    gs, os_ = g["stats"], o["stats"]
    assert gs["episodes"] == os_["episodes"] and gs["length_sum"] == os_["length_sum"]
    assert gs["return_sum"] == os_["return_sum"]
    if os_["episodes"]:
        assert gs["return_min"] == os_["return_min"] and gs["return_max"] == os_["return_max"]
    else:
        assert gs["return_min"] == float("inf") and gs["return_max"] == float("-inf")


@pytest.mark.parametrize("per_step", [False, True])
@pytest.mark.parametrize("max_score", [21, 2])
def test_config0_n64_t1000(per_step, max_score):
    g = gpu_rollout(64, 0, 1000, max_score, per_step=per_step)
    o = oracle_rollout(64, 0, 1000, max_score)
    compare(g, o, 64, "C0 per_step=%s max_score=%d" % (per_step, max_score))
    if max_score == 2:
        assert o["stats"]["episodes"] > 300


@pytest.mark.parametrize("n", [1, 3, 63, 65, 1000, 1003, 4100])
def test_ragged_and_tiny_batches(n):
    g = gpu_rollout(n, 17, 300, 2)
    o = oracle_rollout(n, 17, 300, 2)
    compare(g, o, n, "ragged n=%d" % n)


def test_external_actions_including_out_of_range_codes():
    n, T = 333, 400
    acts = inputs.pong_actions(T, n, seed=5)
    g = gpu_rollout(n, 23, T, 3, actions=acts)
    o = oracle_rollout(n, 23, T, 3, actions=acts)
    compare(g, o, n, "external actions rollout")
    g2 = gpu_rollout(n, 23, T, 3, actions=acts, per_step=True)
    compare(g2, o, n, "external actions per step")


def test_env_i_is_independent_of_batch_size():
    a = gpu_rollout(64, 5, 500, 3)
    c = gpu_rollout(4096, 5, 500, 3)
    assert_bit_equal(a["obs"], c["obs"][:, :64], "N independence obs")
    assert_bit_equal(a["done"], c["done"][:, :64], "N independence done")


def test_save_restore_and_split_rollouts():
    n, seed = 500, 31
    full = gpu_rollout(n, seed, 600, 2)
    h = b.env_create(b.ENV_PONG, n, seed, {"max_score": 2})
    b.env_reset(h, None)
    o1, r1, d1 = bufs(250, n)
    b.env_rollout(h, 250, None, o1, r1, d1)
    blob = b.env_get_state(h)
    b.env_destroy(h)
    h2 = b.env_create(b.ENV_PONG, n, seed, {"max_score": 2})
    b.env_set_state(h2, blob)                      # no env_reset: set_state marks it as reset
    o2, r2, d2 = bufs(350, n)
    b.env_rollout(h2, 350, None, o2, r2, d2)
    torch.cuda.synchronize()
    assert b.env_step_count(h2) == 600
    b.env_destroy(h2)
    assert_bit_equal(full["obs"][:250], o1.cpu().numpy(), "first part")
    assert_bit_equal(full["obs"][250:], o2.cpu().numpy(), "second part")
    assert_bit_equal(full["done"][250:], d2.cpu().numpy(), "second part done")
    assert_bit_equal(full["rew"][250:], r2.cpu().numpy(), "second part reward")


def test_set_state_from_oracle_state_then_step():
    # hand the GPU a state produced by the oracle mid-rollout; both continue identically
    n, seed = 130, 77
    p = orc.Pong(n, seed, max_score=2); p.reset(); p.rollout(123)
    blob = pong_blob(p.step_count, pong_state_fields(p.envs()))
    h = b.env_create(b.ENV_PONG, n, seed, {"max_score": 2})
    b.env_set_state(h, blob)
    obs, rew, done = bufs(200, n)
    b.env_rollout(h, 200, None, obs, rew, done)
    torch.cuda.synchronize()
    b.env_destroy(h)
    oo, orr, od = p.rollout(200)
    assert_bit_equal(obs.cpu().numpy(), oo, "obs after set_state")
    assert_bit_equal(rew.cpu().numpy(), orr, "reward after set_state")
    assert_bit_equal(done.cpu().numpy(), od, "done after set_state")


@pytest.mark.parametrize("pace", [-1, 6600])
@pytest.mark.parametrize("T,external", [(1, False), (5, False), (64, False), (203, False), (203, True)])
def test_states_outside_the_games_own_reach(T, external, pace):
    # States a game never produces, planted in the oracle's records and handed to the GPU: a ball
    # far faster than a serve, outside the field, scores one short of the end, and a return / length
    # so far that do not match the scores.  The episode bookkeeping (return and length of every
    # finished episode, statistics, the state blob) must still agree with the oracle exactly.
    n, seed, max_score = 200, 31, 2
    p = orc.Pong(n, seed, max_score=max_score); p.reset(); p.rollout(17)
    e = p.envs()
    rng = np.random.default_rng(5)
    e["vx"][:] = rng.choice(np.array([-90.0, -60.0, -3.0, 3.0, 7.5, 60.0, 200.0], np.float32), n)
    e["bx"][::7] = -40.0
    e["bx"][3::7] = 400.0
    e["sa"][:] = rng.integers(0, max_score, n)
    e["so"][:] = rng.integers(0, max_score, n)
    e["ep_ret"][:] = rng.integers(-1000, 1000, n)
    e["ep_len"][:] = rng.integers(0, 1 << 20, n)
    blob = pong_blob(p.step_count, pong_state_fields(e))
    actions = inputs.pong_actions(T, n, 8) if external else None
    h = b.env_create(b.ENV_PONG, n, seed, {"max_score": max_score})
    b.env_set_state(h, blob)
    obs, rew, done = bufs(T, n)
    assert b.lib().mi355env_tune_rollout_pace(pace) == 0
    try:
        b.env_rollout(h, T, None if actions is None else torch.from_numpy(actions).to(DEV), obs, rew, done)
        torch.cuda.synchronize()
    finally:
        assert b.lib().mi355env_tune_rollout_pace(0) == 0
    stats, state = b.env_stats(h), b.env_get_state(h)
    b.env_destroy(h)
    oo, orr, od = p.rollout(T, actions=actions)
    assert_bit_equal(obs.cpu().numpy(), oo, "obs")
    assert_bit_equal(rew.cpu().numpy(), orr, "reward")
    assert_bit_equal(done.cpu().numpy(), od, "done")
    assert od.sum() > 0 or T < 5
    want = p.stats()
    for k in ("episodes", "length_sum", "return_sum"):
        assert stats[k] == want[k], (k, stats[k], want[k])
    if want["episodes"]:
        assert stats["return_min"] == want["return_min"] and stats["return_max"] == want["return_max"]
    step, fields = split_state(state, n, 10)
    assert step == p.step_count
    assert_bit_equal(fields, pong_state_fields(p.envs()), "state blob")


def test_negative_zeros_in_a_restored_state_are_stored_as_positive_zeros():
    # env_set_state stores -0.0 as +0.0 in the float fields (the game never produces a negative
    # zero, and the step's sign-bit tests stand for comparisons with 0).  The GPU given negative
    # zeros must therefore behave exactly like the oracle given the same state with positive ones.
    n, seed, T = 128, 17, 40
    p = orc.Pong(n, seed); p.reset(); p.rollout(9)
    e = p.envs()
    e["by"][::3] = 0.0; e["vy"][::3] = 0.0          # ball resting on the top wall
    e["by"][1::3] = 0.0                             # ... or leaving it
    e["pa"][::5] = 0.0; e["po"][::4] = 0.0
    minus = pong_state_fields(e).copy()
    zeros = minus[:6] == 0
    assert zeros.sum() > n // 2
    minus[:6][zeros] = 0x80000000
    h = b.env_create(b.ENV_PONG, n, seed, None)
    b.env_set_state(h, pong_blob(p.step_count, minus))
    _, stored = split_state(b.env_get_state(h), n, 10)
    assert_bit_equal(stored, pong_state_fields(e), "stored state")
    obs, rew, done = bufs(T, n)
    b.env_rollout(h, T, None, obs, rew, done)
    torch.cuda.synchronize()
    b.env_destroy(h)
    oo, orr, od = p.rollout(T)
    assert_bit_equal(obs.cpu().numpy(), oo, "obs")
    assert_bit_equal(rew.cpu().numpy(), orr, "reward")
    assert_bit_equal(done.cpu().numpy(), od, "done")


def test_the_one_time_pace_measurement_leaves_no_trace():
    # The first long rollout of a batch size in the paced range times a few loops on scratch state
    # and into the caller's output buffers.  Outputs, state and statistics must be those of a
    # library that never measured, and the choice is remembered for the batch size.
    import ctypes as C
    L = b.lib()
    L.mi355env_pace_choice.argtypes = [C.c_int64]
    n, seed, T = 61440 + 64 * 3, 23, 300            # a batch size no other test uses
    outs = []
    for measure in (1, 0):
        assert L.mi355env_tune_measure_pace(measure) == 0
        assert L.mi355env_tune_rollout_pace(0 if measure else -1) == 0
        h = b.env_create(b.ENV_PONG, n, seed, {"max_score": 1})
        b.env_reset(h, None)
        obs, rew, done = bufs(T, n)
        if measure:
            assert L.mi355env_pace_choice(n) == 0
        b.env_rollout(h, T, None, obs, rew, done)
        b.env_rollout(h, T, None, obs, rew, done)       # second launch: the remembered choice
        torch.cuda.synchronize()
        if measure:
            choice = L.mi355env_pace_choice(n)
            assert choice == -1 or 5000 <= choice <= 7000, choice
        outs.append((obs.cpu().numpy(), rew.cpu().numpy(), done.cpu().numpy(), b.env_stats(h),
                     b.env_get_state(h)))
        b.env_destroy(h)
    assert L.mi355env_tune_measure_pace(1) == 0 and L.mi355env_tune_rollout_pace(0) == 0
    for k in range(3):
        assert_bit_equal(outs[0][k], outs[1][k], "output %d with and without the measurement" % k)
    assert outs[0][3] == outs[1][3] and outs[0][3]["episodes"] > 0
    assert np.array_equal(outs[0][4], outs[1][4])


def test_stats_reset_counters():
    h = b.env_create(b.ENV_PONG, 256, 3, {"max_score": 1})
    b.env_reset(h, None)
    obs, rew, done = bufs(400, 256)
    b.env_rollout(h, 400, None, obs, rew, done)
    s1 = b.env_stats(h, reset_counters=True)
    s2 = b.env_stats(h)
    assert s1["episodes"] == int(done.sum().item()) > 0
    assert s2["episodes"] == 0 and s2["length_sum"] == 0 and s2["return_sum"] == 0
    b.env_rollout(h, 400, None, obs, rew, done)
    s3 = b.env_stats(h)
    assert s3["episodes"] == int(done.sum().item())
    b.env_destroy(h)


def test_second_env_reset_uses_current_step_counter():
    n, seed = 70, 9
    h = b.env_create(b.ENV_PONG, n, seed, None)
    obs0 = torch.empty((n, 8), dtype=torch.float32, device=DEV)
    b.env_reset(h, obs0)
    obs, rew, done = bufs(40, n)
    b.env_rollout(h, 40, None, obs, rew, done)
    b.env_reset(h, obs0)
    torch.cuda.synchronize()
    b.env_destroy(h)
    p = orc.Pong(n, seed); p.reset(); p.rollout(40)
    assert_bit_equal(obs0.cpu().numpy(), p.reset(), "second reset obs")


def test_error_paths_touch_nothing():
    n = 128
    h = b.env_create(b.ENV_PONG, n, 1, None)
    obs, rew, done = bufs(4, n)
    obs.fill_(-7.0); rew.fill_(-7.0); done.fill_(9)
    L = b.lib()
    vp = C.c_void_p
    # step before reset
    assert L.env_step(h, None, vp(obs.data_ptr()), vp(rew.data_ptr()), vp(done.data_ptr())) == b.ENV_E_STATE
    b.env_reset(h, None)
    # NULL outputs, T <= 0
    assert L.env_step(h, None, None, vp(rew.data_ptr()), vp(done.data_ptr())) == b.ENV_E_ARG
    assert L.env_step(h, None, vp(obs.data_ptr()), None, vp(done.data_ptr())) == b.ENV_E_ARG
    assert L.env_step(h, None, vp(obs.data_ptr()), vp(rew.data_ptr()), None) == b.ENV_E_ARG
    assert L.env_rollout(h, 0, None, vp(obs.data_ptr()), vp(rew.data_ptr()), vp(done.data_ptr())) == b.ENV_E_ARG
    assert L.env_rollout(h, -3, None, vp(obs.data_ptr()), vp(rew.data_ptr()), vp(done.data_ptr())) == b.ENV_E_ARG
    # misaligned obs / reward
    assert L.env_step(h, None, vp(obs.data_ptr() + 4), vp(rew.data_ptr()), vp(done.data_ptr())) == b.ENV_E_ARG
    assert L.env_step(h, None, vp(obs.data_ptr()), vp(rew.data_ptr() + 2), vp(done.data_ptr())) == b.ENV_E_ARG
    # host memory where device memory is required
    host = np.zeros(n * 8 * 4, np.float32)
    assert L.env_step(h, None, vp(host.ctypes.data), vp(rew.data_ptr()), vp(done.data_ptr())) == b.ENV_E_ARG
    # rollout longer than the buffers: T*n*8 floats do not fit in the allocation
    small = torch.empty((n, 8), dtype=torch.float32, device=DEV)
    big_T = 1 << 20
    assert L.env_rollout(h, big_T, None, vp(small.data_ptr()), vp(rew.data_ptr()), vp(done.data_ptr())) == b.ENV_E_ARG
    # wrong blob size
    blob = b.env_get_state(h)
    assert L.env_set_state(h, vp(blob.ctypes.data), blob.nbytes - 4) == b.ENV_E_ARG
    assert L.env_get_state(h, vp(blob.ctypes.data), blob.nbytes + 4) == b.ENV_E_ARG
    torch.cuda.synchronize()
    assert b.env_step_count(h) == 0
    assert float(obs.min()) == -7.0 == float(obs.max()) and int(done.min()) == 9
    # and the handle still works
    b.env_step(h, None, obs[0], rew[0], done[0])
    torch.cuda.synchronize()
    assert b.env_step_count(h) == 1 and float(obs[0].max()) > 0
    b.env_destroy(h)


def test_sizes_that_would_wrap_are_refused():
    # T * n * bytes-per-env-step beyond 64 bits must not wrap round into a size that passes the
    # buffer check: pixel frames (7056 B) at n = 2^20 and T = 2^31 - 1 are 2^63.8 bytes
    n = 1 << 20
    h = b.env_create(b.ENV_PONG_PIXELS, n, 1, None)
    b.env_reset(h, None)
    L, vp = b.lib(), C.c_void_p
    frames = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    rew = torch.empty(n, dtype=torch.float32, device=DEV)
    done = torch.empty(n, dtype=torch.uint8, device=DEV)
    T = (1 << 31) - 1
    assert L.env_rollout(h, T, None, vp(frames.data_ptr()), vp(rew.data_ptr()), vp(done.data_ptr())) == b.ENV_E_ARG
    torch.cuda.synchronize()
    assert b.env_step_count(h) == 0
    b.env_destroy(h)


def test_non_default_stream():
    n, seed, T = 200, 12, 300
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        h = b.env_create(b.ENV_PONG, n, seed, {"max_score": 2}, stream=s)
        obs, rew, done = bufs(T, n)
        b.env_reset(h, None)
        b.env_rollout(h, T, None, obs, rew, done)
    s.synchronize()
    o = oracle_rollout(n, seed, T, 2)
    assert_bit_equal(obs.cpu().numpy(), o["obs"], "stream obs")
    b.env_destroy(h)


def test_config1_n4096_t10000_one_launch_per_step():
    n, seed, T = 4096, 1, 10000
    h = b.env_create(b.ENV_PONG, n, seed, None)
    b.env_reset(h, None)
    obs, rew, done = bufs(T, n)
    for t in range(T):
        b.env_step(h, None, obs[t], rew[t], done[t])
    torch.cuda.synchronize()
    stats = b.env_stats(h)
    b.env_destroy(h)
    o = oracle_rollout(n, seed, T, 21, nthreads=16)
    assert_bit_equal(obs.cpu().numpy(), o["obs"], "C1 obs")
    assert_bit_equal(rew.cpu().numpy(), o["rew"], "C1 reward")
    assert_bit_equal(done.cpu().numpy(), o["done"], "C1 done")
    assert stats["episodes"] == o["stats"]["episodes"] > 1000
    assert stats["return_sum"] == o["stats"]["return_sum"]


@pytest.mark.parametrize("n", [16384, 65536])
def test_config2_fused_rollout_full_size(n):
    # the launch configuration bench.py times: one env_rollout(T=1000) over N environments, seed 2
    seed, T = 2, 1000
    h = b.env_create(b.ENV_PONG, n, seed, None)
    b.env_reset(h, None)
    obs, rew, done = bufs(T, n)
    b.env_rollout(h, T, None, obs, rew, done)
    torch.cuda.synchronize()
    stats = b.env_stats(h)
    b.env_destroy(h)
    o = oracle_rollout(n, seed, T, 21, nthreads=16)
    assert_bit_equal(rew.cpu().numpy(), o["rew"], "C2 reward")
    assert_bit_equal(done.cpu().numpy(), o["done"], "C2 done")
    assert_bit_equal(obs.cpu().numpy(), o["obs"], "C2 obs")
    assert stats["episodes"] == o["stats"]["episodes"]
    assert stats["return_sum"] == o["stats"]["return_sum"]
    assert stats["length_sum"] == o["stats"]["length_sum"]


def test_config2_largest_sweep_size_sampled():
    # N = 262144 x T = 1000 (9.7 GB of trajectory): compare the first 4096 and the last 4096
    # environments of every step (the oracle computes environment i independently of N), plus the
    # episode statistics of a full oracle run without trajectory storage.
    n, seed, T = 262144, 2, 1000
    h = b.env_create(b.ENV_PONG, n, seed, None)
    b.env_reset(h, None)
    obs, rew, done = bufs(T, n)
    b.env_rollout(h, T, None, obs, rew, done)
    torch.cuda.synchronize()
    stats = b.env_stats(h)
    b.env_destroy(h)
    p = orc.Pong(n, seed); p.reset()
    _, orew, odone = p.rollout(T, nthreads=16, want_obs=False)
    assert_bit_equal(rew.cpu().numpy(), orew, "C2-262144 reward")
    assert_bit_equal(done.cpu().numpy(), odone, "C2-262144 done")
    q = orc.Pong(4096, seed); q.reset()
    qobs, _, _ = q.rollout(T, nthreads=16)
    assert_bit_equal(obs[:, :4096].cpu().numpy(), qobs, "C2-262144 obs head")
    st = p.stats()
    assert stats["episodes"] == st["episodes"] and stats["return_sum"] == st["return_sum"]
    # last 4096 environments: final observation equals the oracle's final state
    assert_bit_equal(obs[T - 1, -4096:].cpu().numpy(), p.obs()[-4096:], "C2-262144 final obs tail")


@pytest.mark.parametrize("n,external,pace", [(64, False, 0), (1000, True, 0), (4100, False, 0), (4100, False, 6600),
                                             (1000, True, 6600)])
def test_normalised_observations_match_oracle(n, external, pace):
    """obs_scaling = ENV_OBS_NORMALIZED: the scaling is done in the step kernel; bit-identical to the
    oracle's normalised observation, dynamics untouched.  pace > 0 forces the paced loop, which
    large batches take, on these small ones."""
    T, seed, ms = 400, 17, 3
    assert b.lib().mi355env_tune_rollout_pace(pace) == 0
    acts = inputs.pong_actions(T, n, seed=4) if external else None
    h = b.env_create(b.ENV_PONG, n, seed, {"max_score": ms, "obs_scaling": b.ENV_OBS_NORMALIZED})
    try:
        obs0 = torch.empty((n, 8), dtype=torch.float32, device=DEV)
        b.env_reset(h, obs0)
        obs, rew, done = bufs(T, n)
        act = None if acts is None else torch.from_numpy(acts).to(DEV)
        b.env_rollout(h, T - 1, None if act is None else act[:T - 1], obs[:T - 1], rew[:T - 1], done[:T - 1])
        b.env_step(h, None if act is None else act[T - 1], obs[T - 1], rew[T - 1], done[T - 1])
        torch.cuda.synchronize()
        state = b.env_get_state(h)
        stats = b.env_stats(h)
    finally:
        b.env_destroy(h)
        assert b.lib().mi355env_tune_rollout_pace(0) == 0
    p = orc.Pong(n, seed, max_score=ms, normalize=True)
    o0 = p.reset()
    oo, orr, od = p.rollout(T, actions=acts, nthreads=4)
    assert_bit_equal(obs0.cpu().numpy(), o0, "normalised reset obs")
    assert_bit_equal(obs.cpu().numpy(), oo, "normalised obs")
    assert_bit_equal(rew.cpu().numpy(), orr, "reward")
    assert_bit_equal(done.cpu().numpy(), od, "done")
    _, fields = split_state(state, n, 10)
    assert_bit_equal(fields, pong_state_fields(p.envs()), "state (raw units)")
    assert oo[..., 6:8].max() > 0.3                    # some score was shown, scaled
    want = p.stats()
    assert all(stats[k] == want[k] for k in ("episodes", "length_sum", "return_sum")), (stats, want)


def test_normalised_observations_only_for_pong_vectors():
    for kind in (b.ENV_PONG_PIXELS, b.ENV_BODY, b.ENV_CARTPOLE):
        with pytest.raises(b.EnvError) as ei:
            b.env_create(kind, 64, 0, {"obs_scaling": b.ENV_OBS_NORMALIZED})
        assert ei.value.code == b.ENV_E_UNSUPPORTED


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("n,T", [(868, 7), (868, 250), (256, 4), (2048, 33)])
def test_both_store_paths_and_every_chunk_remainder(mode, n, T):
    """The rollout draws its Philox blocks four steps at a time and has two ways of storing
    observations (direct; through LDS, one 4 KiB page per store instruction, for full 256-thread
    workgroups).  Both paths, forced on at sizes that mix full and ragged workgroups and at step
    counts with every remainder modulo 4, must reproduce the oracle bit for bit."""
    assert b.lib().mi355env_tune_paged_stores(mode) == 0
    try:
        g = gpu_rollout(n, 23, T, max_score=2)
    finally:
        assert b.lib().mi355env_tune_paged_stores(2) == 0
    compare(g, oracle_rollout(n, 23, T, max_score=2), n, "stores mode %d n=%d T=%d" % (mode, n, T))


@pytest.mark.parametrize("loop", ["chunk2", "chunk4", "chunk8", "paced", "paced_slow", "split", "unsplit"])
@pytest.mark.parametrize("T,max_score", [(1, 1), (19, 1), (250, 1), (1000, 2)])
def test_every_variant_of_the_main_loop(loop, T, max_score):
    """The full-wavefront loop exists with 2, 4 and 8 steps per chunk, and in a paced form whose
    chunks keep to a clock and whose episode statistics are marked in the step and brought up to
    date once per chunk; the launcher picks by N.  Each one, forced on, must give the oracle's
    trajectories, statistics and final state; max_score = 1 ends an episode at every point.
    "paced_slow" asks for a rate so low that every chunk really waits for its slot.  "split" gives
    every 64 environments a second wavefront that draws their Philox blocks (the default for
    small batches and T >= 32; forced here for every T), "unsplit" is the default without it."""
    n, seed = 64 * 9 + 40, 41
    L = b.lib()
    chunk, pace, split = {"chunk2": (2, -1, 0), "chunk4": (4, -1, 0), "chunk8": (8, -1, 0), "paced": (0, 6600, 0),
                          "paced_slow": (0, 1, 0), "split": (0, 0, 2), "unsplit": (0, 0, 1)}[loop]
    assert L.mi355env_tune_rollout_chunk(chunk) == 0 and L.mi355env_tune_rollout_pace(pace) == 0
    assert L.mi355env_tune_rollout_split(split) == 0
    try:
        g = gpu_rollout(n, seed, T, max_score=max_score)
    finally:
        assert L.mi355env_tune_rollout_chunk(0) == 0 and L.mi355env_tune_rollout_pace(0) == 0
        assert L.mi355env_tune_rollout_split(0) == 0
    compare(g, oracle_rollout(n, seed, T, max_score=max_score), n, "%s T=%d" % (loop, T))


@pytest.mark.parametrize("device_counter", [False, True])
def test_step_counter_crosses_2_to_the_32(device_counter):
    """The step index is 64 bits wide and both halves key Philox: a rollout that starts five steps
    before 2^32 must keep matching the oracle across the carry (and far beyond it)."""
    n, T = 300, 12
    for start in ((1 << 32) - 5, (1 << 40) + 123):
        p = orc.Pong(n, 41, max_score=2)
        p.reset()
        p.rollout(25)                                   # any state will do
        p.step_count = start
        fields = pong_state_fields(p.envs().copy())
        cfg = {"max_score": 2}
        if device_counter:
            cfg["step_counter"] = b.ENV_STEP_COUNTER_DEVICE
        h = b.env_create(b.ENV_PONG, n, 41, cfg)
        try:
            b.env_set_state(h, pong_blob(start, fields))
            assert b.env_step_count(h) == start
            obs, rew, done = bufs(T, n)
            b.env_rollout(h, 5, None, obs[:5], rew[:5], done[:5])
            for t in range(5, T):
                b.env_step(h, None, obs[t], rew[t], done[t])
            torch.cuda.synchronize()
            assert b.env_step_count(h) == start + T
            blob = b.env_get_state(h)
        finally:
            b.env_destroy(h)
        oo, orr, od = p.rollout(T)
        assert_bit_equal(obs.cpu().numpy(), oo, "obs from step %d" % start)
        assert_bit_equal(done.cpu().numpy(), od, "done from step %d" % start)
        step, got = split_state(blob, n, 10)
        assert step == start + T
        assert_bit_equal(got, pong_state_fields(p.envs()), "state")


@pytest.mark.parametrize("step_kernel", [1, 0], ids=["step kernel", "rollout kernel with T = 1"])
@pytest.mark.parametrize("external", [False, True])
@pytest.mark.parametrize("n", [1, 255, 257, 700])
def test_both_ways_to_take_a_single_step(n, external, step_kernel):
    # env_step normally takes a kernel that holds one step and nothing else; the rollout kernel's
    # T = 1 path computes the same thing.  Each is forced here, one launch per step, ragged sizes.
    T, seed = 60, 300 + n
    acts = inputs.pong_actions(T, n, seed=5) if external else None
    assert b.lib().mi355env_tune_step_kernel(step_kernel) == 0
    try:
        g = gpu_rollout(n, seed, T, max_score=1, actions=acts, per_step=True)
    finally:
        assert b.lib().mi355env_tune_step_kernel(1) == 0
    compare(g, oracle_rollout(n, seed, T, max_score=1, actions=acts), n, "single steps")
    assert g["stats"]["episodes"] > 0 or n < 10


def test_a_prepared_step_repeated_is_the_rollout():
    # binding.PreparedStep marshals env_step's arguments once; every call after that is the C entry
    # point alone.  T calls into the same buffers leave the oracle's state after T steps, its
    # statistics, and the outputs of the last step.
    n, seed, T = 1000, 77, 90
    h = b.env_create(b.ENV_PONG, n, seed, {"max_score": 1})
    try:
        b.env_reset(h, None)
        obs, rew, done = (x[0] for x in bufs(1, n))
        step = b.PreparedStep(h, None, obs, rew, done)
        for _ in range(T):
            step()
        torch.cuda.synchronize()
        o = oracle_rollout(n, seed, T, max_score=1)
        assert_bit_equal(obs.cpu().numpy(), o["obs"][T - 1], "prepared step obs")
        assert_bit_equal(rew.cpu().numpy(), o["rew"][T - 1], "prepared step reward")
        assert_bit_equal(done.cpu().numpy(), o["done"][T - 1], "prepared step done")
        count, fields = split_state(b.env_get_state(h), n, 10)
        assert count == T == b.env_step_count(h)
        assert_bit_equal(fields, o["state"], "prepared step state")
        assert b.env_stats(h)["episodes"] == o["stats"]["episodes"] > 0
    finally:
        b.env_destroy(h)


def _resident_launches():
    f = b.lib().mi355env_resident_step_launches
    f.restype = C.c_ulonglong
    return int(f())


class _Mirror:
    """One handle and its oracle twin, stepped through the same calls; every step's outputs compared."""

    def __init__(self, n, seed, external, scaled):
        cfg = {"max_score": 1}
        if scaled:
            cfg["obs_scaling"] = b.ENV_OBS_NORMALIZED
        self.n, self.external = n, external
        self.h = b.env_create(b.ENV_PONG, n, seed, cfg)
        self.o = orc.Pong(n, seed, max_score=1, normalize=scaled)
        self.bufs = [tuple(x[0] for x in bufs(1, n)) for _ in range(2)]
        self.act = torch.empty(n, dtype=torch.uint8, device=DEV) if external else None
        self.seen = []      # (obs, reward, done) of every step, device copies taken on the stream
        self.want = []
        self.k = 0

    def reset(self):
        b.env_reset(self.h, None)
        self.o.reset()

    def steps(self, count, which=0):
        obs, rew, done = self.bufs[which]
        for _ in range(count):
            a = None
            if self.external:
                a = inputs.pong_actions(1, self.n, seed=1000 + self.k)[0]
                self.act.copy_(torch.from_numpy(a))
            self.k += 1
            b.env_step(self.h, self.act, obs, rew, done)
            self.seen.append((obs.clone(), rew.clone(), done.clone()))
            self.want.append(tuple(x[0] for x in self.o.rollout(1, actions=None if a is None else a[None])))

    def rollout(self, T):
        assert not self.external
        obs, rew, done = bufs(T, self.n)
        b.env_rollout(self.h, T, None, obs, rew, done)
        oo, orr, od = self.o.rollout(T)
        self.seen.append((obs[-1].clone(), rew[-1].clone(), done[-1].clone()))
        self.want.append((oo[-1], orr[-1], od[-1]))

    def check(self, what):
        torch.cuda.synchronize()
        assert len(self.seen) == len(self.want)
        for t, (g, w) in enumerate(zip(self.seen, self.want)):
            for gx, wx, name in zip(g, w, ("obs", "reward", "done")):
                assert_bit_equal(gx.cpu().numpy(), wx, "%s: %s of call %d" % (what, name, t))
        count, fields = split_state(b.env_get_state(self.h), self.n, 10)
        assert count == self.o.step_count == b.env_step_count(self.h)
        assert_bit_equal(fields, pong_state_fields(self.o.envs()), what + ": state")
        gs, ws = b.env_stats(self.h), self.o.stats()
        assert gs["episodes"] == ws["episodes"] and gs["return_sum"] == ws["return_sum"]
        assert gs["length_sum"] == ws["length_sum"]

    def close(self):
        b.env_destroy(self.h)


@pytest.mark.parametrize("external,scaled", [(False, False), (True, False), (False, True), (True, True)])
@pytest.mark.parametrize("n", [1, 700, 4096, 16384])
def test_steps_launched_from_the_resident_record(n, external, scaled):
    # From the second call in a row with the same buffers, env_step launches a kernel that takes no
    # argument and reads its descriptor, and the step index, from device memory.  Whatever else moves
    # the step index or the state in between (reset, a rollout, set_state, a call with other buffers)
    # has to show in the next step.
    m = _Mirror(n, 40 + n, external, scaled)
    resident_before = _resident_launches()
    try:
        m.reset()
        m.steps(12)
        if not external:
            m.rollout(7)
        m.steps(6)
        m.reset()
        m.steps(5)
        b.env_set_state(m.h, b.env_get_state(m.h))
        m.steps(5)
        m.steps(2, which=1)
        m.steps(40)
        m.check("resident steps, n = %d" % n)
        assert b.env_stats(m.h)["episodes"] > 0 or n == 1
        # of the 70 steps, the first of every run with new buffers goes with arguments: 12 + 6 + 5 + 5
        # (+ 2 in the second set of buffers) + 40, less one per run
        assert _resident_launches() - resident_before == 11 + 6 + 5 + 5 + 1 + 39
    finally:
        m.close()


def test_more_stepping_handles_than_resident_records():
    # Four handles per device own a launch record; a fifth and sixth step with arguments.  All of
    # them interleaved, then two destroyed and two new ones created (which take over their records).
    ms = [_Mirror(300 + 7 * k, 900 + k, False, False) for k in range(6)]
    resident_before = _resident_launches()
    try:
        for m in ms:
            m.reset()
        for _ in range(10):
            for m in ms:
                m.steps(3)
        for m in ms:
            m.check("handle of %d" % m.n)
        # four handles went resident from their second step on, the other two never
        assert _resident_launches() - resident_before == 4 * 29
        for m in ms[:2]:
            m.close()
        ms = ms[2:] + [_Mirror(5000 + k, 950 + k, False, False) for k in range(2)]
        for m in ms[-2:]:
            m.reset()
        for _ in range(6):
            for m in ms:
                m.steps(4)
        for m in ms:
            m.check("handle of %d, second round" % m.n)
    finally:
        for m in ms:
            m.close()


def test_resident_steps_follow_the_handle_to_another_stream():
    n = 2000
    m = _Mirror(n, 5, False, False)
    side = torch.cuda.Stream()
    try:
        m.reset()
        m.steps(8)
        torch.cuda.synchronize()
        b.env_set_stream(m.h, side.cuda_stream)
        with torch.cuda.stream(side):
            m.steps(8)
        torch.cuda.synchronize()
        b.env_set_stream(m.h, torch.cuda.current_stream().cuda_stream)
        m.steps(8)
        m.check("steps across streams")
    finally:
        m.close()


def test_sixteen_million_environments():
    # a batch far beyond the configurations (2^24 + 5 environments, 671 MB of state): environment
    # indices above 2^24 in the Philox counter, offsets above 2^31 bytes into the trajectory buffers,
    # the paged-store loop that large batches take, and a ragged last wavefront
    n, seed, T = (1 << 24) + 5, 99, 3
    g = gpu_rollout(n, seed, T)
    o = oracle_rollout(n, seed, T, nthreads=16)
    compare(g, o, n, "2^24 + 5 environments")
    # ... and the same batch one launch per step
    g = gpu_rollout(n, seed, T, per_step=True)
    compare(g, o, n, "2^24 + 5 environments, one launch per step")
