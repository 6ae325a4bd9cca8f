"""GPU parity: CartPole, HIP path vs CPU oracle, bit for bit (float32 with fixed polynomials for
sin / cos on both sides).  Every call goes through the C-ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle.cartpole_binding import CartPole          # noqa: E402
from paper_2603_12145_amd import binding as b         # noqa: E402
from paper_2603_12145_amd import inputs               # noqa: E402
from gpu_helpers import assert_bit_equal, split_state  # noqa: E402

DEV = "cuda:0"


def gpu_rollout(n, seed, T, max_steps=500, actions=None, per_step=False, chunks=None):
    h = b.env_create(b.ENV_CARTPOLE, n, seed, {"max_episode_steps": max_steps})
    try:
        obs0 = torch.empty((n, 4), dtype=torch.float32, device=DEV)
        b.env_reset(h, obs0)
        obs = torch.empty((T, n, 4), dtype=torch.float32, device=DEV)
        rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
        done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
        act = None if actions is None else torch.from_numpy(actions).to(DEV)
        if per_step:
            for t in range(T):
                b.env_step(h, None if act is None else act[t], obs[t], rew[t], done[t])
        else:
            t0 = 0
            for c in (chunks or [T]):
                b.env_rollout(h, c, None if act is None else act[t0:t0 + c], obs[t0:t0 + c],
                              rew[t0:t0 + c], done[t0:t0 + c])
                t0 += c
            assert t0 == T
        torch.cuda.synchronize()
        return dict(obs0=obs0.cpu().numpy(), obs=obs.cpu().numpy(), rew=rew.cpu().numpy(),
                    done=done.cpu().numpy(), stats=b.env_stats(h), state=b.env_get_state(h),
                    steps=b.env_step_count(h))
    finally:
        b.env_destroy(h)


def oracle_rollout(n, seed, T, max_steps=500, actions=None, nthreads=8):
    p = CartPole(n, seed, max_steps=max_steps)
    obs0 = p.reset()
    obs, rew, done = p.rollout(T, actions=actions, nthreads=nthreads)
    return dict(obs0=obs0, obs=obs, rew=rew, done=done, stats=p.stats(), envs=p.envs().copy(),
                steps=p.step_count)


def compare(g, o, n, what):
    assert_bit_equal(g["obs0"], o["obs0"], what + " reset obs")
    assert_bit_equal(g["obs"], o["obs"], what + " obs")
    assert_bit_equal(g["rew"], o["rew"], what + " reward")
    assert_bit_equal(g["done"], o["done"], what + " done")
    step, f = split_state(g["state"], n, 6)
    assert step == o["steps"] == g["steps"]
    e = o["envs"]
    for k, name in enumerate(["x", "xd", "th", "thd"]):
        assert_bit_equal(f[k], np.ascontiguousarray(e[name]).view(np.uint32), what + " state " + name)
    assert_bit_equal(f[5], np.ascontiguousarray(e["ep_len"]).view(np.uint32), what + " state ep_len")
    assert_bit_equal(f[4].view(np.float32), e["ep_len"].astype(np.float32), what + " state ep_ret")
    gs, os_ = g["stats"], o["stats"]
    assert gs["episodes"] == os_["episodes"] and gs["length_sum"] == os_["length_sum"]
    assert gs["return_sum"] == float(os_["length_sum"])      # reward is 1 per step
    assert gs["nonfinite"] == 0
    if os_["episodes"]:
        assert gs["return_min"] == os_["length_min"] and gs["return_max"] == os_["length_max"]
    else:
        assert gs["return_min"] == float("inf") and gs["return_max"] == float("-inf")


@pytest.mark.parametrize("per_step", [False, True])
def test_n64_t1000_internal_actions(per_step):
    g = gpu_rollout(64, 0, 1000, per_step=per_step)
    o = oracle_rollout(64, 0, 1000)
    compare(g, o, 64, "cartpole n=64 per_step=%s" % per_step)
    assert o["stats"]["episodes"] > 1000          # random pushes fail after ~22 steps


@pytest.mark.parametrize("n", [1, 63, 65, 257, 2049, 5000])
def test_ragged_sizes(n):
    compare(gpu_rollout(n, 11, 200), oracle_rollout(n, 11, 200), n, "cartpole n=%d" % n)


def test_external_actions_and_chunked_rollout():
    n, T = 777, 300
    act = inputs.cartpole_actions(T, n, 5)
    g = gpu_rollout(n, 3, T, actions=act, chunks=[1, 99, 150, 50])
    o = oracle_rollout(n, 3, T, actions=act)
    compare(g, o, n, "cartpole external actions")


def test_balancing_policy_reaches_truncation():
    """A hand-written feedback law (computed on the host from the oracle's observations) keeps the
    pole up, so episodes end by truncation; the recorded actions are then replayed on the GPU."""
    n, T, max_steps = 300, 450, 200
    p = CartPole(n, 9, max_steps=max_steps)
    ob = p.reset()
    acts = np.empty((T, n), np.uint8)
    o_obs = np.empty((T, n, 4), np.float32)
    o_done = np.empty((T, n), np.uint8)
    for t in range(T):
        acts[t] = (ob[:, 2] + 0.5 * ob[:, 3] + 0.05 * ob[:, 0] + 0.1 * ob[:, 1] > 0).astype(np.uint8)
        o, _, d = p.rollout(1, actions=acts[t:t + 1])
        ob, o_obs[t], o_done[t] = o[0], o[0], d[0]
    st = p.stats()
    assert st["length_max"] == max_steps and st["episodes"] >= n
    g = gpu_rollout(n, 9, T, max_steps=max_steps, actions=acts)
    assert_bit_equal(g["obs"], o_obs, "policy obs")
    assert_bit_equal(g["done"], o_done, "policy done")
    assert g["stats"]["episodes"] == st["episodes"] and g["stats"]["length_sum"] == st["length_sum"]
    assert g["stats"]["return_max"] == max_steps


def test_state_roundtrip_continues_identically():
    n = 1000
    h = b.env_create(b.ENV_CARTPOLE, n, 21)
    h2 = b.env_create(b.ENV_CARTPOLE, n, 21)
    try:
        b.env_reset(h)
        mk = lambda T: (torch.empty((T, n, 4), dtype=torch.float32, device=DEV),
                        torch.empty((T, n), dtype=torch.float32, device=DEV),
                        torch.empty((T, n), dtype=torch.uint8, device=DEV))
        a = mk(40); b.env_rollout(h, 40, None, *a)
        blob = b.env_get_state(h)
        b.env_set_state(h2, blob)
        c1, c2 = mk(60), mk(60)
        b.env_rollout(h, 60, None, *c1)
        b.env_rollout(h2, 60, None, *c2)
        torch.cuda.synchronize()
        for x, y in zip(c1, c2):
            assert torch.equal(x, y)
        assert np.array_equal(b.env_get_state(h), b.env_get_state(h2))
    finally:
        b.env_destroy(h); b.env_destroy(h2)


def test_full_size_sampled_against_oracle():
    """N = 65536 x T = 500 in the launch configuration the benchmark times: statistics over the
    whole batch match the oracle exactly, observations are compared on the final step."""
    n, T = 65536, 500
    h = b.env_create(b.ENV_CARTPOLE, n, 2)
    try:
        b.env_reset(h)
        obs = torch.empty((T, n, 4), dtype=torch.float32, device=DEV)
        rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
        done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
        b.env_rollout(h, T, None, obs, rew, done)
        torch.cuda.synchronize()
        gs = b.env_stats(h)
        last = obs[-1].cpu().numpy()
        dsum = int(done.sum(dtype=torch.int64).item())
        col = obs[:, 12345].cpu().numpy()
    finally:
        b.env_destroy(h)
    p = CartPole(n, 2)
    p.reset()
    o_obs, _, o_done = p.rollout(T, nthreads=8)
    st = p.stats()
    assert gs["episodes"] == st["episodes"] == dsum == int(o_done.sum())
    assert gs["length_sum"] == st["length_sum"]
    assert gs["return_min"] == st["length_min"] and gs["return_max"] == st["length_max"]
    assert_bit_equal(last, o_obs[-1], "final obs")
    assert_bit_equal(col, o_obs[:, 12345], "env 12345 trajectory")


@pytest.mark.parametrize("mode", [1, 2], ids=["one wavefront per 64 environments", "producer and consumer wavefront"])
@pytest.mark.parametrize("n,T", [(1, 5), (63, 40), (64, 33), (130, 7), (1000, 100), (4096, 41)])
def test_both_rollout_loops_match_the_oracle(n, T, mode):
    # batches of up to 65536 environments normally take the loop with a second wavefront per 64
    # environments that draws the Philox blocks (from T = 32 on); here each loop is forced for
    # every size and length, ragged wavefronts and partial last rounds included
    assert b.lib().mi355env_tune_cartpole_split(mode) == 0
    try:
        seed = 700 + n
        g = gpu_rollout(n, seed, T, max_steps=9, chunks=[T // 2, T - T // 2] if T > 1 else None)
    finally:
        assert b.lib().mi355env_tune_cartpole_split(0) == 0
    compare(g, oracle_rollout(n, seed, T, max_steps=9), n, "cart-pole loop %d" % mode)
    assert g["stats"]["episodes"] >= n * (T // 9)


def _resident_launches():
    import ctypes
    f = b.lib().mi355env_resident_step_launches
    f.restype = ctypes.c_ulonglong
    return int(f())


@pytest.mark.parametrize("step_kernel", [0, 1, 2], ids=["rollout kernel with T = 1", "step kernel", "step kernel, always with arguments"])
@pytest.mark.parametrize("external", [False, True])
@pytest.mark.parametrize("n", [1, 65, 1000, 4096])
def test_single_steps_into_a_trajectory(n, external, step_kernel):
    # one launch per step, each step into its own row of the trajectory buffers (so the launch
    # always carries its arguments); the rollout kernel's T = 1 path computes the same thing
    T, seed = 70, 900 + n
    acts = inputs.cartpole_actions(T, n, seed=3) if external else None
    assert b.lib().mi355env_tune_step_kernel(step_kernel) == 0
    try:
        g = gpu_rollout(n, seed, T, max_steps=30, actions=acts, per_step=True)
    finally:
        assert b.lib().mi355env_tune_step_kernel(1) == 0
    compare(g, oracle_rollout(n, seed, T, max_steps=30, actions=acts), n, "single steps")
    assert g["stats"]["episodes"] > 0


@pytest.mark.parametrize("external", [False, True])
@pytest.mark.parametrize("n", [1, 700, 4096, 16384])
def test_steps_launched_from_the_resident_record(n, external):
    # The same buffers step after step: from the second call on the launch takes no arguments and
    # reads its descriptor and step index from device memory.  A rollout, a reset and a restored
    # state in between have to show in the next step.
    seed, max_steps = 77 + n, 25
    h = b.env_create(b.ENV_CARTPOLE, n, seed, {"max_episode_steps": max_steps})
    o = CartPole(n, seed, max_steps=max_steps)
    obs = torch.empty((n, 4), dtype=torch.float32, device=DEV)
    rew = torch.empty(n, dtype=torch.float32, device=DEV)
    done = torch.empty(n, dtype=torch.uint8, device=DEV)
    act = torch.empty(n, dtype=torch.uint8, device=DEV) if external else None
    seen, want, k = [], [], [0]

    def steps(count):
        for _ in range(count):
            a = None
            if external:
                a = inputs.cartpole_actions(1, n, seed=5000 + k[0])
                act.copy_(torch.from_numpy(a[0]))
            k[0] += 1
            b.env_step(h, act, obs, rew, done)
            seen.append((obs.clone(), done.clone()))
            oo, _, od = o.rollout(1, actions=a)
            want.append((oo[0], od[0]))

    before = _resident_launches()
    try:
        b.env_reset(h, None)
        o.reset()
        steps(15)
        if not external:
            big = [torch.empty((9, n, 4), dtype=torch.float32, device=DEV), torch.empty((9, n), dtype=torch.float32, device=DEV),
                   torch.empty((9, n), dtype=torch.uint8, device=DEV)]
            b.env_rollout(h, 9, None, *big)
            o.rollout(9)
        steps(10)
        b.env_reset(h, None)
        o.reset()
        steps(10)
        b.env_set_state(h, b.env_get_state(h))
        steps(20)
        torch.cuda.synchronize()
        for t, ((go, gd), (wo, wd)) in enumerate(zip(seen, want)):
            assert_bit_equal(go.cpu().numpy(), wo, "obs of step %d" % t)
            assert_bit_equal(gd.cpu().numpy(), wd, "done of step %d" % t)
        assert _resident_launches() - before == 14 + 10 + 10 + 20
        gs, ws = b.env_stats(h), o.stats()
        assert gs["episodes"] == ws["episodes"] > 0 and gs["length_sum"] == ws["length_sum"]
        count, f = split_state(b.env_get_state(h), n, 6)
        assert count == o.step_count
        assert_bit_equal(f[0], np.ascontiguousarray(o.envs()["x"]).view(np.uint32), "state x")
        assert_bit_equal(f[5], np.ascontiguousarray(o.envs()["ep_len"]).view(np.uint32), "state ep_len")
    finally:
        b.env_destroy(h)


def test_four_million_environments():
    # far beyond the sizes above: environment indices above 2^22 in the Philox counters, a ragged
    # last wavefront, fused and one launch per step
    n, seed, T = (1 << 22) + 1, 8, 4
    o = oracle_rollout(n, seed, T, max_steps=3, nthreads=16)
    compare(gpu_rollout(n, seed, T, max_steps=3), o, n, "2^22 + 1 environments")
    compare(gpu_rollout(n, seed, T, max_steps=3, per_step=True), o, n, "2^22 + 1 environments, one launch per step")
