"""GPU parity on seeded random configurations: sizes around every tile boundary, 62-bit seeds, random
splits of a rollout into launches, and every option that changes a code path (external actions,
observation scaling, device step counter, store path, ring layout, renderer) drawn from a fixed
generator.  Everything is compared bit for bit with the oracle.  Each case is printed before it
runs."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import oracle as orc                      # noqa: E402
from oracle.cartpole_binding import CartPole          # noqa: E402
from paper_2603_12145_amd import binding as b         # noqa: E402
from paper_2603_12145_amd import inputs               # noqa: E402
from gpu_helpers import assert_bit_equal, split_state, pong_state_fields   # noqa: E402

DEV = "cuda:0"


def _trajectory_buffers(T, n, obs_dim):
    return (torch.empty((T, n, obs_dim), dtype=torch.float32, device=DEV),
            torch.empty((T, n), dtype=torch.float32, device=DEV),
            torch.empty((T, n), dtype=torch.uint8, device=DEV))


def pong_case(rng, k):
    n = int(rng.choice([1, 2, 63, 64, 65, 255, 256, 257, 1000, 4097, 16384, 20000, 70001, 131100]))
    T = int(rng.integers(1, 400))
    seed = int(rng.integers(0, 2 ** 62))
    max_score = int(rng.choice([1, 2, 5, 21]))
    external, scaled, device_counter = (bool(rng.integers(0, 2)) for _ in range(3))
    paged = int(rng.integers(0, 3))
    print("pong case", k, dict(n=n, T=T, seed=seed, max_score=max_score, external=external, scaled=scaled,
                               device_counter=device_counter, paged=paged), flush=True)
    acts = inputs.pong_actions(T, n, seed=k) if external else None
    cfg = {"max_score": max_score}
    if scaled:
        cfg["obs_scaling"] = b.ENV_OBS_NORMALIZED
    if device_counter:
        cfg["step_counter"] = b.ENV_STEP_COUNTER_DEVICE
    assert b.lib().mi355env_tune_paged_stores(paged) == 0
    h = b.env_create(b.ENV_PONG, n, seed, cfg)
    try:
        obs0 = torch.empty((n, 8), dtype=torch.float32, device=DEV)
        b.env_reset(h, obs0)
        obs, rew, done = _trajectory_buffers(T, n, 8)
        act = None if acts is None else torch.from_numpy(acts).to(DEV)
        t = 0
        while t < T:                                   # the rollout cut into launches at random
            c = int(min(T - t, rng.integers(1, max(2, T // 2 + 1))))
            b.env_rollout(h, c, None if act is None else act[t:t + c], obs[t:t + c], rew[t:t + c], done[t:t + c])
            t += c
        torch.cuda.synchronize()
        stats, blob = b.env_stats(h), b.env_get_state(h)
    finally:
        b.env_destroy(h)
    p = orc.Pong(n, seed, max_score=max_score, normalize=scaled)
    o0 = p.reset()
    oo, orr, od = p.rollout(T, actions=acts, nthreads=8)
    assert_bit_equal(obs0.cpu().numpy(), o0, "reset obs")
    assert_bit_equal(obs.cpu().numpy(), oo, "obs")
    assert_bit_equal(rew.cpu().numpy(), orr, "reward")
    assert_bit_equal(done.cpu().numpy(), od, "done")
    want = p.stats()
    assert stats["episodes"] == want["episodes"] and stats["return_sum"] == want["return_sum"]
    assert stats["length_sum"] == want["length_sum"]
    _, fields = split_state(blob, n, 10)
    assert_bit_equal(fields, pong_state_fields(p.envs()), "state")


def cartpole_case(rng, k):
    n = int(rng.choice([1, 63, 65, 300, 5000, 66000]))
    T = int(rng.integers(1, 300))
    seed = int(rng.integers(0, 2 ** 62))
    max_steps = int(rng.choice([5, 50, 500]))
    external = bool(rng.integers(0, 2))
    print("cartpole case", k, dict(n=n, T=T, seed=seed, max_steps=max_steps, external=external), flush=True)
    acts = inputs.cartpole_actions(T, n, seed=k) if external else None
    h = b.env_create(b.ENV_CARTPOLE, n, seed, {"max_episode_steps": max_steps})
    try:
        b.env_reset(h, None)
        obs, rew, done = _trajectory_buffers(T, n, 4)
        b.env_rollout(h, T, None if acts is None else torch.from_numpy(acts).to(DEV), obs, rew, done)
        torch.cuda.synchronize()
        stats = b.env_stats(h)
    finally:
        b.env_destroy(h)
    p = CartPole(n, seed, max_steps=max_steps)
    p.reset()
    oo, _, od = p.rollout(T, actions=acts, nthreads=8)
    assert_bit_equal(obs.cpu().numpy(), oo, "obs")
    assert_bit_equal(done.cpu().numpy(), od, "done")
    assert stats["episodes"] == p.stats()["episodes"]


def pixel_case(rng, k):
    n = int(rng.choice([1, 17, 100, 257, 3000]))
    T = int(rng.integers(4, 40))
    seed = int(rng.integers(0, 2 ** 62))
    layout = int(rng.choice([b.ENV_PIXELS_SLOT_MAJOR, b.ENV_PIXELS_ENV_MAJOR]))
    renderer = int(rng.integers(0, 3))
    print("pixel case", k, dict(n=n, T=T, seed=seed, layout=layout, renderer=renderer), flush=True)
    assert b.lib().mi355env_tune_plane_path(renderer) == 0
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1, "pixel_layout": layout})
    try:
        shape = (4, n, 84, 84) if layout == b.ENV_PIXELS_SLOT_MAJOR else (n, 4, 84, 84)
        ring = torch.zeros(shape, dtype=torch.uint8, device=DEV)
        b.env_reset(h, ring)
        rew = torch.empty(n, dtype=torch.float32, device=DEV)
        done = torch.empty(n, dtype=torch.uint8, device=DEV)
        p = orc.Pong(n, seed, max_score=1)
        p.reset()
        stack = np.zeros((n, 4, 84, 84), np.uint8)
        for t in range(T):
            b.env_step(h, None, ring, rew, done)
            _, orew, odone = p.step(stack=stack)
            assert_bit_equal(rew.cpu().numpy(), orew, "reward %d" % t)
            assert_bit_equal(done.cpu().numpy(), odone, "done %d" % t)
        torch.cuda.synchronize()
        got = ring.cpu().numpy()
    finally:
        b.env_destroy(h)
    if layout == b.ENV_PIXELS_SLOT_MAJOR:
        got = np.ascontiguousarray(got.transpose(1, 0, 2, 3))
    assert_bit_equal(got, stack, "ring after %d steps" % T)      # T >= 4: every slot rewritten


def body_case(rng, k):
    """Random size, length, contact model, arithmetic, action source and episode length.  A rollout
    cut into launches at random must equal the same steps taken one launch each, bit for bit; the
    first step must agree with the float64 oracle (1e-5 in float64, as close as float32 gets
    otherwise); truncation times and episode counts are exact."""
    from oracle.body_binding import Body
    sizes = [1, 2, 31, 32, 33, 63, 64, 65, 500, 2049, 9000, 33000]      # every one is taken in turn
    n = sizes[k % len(sizes)]
    T = int(rng.integers(1, 40))
    seed = int(rng.integers(0, 2 ** 62))
    solver, f32, external, device_counter = (int(rng.integers(0, 2)) for _ in range(4))
    limit = int(rng.integers(3, 30))
    print("body case", k, dict(n=n, T=T, seed=seed, solver=solver, f32=f32, external=external,
                               device_counter=device_counter, max_episode_steps=limit), flush=True)
    cfg = {"max_episode_steps": limit}
    if solver:
        cfg["contact_solver"] = b.ENV_CONTACT_NEWTON
    if f32:
        cfg["body_arithmetic"] = b.ENV_BODY_F32
    if device_counter:
        cfg["step_counter"] = b.ENV_STEP_COUNTER_DEVICE
    acts = inputs.body_actions(T, n, seed=k, scale=1.3) if external else None
    act = None if acts is None else torch.from_numpy(acts).to(DEV)
    outs = []
    for per_step in (False, True):
        h = b.env_create(b.ENV_BODY, n, seed, cfg)
        try:
            obs0 = torch.empty((n, 17), dtype=torch.float32, device=DEV)
            b.env_reset(h, obs0)
            obs, rew, done = _trajectory_buffers(T, n, 17)
            t = 0
            while t < T:
                c = 1 if per_step else int(min(T - t, rng.integers(1, max(2, T // 2 + 1))))
                b.env_rollout(h, c, None if act is None else act[t:t + c], obs[t:t + c], rew[t:t + c], done[t:t + c])
                t += c
            torch.cuda.synchronize()
            outs.append((obs0.cpu().numpy(), obs.cpu().numpy(), rew.cpu().numpy(), done.cpu().numpy(),
                         b.env_stats(h), b.env_get_state(h)))
        finally:
            b.env_destroy(h)
    for j, name in enumerate(("reset obs", "obs", "reward", "done")):
        assert_bit_equal(outs[0][j], outs[1][j], "body case %d %s: fused vs one launch per step" % (k, name))
    # the statistics add float32 returns up per lane and launch before the float64 atomics: the sum
    # depends on how the rollout was cut (in the ninth digit), everything else does not
    for key in ("episodes", "length_sum", "nonfinite", "return_min", "return_max"):
        assert outs[0][4][key] == outs[1][4][key], key
    assert abs(outs[0][4]["return_sum"] - outs[1][4]["return_sum"]) <= 1e-6 * max(1.0, abs(outs[1][4]["return_sum"]))
    assert np.array_equal(outs[0][5], outs[1][5])
    o = Body(n, seed, np.float64, max_episode_steps=limit, solver=solver)
    o0 = o.reset()
    oo, orr, od = o.rollout(T, actions=None if acts is None else acts.astype(np.float64), nthreads=8)
    g0, go, gr, gd, st, _ = outs[0]
    assert np.abs(g0 - o0).max() < 5e-7                           # Box-Muller through float32 log / cos / sin
    assert np.array_equal(gd, od), "truncation times"
    assert st["episodes"] == int(od.sum()) == n * (T // limit) and st["nonfinite"] == 0
    # first step: same physics from (nearly) the same initial state
    err = np.abs(go[0].astype(np.float64) - oo[0]) / np.maximum(np.abs(oo[0]), 1.0)
    live = od[0] == 0
    tol = 2e-3 if f32 else 2e-5          # v0 itself differs by up to 5e-7; float32: see test_gpu_body_f32.py
    assert err[live].max() < tol if live.any() else True, err.max()
    assert np.isfinite(go).all() and np.isfinite(gr).all()


def test_random_body_cases():
    rng = np.random.default_rng(45678)
    for k in range(14):
        body_case(rng, k)


def test_random_pong_cases():
    rng = np.random.default_rng(12345)
    try:
        for k in range(18):
            pong_case(rng, k)
    finally:
        assert b.lib().mi355env_tune_paged_stores(2) == 0


def test_random_cartpole_cases():
    rng = np.random.default_rng(23456)
    for k in range(6):
        cartpole_case(rng, k)


def test_random_pixel_cases():
    rng = np.random.default_rng(34567)
    try:
        for k in range(8):
            pixel_case(rng, k)
    finally:
        assert b.lib().mi355env_tune_plane_path(2) == 0


PIXEL_MODES = {
    "ring slot-major": dict(pixel_layout=b.ENV_PIXELS_SLOT_MAJOR),
    "ring env-major": dict(pixel_layout=b.ENV_PIXELS_ENV_MAJOR),
    "ring slot-major, device counter": dict(pixel_layout=b.ENV_PIXELS_SLOT_MAJOR,
                                            step_counter=b.ENV_STEP_COUNTER_DEVICE),
    "ring env-major, device counter": dict(pixel_layout=b.ENV_PIXELS_ENV_MAJOR,
                                           step_counter=b.ENV_STEP_COUNTER_DEVICE),
    "ring slot-major, delta": dict(pixel_layout=b.ENV_PIXELS_SLOT_MAJOR, pixel_update=b.ENV_PIXELS_DELTA),
    "ring env-major, delta": dict(pixel_layout=b.ENV_PIXELS_ENV_MAJOR, pixel_update=b.ENV_PIXELS_DELTA),
    "ordered stack": dict(pixel_layout=b.ENV_PIXELS_ORDERED),
    "ring slot-major, delta, device counter": dict(pixel_layout=b.ENV_PIXELS_SLOT_MAJOR,
                                                   pixel_update=b.ENV_PIXELS_DELTA,
                                                   step_counter=b.ENV_STEP_COUNTER_DEVICE),
    "ordered stack, device counter": dict(pixel_layout=b.ENV_PIXELS_ORDERED,
                                          step_counter=b.ENV_STEP_COUNTER_DEVICE),
}


def pixel_call_sequence(rng, k, mode):
    """A random sequence of calls on one pixel handle -- steps with in-kernel or external actions,
    frame-trajectory rollouts, save / restore, resets, a change of observation buffer -- with the
    observation buffer, rewards, done flags and frames compared with the oracle after every call.
    The reference keeps the oracle's own ring (slot = step mod 4) and, for the ordered stack, moves
    its channels down on every step, as the boundary defines it."""
    n = int(rng.choice([1, 9, 64, 130, 300]))
    seed = int(rng.integers(0, 2 ** 62))
    calls = int(rng.integers(30, 70))
    cfg = dict(PIXEL_MODES[mode], max_score=1)
    ordered = cfg["pixel_layout"] == b.ENV_PIXELS_ORDERED
    slot_major = cfg["pixel_layout"] == b.ENV_PIXELS_SLOT_MAJOR
    print("pixel sequence", k, mode, dict(n=n, seed=seed, calls=calls), flush=True)

    def as_env_major(buf):
        a = buf.cpu().numpy()
        return np.ascontiguousarray(a.transpose(1, 0, 2, 3)) if slot_major else a

    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, cfg)
    try:
        buf = torch.full((4, n, 84, 84) if slot_major else (n, 4, 84, 84), 33, dtype=torch.uint8, device=DEV)
        rew = torch.empty(n, dtype=torch.float32, device=DEV)
        done = torch.empty(n, dtype=torch.uint8, device=DEV)
        p = orc.Pong(n, seed, max_score=1)
        ring = np.zeros((n, 4, 84, 84), np.uint8)          # the oracle's ring
        b.env_reset(h, buf)
        p.reset(); p.fill_stack(ring)
        want = ring.copy()                                  # what buf must hold (env-major view)
        assert_bit_equal(as_env_major(buf), want, "after the first reset")
        for c in range(calls):
            op = rng.choice(["step", "step", "step", "step", "step_ext", "step_ext", "rollout", "restore",
                             "reset", "new_buffer"], p=[.2, .2, .15, .15, .08, .07, .05, .04, .03, .03])
            s = p.step_count
            if op in ("step", "step_ext"):
                a = inputs.pong_actions(1, n, seed=1000 * k + c) if op == "step_ext" else None
                b.env_step(h, None if a is None else torch.from_numpy(a[0]).to(DEV), buf, rew, done)
                _, orew, odone = p.step(actions=None if a is None else a[0], stack=ring)
                if ordered:
                    want[:, :3] = want[:, 1:].copy()
                    want[:, 3] = ring[:, s & 3]
                else:
                    want[:, s & 3] = ring[:, s & 3]
                assert_bit_equal(rew.cpu().numpy(), orew, "call %d reward" % c)
                assert_bit_equal(done.cpu().numpy(), odone, "call %d done" % c)
            elif op == "rollout":
                T = int(rng.integers(1, 6))
                fr = torch.empty((T, n, 84, 84), dtype=torch.uint8, device=DEV)
                rT = torch.empty((T, n), dtype=torch.float32, device=DEV)
                dT = torch.empty((T, n), dtype=torch.uint8, device=DEV)
                b.env_rollout(h, T, None, fr, rT, dT)
                scratch = np.zeros((n, 4, 84, 84), np.uint8)
                for t in range(T):                          # frames of the oracle, one step at a time
                    _, orew, odone = p.step(stack=scratch)
                    assert_bit_equal(fr[t].cpu().numpy(), scratch[:, (s + t) & 3], "call %d frame %d" % (c, t))
                    assert_bit_equal(rT[t].cpu().numpy(), orew, "call %d reward %d" % (c, t))
                    assert_bit_equal(dT[t].cpu().numpy(), odone, "call %d done %d" % (c, t))
            elif op == "restore":
                b.env_set_state(h, b.env_get_state(h))
            elif op == "reset":
                buf.fill_(int(rng.integers(0, 256)))
                b.env_reset(h, buf)
                p.reset(); p.fill_stack(ring)
                want = ring.copy()
            elif op == "new_buffer":
                buf = buf.clone()
            assert_bit_equal(as_env_major(buf), want, "call %d (%s): observation buffer" % (c, op))
        assert b.env_step_count(h) == p.step_count
        assert b.env_stats(h)["episodes"] == p.stats()["episodes"]
    finally:
        b.env_destroy(h)


@pytest.mark.parametrize("mode", sorted(PIXEL_MODES))
def test_random_pixel_call_sequences(mode):
    rng = np.random.default_rng(45678 + sorted(PIXEL_MODES).index(mode))
    for k in range(3):
        pixel_call_sequence(rng, k, mode)
