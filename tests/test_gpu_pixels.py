"""GPU parity: Pong with pixel observations (84x84 uint8, 4-slot ring / frame trajectory) vs the
CPU oracle's rasteriser, byte for byte, through the C-ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import oracle as orc                      # noqa: E402
from paper_2603_12145_amd import binding as b         # noqa: E402
from paper_2603_12145_amd import inputs               # noqa: E402
from gpu_helpers import assert_bit_equal, split_state, pong_state_fields, pong_blob  # noqa: E402

DEV = "cuda:0"
F = 84


LAYOUTS = {"slot_major": b.ENV_PIXELS_SLOT_MAJOR, "env_major": b.ENV_PIXELS_ENV_MAJOR}


def new_ring(n, layout):
    shape = (4, n, F, F) if layout == "slot_major" else (n, 4, F, F)
    return torch.zeros(shape, dtype=torch.uint8, device=DEV)


def ring_as_env_major(ring, layout):
    """numpy [n,4,84,84] view of the ring's content, whatever its layout."""
    a = ring.cpu().numpy()
    return np.ascontiguousarray(a.transpose(1, 0, 2, 3)) if layout == "slot_major" else a


def _tune(epw, streaming=0):
    assert b.lib().mi355env_tune_pixels(epw, streaming) == 0


@pytest.fixture(autouse=True)
def _default_tuning():
    yield
    _tune(0, 0)
    assert b.lib().mi355env_tune_plane_path(2) == 0


@pytest.mark.parametrize("layout", ["slot_major", "env_major"])
@pytest.mark.parametrize("epw", [4, 8, 16, 32, 64])
@pytest.mark.parametrize("n", [37, 200])
def test_ring_steps_match_oracle(n, epw, layout):
    _tune(epw)
    seed, T = 40 + n, 14
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1, "pixel_layout": LAYOUTS[layout]})
    ring = new_ring(n, layout)
    rew = torch.empty(n, dtype=torch.float32, device=DEV)
    done = torch.empty(n, dtype=torch.uint8, device=DEV)
    b.env_reset(h, ring)
    p = orc.Pong(n, seed, max_score=1); p.reset()
    stack = np.zeros((n, 4, F, F), np.uint8)
    p.fill_stack(stack)
    torch.cuda.synchronize()
    assert_bit_equal(ring_as_env_major(ring, layout), stack, "ring after reset")
    for t in range(T):
        b.env_step(h, None, ring, rew, done)
        _, orew, odone = p.step(stack=stack)
        torch.cuda.synchronize()
        assert_bit_equal(ring_as_env_major(ring, layout), stack, "ring after step %d" % t)
        assert_bit_equal(rew.cpu().numpy(), orew, "reward step %d" % t)
        assert_bit_equal(done.cpu().numpy(), odone, "done step %d" % t)
    _, fields = split_state(b.env_get_state(h), n, 10)
    assert_bit_equal(fields, pong_state_fields(p.envs()), "state")
    b.env_destroy(h)


@pytest.mark.parametrize("n", [1, 7, 255, 256, 257, 1000])
def test_plane_renderer_and_wave_renderer_agree_with_oracle(n):
    # slot-major steps normally take the page renderer with the dynamics launch overlapped on a
    # second stream (2); the same two launches in series (1) and the per-wavefront tile renderer (0)
    # write the same ring.  Plane starts are 4 KiB-aligned only when
    # n is a multiple of 256: the other sizes exercise the partial first and last pages.
    seed, T = 90 + n, 9
    p = orc.Pong(n, seed, max_score=1); p.reset()
    stack = np.zeros((n, 4, F, F), np.uint8); p.fill_stack(stack)
    rings = []
    for plane_path in (2, 1, 0):
        assert b.lib().mi355env_tune_plane_path(plane_path) == 0
        h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1})
        ring = new_ring(n, "slot_major")
        ring.fill_(77)                       # stale content must be overwritten, not OR-ed into
        rew = torch.empty(n, dtype=torch.float32, device=DEV)
        done = torch.empty(n, dtype=torch.uint8, device=DEV)
        b.env_reset(h, ring)
        for t in range(T):
            b.env_step(h, None, ring, rew, done)
        torch.cuda.synchronize()
        rings.append(ring_as_env_major(ring, "slot_major"))
        stats = b.env_stats(h)
        b.env_destroy(h)
    for t in range(T):
        p.step(stack=stack)
    assert_bit_equal(rings[0], stack, "overlapped plane renderer")
    assert_bit_equal(rings[1], stack, "serial plane renderer")
    assert_bit_equal(rings[2], stack, "wave renderer")
    assert stats["episodes"] == p.stats()["episodes"]


def test_overlapped_and_serial_steps_interleave_correctly():
    # in-kernel actions take the two-stream pipeline, external actions the serial path; switching
    # between them, resetting and restoring state in between must not reorder anything
    n, seed, T = 700, 13, 60
    rng = np.random.default_rng(1)
    acts = inputs.pong_actions(T, n, seed=9)
    use_ext = rng.random(T) < 0.4
    L = b.lib()
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1})
    ring = new_ring(n, "slot_major")
    rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
    done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
    dacts = torch.from_numpy(acts).to(DEV)
    b.env_reset(h, ring)
    p = orc.Pong(n, seed, max_score=1); p.reset()
    stack = np.zeros((n, 4, F, F), np.uint8); p.fill_stack(stack)
    orew = np.zeros((T, n), np.float32); odone = np.zeros((T, n), np.uint8)
    for t in range(T):
        b.env_step(h, dacts[t] if use_ext[t] else None, ring, rew[t], done[t])
        _, orew[t], odone[t] = p.step(actions=acts[t] if use_ext[t] else None, stack=stack)
        if t == 20:                         # save / restore in the middle of the pipeline
            blob = b.env_get_state(h)
            b.env_set_state(h, blob)
        if t == 40:                         # second reset: all four slots rewritten
            b.env_reset(h, ring)
            p.reset(); p.fill_stack(stack)
    torch.cuda.synchronize()
    assert_bit_equal(ring_as_env_major(ring, "slot_major"), stack, "ring")
    assert_bit_equal(rew.cpu().numpy(), orew, "reward")
    assert_bit_equal(done.cpu().numpy(), odone, "done")
    assert b.env_stats(h)["episodes"] == p.stats()["episodes"] > 0
    b.env_destroy(h)


def test_streaming_store_variant_matches():
    _tune(16, 1)
    n, seed = 100, 3
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, None)          # default layout: slot-major
    ring = new_ring(n, "slot_major")
    rew = torch.empty(n, dtype=torch.float32, device=DEV)
    done = torch.empty(n, dtype=torch.uint8, device=DEV)
    b.env_reset(h, ring)
    p = orc.Pong(n, seed); p.reset()
    stack = np.zeros((n, 4, F, F), np.uint8); p.fill_stack(stack)
    for t in range(6):
        b.env_step(h, None, ring, rew, done)
        p.step(stack=stack)
    torch.cuda.synchronize()
    assert_bit_equal(ring_as_env_major(ring, "slot_major"), stack, "streaming ring")
    b.env_destroy(h)


@pytest.mark.parametrize("mode", [0, 1])       # single launch; staged and rendered in chunks
def test_frame_trajectory_rollout_with_external_actions(mode):
    n, seed, T = 150, 8, 40
    acts = inputs.pong_actions(T, n, seed=2)
    assert b.lib().mi355env_tune_frame_trajectory(mode) == 0
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1})
    try:
        b.env_reset(h, None)
        frames = torch.empty((T, n, F, F), dtype=torch.uint8, device=DEV)
        rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
        done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
        b.env_rollout(h, T, torch.from_numpy(acts).to(DEV), frames, rew, done)
        torch.cuda.synchronize()
        stats = b.env_stats(h)
    finally:
        b.env_destroy(h)
        assert b.lib().mi355env_tune_frame_trajectory(2) == 0
    p = orc.Pong(n, seed, max_score=1); p.reset()
    stack = np.zeros((n, 4, F, F), np.uint8)
    got = frames.cpu().numpy()
    for t in range(T):
        _, orew, odone = p.step(actions=acts[t], stack=stack)
        assert_bit_equal(got[t], stack[:, t % 4], "frame %d" % t)
        assert_bit_equal(rew[t].cpu().numpy(), orew, "reward %d" % t)
        assert_bit_equal(done[t].cpu().numpy(), odone, "done %d" % t)
    assert stats["episodes"] == p.stats()["episodes"] > 0


def test_rasteriser_on_arbitrary_positions():
    # states injected through env_set_state (ball velocity zero, far from events is not needed:
    # the frame shows the post-step state, which the oracle renders from its own post-step state)
    n = 2048
    pos = inputs.pong_positions(n, seed=11)
    envs = np.zeros(n, orc.PONG_ENV_DTYPE)
    envs["bx"], envs["by"], envs["pa"], envs["po"] = pos[:, 0], pos[:, 1], pos[:, 2], pos[:, 3]
    envs["vx"] = np.where(np.arange(n) % 2 == 0, 3.0, -3.0)
    envs["vy"] = np.linspace(-2, 2, n).astype(np.float32)
    p = orc.Pong(n, 5)
    p.envs()[:] = envs
    h = b.env_create(b.ENV_PONG_PIXELS, n, 5, {"pixel_layout": b.ENV_PIXELS_ENV_MAJOR})
    b.env_set_state(h, pong_blob(0, pong_state_fields(envs)))
    ring = torch.zeros((n, 4, F, F), dtype=torch.uint8, device=DEV)
    rew = torch.empty(n, dtype=torch.float32, device=DEV)
    done = torch.empty(n, dtype=torch.uint8, device=DEV)
    stack = np.zeros((n, 4, F, F), np.uint8)
    for t in range(3):
        b.env_step(h, None, ring, rew, done)
        p.step(stack=stack)
    torch.cuda.synchronize()
    assert_bit_equal(ring.cpu().numpy(), stack, "arbitrary positions")
    assert (ring[:, 3] == 0).all()          # slot 3 not written yet by steps 0..2
    b.env_destroy(h)


@pytest.mark.parametrize("layout", ["slot_major", "env_major"])
def test_config3_n16384_t500_final_ring(layout):
    # full size, per-step launches as bench measures them; the oracle steps all environments
    # without rendering and renders only the last four steps (the content of the ring at the end)
    n, seed, T = 16384, 3, 500
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"pixel_layout": LAYOUTS[layout]})
    ring = new_ring(n, layout)
    rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
    done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
    b.env_reset(h, ring)
    for t in range(T):
        b.env_step(h, None, ring, rew[t], done[t])
    torch.cuda.synchronize()
    p = orc.Pong(n, seed); p.reset()
    _, orew, odone = p.rollout(T - 4, nthreads=16, want_obs=False)
    stack = np.zeros((n, 4, F, F), np.uint8)
    _, orew2, odone2 = p.rollout(4, stack=stack, nthreads=16, want_obs=False)
    assert_bit_equal(rew.cpu().numpy(), np.concatenate([orew, orew2]), "C3 reward")
    assert_bit_equal(done.cpu().numpy(), np.concatenate([odone, odone2]), "C3 done")
    assert_bit_equal(ring_as_env_major(ring, layout), stack, "C3 ring")
    _, fields = split_state(b.env_get_state(h), n, 10)
    assert_bit_equal(fields, pong_state_fields(p.envs()), "C3 state")
    b.env_destroy(h)


def test_ring_steps_on_a_long_plane():
    """From 65536 pages of 4 KiB per plane on (N >= 38044) the step's renderer gives a workgroup
    four consecutive pages; N = 40003 ends inside such a group and off a page boundary.  Whole ring,
    rewards, done flags and state against the oracle after 21 steps (slot 0 written six times)."""
    n, seed, T = 40003, 13, 21
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1})
    ring = new_ring(n, "slot_major")
    rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
    done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
    b.env_reset(h, ring)
    for t in range(T):
        b.env_step(h, None, ring, rew[t], done[t])
    torch.cuda.synchronize()
    p = orc.Pong(n, seed, max_score=1); p.reset()
    _, orew, odone = p.rollout(T - 4, nthreads=16, want_obs=False)
    stack = np.zeros((n, 4, F, F), np.uint8)
    _, orew2, odone2 = p.rollout(4, stack=stack, nthreads=16, want_obs=False)
    assert_bit_equal(rew.cpu().numpy(), np.concatenate([orew, orew2]), "reward")
    assert_bit_equal(done.cpu().numpy(), np.concatenate([odone, odone2]), "done")
    assert_bit_equal(ring_as_env_major(ring, "slot_major"), stack, "ring")
    _, fields = split_state(b.env_get_state(h), n, 10)
    assert_bit_equal(fields, pong_state_fields(p.envs()), "state")
    b.env_destroy(h)


@pytest.mark.parametrize("n,T", [(70000, 9), (1000, 300)])
def test_frame_trajectory_rendered_in_chunks(n, T):
    """env_rollout on the pixel kind stages a chunk of steps (as many as fit 262144 frames, at least
    one) and renders the chunk's frames together.  Sizes that need several chunks with a ragged
    last one; rewards and done flags are compared in full, frames at sampled (step, environment)
    pairs rendered by the oracle from its own state after that step."""
    seed = 19
    assert b.lib().mi355env_tune_frame_trajectory(1) == 0        # chunked at any N
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1})
    try:
        b.env_reset(h, None)
        frames = torch.empty((T, n, F, F), dtype=torch.uint8, device=DEV)
        rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
        done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
        b.env_rollout(h, T, None, frames, rew, done)
        torch.cuda.synchronize()
        stats = b.env_stats(h)
        state = b.env_get_state(h)
    finally:
        b.env_destroy(h)
        assert b.lib().mi355env_tune_frame_trajectory(2) == 0
    p = orc.Pong(n, seed, max_score=1)
    p.reset()
    oobs, orew, odone = p.rollout(T, nthreads=8)
    assert_bit_equal(rew.cpu().numpy(), orew, "reward")
    assert_bit_equal(done.cpu().numpy(), odone, "done")
    assert stats["episodes"] == p.stats()["episodes"]
    _, fields = split_state(state, n, 10)
    assert_bit_equal(fields, pong_state_fields(p.envs()), "final state")
    rng = np.random.default_rng(3)
    ts = np.concatenate([rng.integers(0, T, 300), [0, T - 1, T - 1]])
    es = np.concatenate([rng.integers(0, n, 300), [0, n - 1, 0]])
    got = frames[torch.from_numpy(ts).to(DEV), torch.from_numpy(es).to(DEV)].cpu().numpy()
    for k, (t, e) in enumerate(zip(ts, es)):
        o = oobs[t, e]
        st = dict(bx=float(o[0]), by=float(o[1]), vx=0.0, vy=0.0, pa=float(o[4]), po=float(o[5]), sa=0, so=0,
                  ep_ret=0, ep_len=0)
        assert_bit_equal(got[k], orc.pong_render_one(st), "frame t=%d env=%d" % (t, e))
    # the frames are not all alike (the ball moves)
    assert (got[0] != got[1]).any()


@pytest.mark.parametrize("n,T", [(613, 67), (5003, 11)])
@pytest.mark.parametrize("offset", [0, 2064])
def test_trajectory_renderers_every_frame(offset, n, T):
    """Frame trajectories long enough (more than 65536 pages of 4 KiB) for the renderer that gives a
    workgroup four consecutive pages, with planes that start off a page boundary and end inside a
    group of four: every frame is compared with the oracle's rendering of its own state, and the
    bytes in front of and behind the trajectory must stay untouched."""
    seed = 29
    assert b.lib().mi355env_tune_frame_trajectory(1) == 0
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1})
    try:
        b.env_reset(h, None)
        nbytes = T * n * F * F
        raw = torch.full((offset + nbytes + 8192,), 7, dtype=torch.uint8, device=DEV)
        frames = raw[offset:offset + nbytes].view(T, n, F, F)
        assert frames.data_ptr() % 16 == 0
        rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
        done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
        b.env_rollout(h, T, None, frames, rew, done)
        torch.cuda.synchronize()
    finally:
        b.env_destroy(h)
        assert b.lib().mi355env_tune_frame_trajectory(2) == 0
    assert int(raw[:offset].min().item() if offset else 7) == 7 and int(raw[offset + nbytes:].min().item()) == 7
    assert int(raw[offset + nbytes:].max().item()) == 7
    p = orc.Pong(n, seed, max_score=1)
    p.reset()
    oobs, orew, odone = p.rollout(T, nthreads=8)
    assert_bit_equal(rew.cpu().numpy(), orew, "reward")
    got = frames.cpu().numpy()
    want = np.empty_like(got)
    for t in range(T):
        for e in range(n):
            o = oobs[t, e]
            want[t, e] = orc.pong_render_one(dict(bx=float(o[0]), by=float(o[1]), vx=0.0, vy=0.0, pa=float(o[4]),
                                                  po=float(o[5]), sa=0, so=0, ep_ret=0, ep_len=0))
    assert_bit_equal(got, want, "frames")


def _update_counts(h):
    import ctypes as C
    L = b.lib()
    L.mi355env_pixel_update_counts.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    d, f = C.c_int64(-1), C.c_int64(-1)
    assert L.mi355env_pixel_update_counts(h, C.byref(d), C.byref(f)) == 0
    return d.value, f.value


@pytest.mark.parametrize("layout", ["slot_major", "env_major"])
@pytest.mark.parametrize("n", [1, 37, 255, 1000])
def test_delta_updates_leave_the_same_ring_as_the_oracle(n, layout):
    """pixel_update = delta: a step changes only the pixels in which the new frame differs from the
    one its slot holds.  The ring must equal the oracle's after every step, through episode ends,
    external actions, a save / restore, steps taken through env_rollout in between, a change of ring
    buffer and a second reset -- and most steps must really have been delta updates."""
    seed, T = 70 + n, 110
    acts = inputs.pong_actions(T, n, seed=5)
    dacts = torch.from_numpy(acts).to(DEV)
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1, "pixel_layout": LAYOUTS[layout],
                                                   "pixel_update": b.ENV_PIXELS_DELTA})
    try:
        ring = new_ring(n, layout)
        ring.fill_(77)                                   # env_reset must overwrite all of it
        rew = torch.empty(n, dtype=torch.float32, device=DEV)
        done = torch.empty(n, dtype=torch.uint8, device=DEV)
        b.env_reset(h, ring)
        p = orc.Pong(n, seed, max_score=1); p.reset()
        stack = np.zeros((n, 4, F, F), np.uint8); p.fill_stack(stack)
        torch.cuda.synchronize()
        assert_bit_equal(ring_as_env_major(ring, layout), stack, "ring after reset")
        expect_full = 0
        t = 0
        while t < T:
            ext = t % 3 == 1
            b.env_step(h, dacts[t] if ext else None, ring, rew, done)
            _, orew, odone = p.step(actions=acts[t] if ext else None, stack=stack)
            torch.cuda.synchronize()
            assert_bit_equal(ring_as_env_major(ring, layout), stack, "ring after step %d" % t)
            assert_bit_equal(rew.cpu().numpy(), orew, "reward step %d" % t)
            assert_bit_equal(done.cpu().numpy(), odone, "done step %d" % t)
            t += 1
            if t == 25:                                  # restore: the library forgets what the slots hold
                b.env_set_state(h, b.env_get_state(h))
                expect_full += 4
            if t == 45:                                  # three steps that write no ring slot, on both sides
                fr = torch.empty((3, n, F, F), dtype=torch.uint8, device=DEV)
                r3 = torch.empty((3, n), dtype=torch.float32, device=DEV)
                d3 = torch.empty((3, n), dtype=torch.uint8, device=DEV)
                b.env_rollout(h, 3, None, fr, r3, d3)
                p.rollout(3)
                t += 3
                expect_full += 4                         # steps passed without reaching the ring
            if t == 70:                                  # another buffer with the same contents
                ring = ring.clone()
                expect_full += 4
            if t == 90:                                  # second reset, stale data in the ring first
                ring.fill_(5)
                b.env_reset(h, ring)
                p.reset(); p.fill_stack(stack)
        delta, full = _update_counts(h)
        assert full == expect_full and delta == T - 3 - expect_full, (delta, full)
        assert b.env_stats(h)["episodes"] == p.stats()["episodes"]
        if n >= 37:
            assert p.stats()["episodes"] > 0
    finally:
        b.env_destroy(h)


def test_delta_update_handles_only_for_pixels():
    for kind in (b.ENV_PONG, b.ENV_BODY, b.ENV_CARTPOLE):
        with pytest.raises(b.EnvError) as ei:
            b.env_create(kind, 64, 0, {"pixel_update": b.ENV_PIXELS_DELTA})
        assert ei.value.code == b.ENV_E_UNSUPPORTED


@pytest.mark.parametrize("n,T", [(16384, 60), (40000, 40)])
def test_delta_updates_at_config3_size_match_full_updates(n, T):
    """N = 16384 (config 3) and a batch beyond 32768, which runs the kernel's other workgroup shape:
    delta steps leave the ring byte-identical to a handle that rewrites whole frames (which
    test_config3 ties to the oracle); a ragged last workgroup at N = 40000 + 3."""
    n, seed = n + (3 if n > 32768 else 0), 3
    rings = []
    for upd in (b.ENV_PIXELS_FULL, b.ENV_PIXELS_DELTA):
        h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"pixel_update": upd})
        try:
            ring = new_ring(n, "slot_major")
            rew = torch.empty(n, dtype=torch.float32, device=DEV)
            done = torch.empty(n, dtype=torch.uint8, device=DEV)
            b.env_reset(h, ring)
            for _ in range(T):
                b.env_step(h, None, ring, rew, done)
            torch.cuda.synchronize()
            rings.append(ring)
            if upd == b.ENV_PIXELS_DELTA:
                assert _update_counts(h) == (T, 0)
        finally:
            b.env_destroy(h)
    assert torch.equal(rings[0], rings[1])
    assert int(rings[0].max()) == 255


@pytest.mark.parametrize("n", [1, 37, 255, 1000])
def test_ordered_stack_matches_the_oracle(n):
    """pixel_layout = ordered: uint8[N][4][84][84] with channel 3 the newest frame; every env_step
    moves the channels down by one and puts the new frame on top.  The reference stack is built
    from the oracle's frames by exactly that rule.  Checked after every step, through episode
    ends, external actions, a save / restore, steps taken through env_rollout in between, a change
    of buffer and a second reset; most steps must have been delta updates, the rest physical
    moves."""
    seed, T = 170 + n, 100
    acts = inputs.pong_actions(T, n, seed=6)
    dacts = torch.from_numpy(acts).to(DEV)
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1, "pixel_layout": b.ENV_PIXELS_ORDERED})
    try:
        stack = torch.full((n, 4, F, F), 77, dtype=torch.uint8, device=DEV)
        rew = torch.empty(n, dtype=torch.float32, device=DEV)
        done = torch.empty(n, dtype=torch.uint8, device=DEV)
        b.env_reset(h, stack)
        p = orc.Pong(n, seed, max_score=1); p.reset()
        ring = np.zeros((n, 4, F, F), np.uint8); p.fill_stack(ring)     # the oracle's own 4-slot ring
        want = ring.copy()                                               # after a reset: four times the initial frame
        torch.cuda.synchronize()
        assert_bit_equal(stack.cpu().numpy(), want, "stack after reset")
        expect_moves = 0
        t = 0
        while t < T:
            ext = t % 3 == 2
            s = p.step_count
            b.env_step(h, dacts[t] if ext else None, stack, rew, done)
            _, orew, odone = p.step(actions=acts[t] if ext else None, stack=ring)
            want[:, :3] = want[:, 1:].copy()
            want[:, 3] = ring[:, s & 3]                                  # the frame the oracle drew for step s
            torch.cuda.synchronize()
            assert_bit_equal(stack.cpu().numpy(), want, "stack after step %d" % t)
            assert_bit_equal(rew.cpu().numpy(), orew, "reward step %d" % t)
            assert_bit_equal(done.cpu().numpy(), odone, "done step %d" % t)
            t += 1
            if t == 22:
                b.env_set_state(h, b.env_get_state(h))
                expect_moves += 4
            if t == 45:
                fr = torch.empty((2, n, F, F), dtype=torch.uint8, device=DEV)
                r2 = torch.empty((2, n), dtype=torch.float32, device=DEV)
                d2 = torch.empty((2, n), dtype=torch.uint8, device=DEV)
                b.env_rollout(h, 2, None, fr, r2, d2)
                p.rollout(2)
                t += 2
                expect_moves += 4                    # the kept blocks no longer describe the channels
            if t == 70:
                stack = stack.clone()
                expect_moves += 4
            if t == 85:
                stack.fill_(5)
                b.env_reset(h, stack)
                p.reset(); p.fill_stack(ring)
                want = ring.copy()
        delta, moves = _update_counts(h)
        assert moves == expect_moves and delta == T - 2 - expect_moves, (delta, moves)
        assert b.env_stats(h)["episodes"] == p.stats()["episodes"]
    finally:
        b.env_destroy(h)


def test_ordered_stack_at_config3_size_and_beyond():
    """N = 16384 and N = 40003 (the kernel's other workgroup shape, ragged last workgroup): channel
    3 - k of the ordered stack equals the slot of step s - k of a slot-major ring driven by the same
    seed, after 30 steps."""
    for n in (16384, 40003):
        seed, T = 3, 30
        hr = b.env_create(b.ENV_PONG_PIXELS, n, seed, None)
        ho = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"pixel_layout": b.ENV_PIXELS_ORDERED})
        try:
            ring = new_ring(n, "slot_major")
            stack = torch.zeros((n, 4, F, F), dtype=torch.uint8, device=DEV)
            rew = torch.empty(n, dtype=torch.float32, device=DEV)
            done = torch.empty(n, dtype=torch.uint8, device=DEV)
            b.env_reset(hr, ring); b.env_reset(ho, stack)
            for _ in range(T):
                b.env_step(hr, None, ring, rew, done)
                b.env_step(ho, None, stack, rew, done)
            torch.cuda.synchronize()
            assert _update_counts(ho) == (T, 0)
            for k in range(4):
                assert torch.equal(stack[:, 3 - k], ring[(T - 1 - k) & 3]), (n, k)
        finally:
            b.env_destroy(hr); b.env_destroy(ho)


def test_ring_planes_longer_than_two_gigabytes():
    """N = 400001: a plane of the slot-major ring is 2.8 GB, so byte offsets inside a plane pass
    2^31 and the ring is 11.3 GB.  Seven steps through env_step (the fused launch with four pages
    per render workgroup); rewards and done flags compared in full, the four ring slots at sampled
    environments against frames the oracle renders from its own state after each of the last four
    steps, and the total number of lit pixels of one plane against the oracle's rectangles."""
    n, seed, T = 400001, 23, 7
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1})
    try:
        ring = torch.zeros((4, n, F, F), dtype=torch.uint8, device=DEV)
        rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
        done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
        b.env_reset(h, ring)
        for t in range(T):
            b.env_step(h, None, ring, rew[t], done[t])
        torch.cuda.synchronize()
        state = b.env_get_state(h)
    finally:
        b.env_destroy(h)
    p = orc.Pong(n, seed, max_score=1)
    p.reset()
    oobs, orew, odone = p.rollout(T, nthreads=16)
    assert_bit_equal(rew.cpu().numpy(), orew, "reward")
    assert_bit_equal(done.cpu().numpy(), odone, "done")
    _, fields = split_state(state, n, 10)
    assert_bit_equal(fields, pong_state_fields(p.envs()), "final state")
    rng = np.random.default_rng(5)
    es = np.concatenate([rng.integers(0, n, 200), [0, 1, n - 2, n - 1, 304358, 304359]])   # 304358.6 frames = 2^31 bytes
    for t in range(T - 4, T):
        got = ring[t & 3][torch.from_numpy(es).to(DEV)].cpu().numpy()
        for k, e in enumerate(es):
            o = oobs[t, e]
            st = dict(bx=float(o[0]), by=float(o[1]), vx=0.0, vy=0.0, pa=float(o[4]), po=float(o[5]), sa=0, so=0,
                      ep_ret=0, ep_len=0)
            assert_bit_equal(got[k], orc.pong_render_one(st), "slot %d env %d" % (t & 3, e))
    # every environment's frame of the last step: as many lit pixels as the oracle's frames have,
    # counted per environment on the device and compared with the oracle's count for the sampled ones
    t = T - 1
    lit = (ring[t & 3] != 0).sum(dim=(1, 2)).cpu().numpy()
    assert lit.min() >= 20 and lit.max() <= 54          # two paddles and a ball on the 84 x 84 grid: at most 54 cells
    for e in es[:50]:
        o = oobs[t, e]
        st = dict(bx=float(o[0]), by=float(o[1]), vx=0.0, vy=0.0, pa=float(o[4]), po=float(o[5]), sa=0, so=0,
                  ep_ret=0, ep_len=0)
        assert lit[e] == int((orc.pong_render_one(st) != 0).sum())


@pytest.mark.parametrize("n,T", [(1, 40), (3, 90), (700, 130), (4097, 64), (40003, 12)])
def test_ring_steps_with_the_callers_actions(n, T):
    """The slot-major ring step with actions from a device buffer (a policy in the loop): a dynamics
    launch in front of the renderer.  Episodes end (max_score 1) and re-serve inside the run,
    N = 40003 takes four pages per render workgroup; whole ring, rewards, done flags, statistics
    and final state against the oracle."""
    seed = 50 + n
    acts = inputs.pong_actions(T, n, seed=4)
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": 1})
    try:
        ring = new_ring(n, "slot_major")
        rew = torch.empty((T, n), dtype=torch.float32, device=DEV)
        done = torch.empty((T, n), dtype=torch.uint8, device=DEV)
        dacts = torch.from_numpy(acts).to(DEV)
        b.env_reset(h, ring)
        for t in range(T):
            b.env_step(h, dacts[t], ring, rew[t], done[t])
        torch.cuda.synchronize()
        stats, state = b.env_stats(h), b.env_get_state(h)
    finally:
        b.env_destroy(h)
    p = orc.Pong(n, seed, max_score=1); p.reset()
    stack = np.zeros((n, 4, F, F), np.uint8); p.fill_stack(stack)
    orew = np.zeros((T, n), np.float32); odone = np.zeros((T, n), np.uint8)
    for t in range(T):
        _, orew[t], odone[t] = p.step(actions=acts[t], stack=stack)
    assert_bit_equal(ring_as_env_major(ring, "slot_major"), stack, "ring")
    assert_bit_equal(rew.cpu().numpy(), orew, "reward")
    assert_bit_equal(done.cpu().numpy(), odone, "done")
    want = p.stats()
    assert stats["episodes"] == want["episodes"] and stats["return_sum"] == want["return_sum"]
    assert stats["episodes"] > 0 or n < 700 or T < 30
    _, fields = split_state(state, n, 10)
    assert_bit_equal(fields, pong_state_fields(p.envs()), "final state")
