"""GPU: env_step_pixels_noalloc, the pixel step that allocates nothing, against env_step on a handle
(the existing entry point) and against the oracle, through the C-ABI.  Two calls in a row share the
library's fixed scratch array, the second with a smaller batch."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import oracle as orc                      # noqa: E402
from paper_2603_12145_amd import binding as b         # noqa: E402
from paper_2603_12145_amd import inputs               # noqa: E402
from gpu_helpers import assert_bit_equal, split_state, pong_state_fields  # noqa: E402

DEV = "cuda:0"
F = 84


def stats_of(t):
    raw = t.cpu().numpy().tobytes()
    s = b.env_stats_t.from_buffer_copy(raw)
    return {k: getattr(s, k) for k, _ in b.env_stats_t._fields_}


def run_case(n, seed, steps, max_score, external, check_oracle):
    """`steps` steps of n environments both ways; every output compared after every step."""
    L = b.lib()
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, {"max_score": max_score})
    ring_h = torch.zeros((4, n, F, F), dtype=torch.uint8, device=DEV)
    b.env_reset(h, ring_h)
    step0, fields = split_state(b.env_get_state(h), n, 10)
    assert step0 == 0
    state = torch.from_numpy(fields.astype(np.int32)).to(DEV)          # the caller's state, [10, n]
    ring = ring_h.clone()
    rew_h = torch.empty(n, dtype=torch.float32, device=DEV); done_h = torch.empty(n, dtype=torch.uint8, device=DEV)
    # outputs start with garbage so that every element must be written
    rew = torch.full((n,), 7.5, dtype=torch.float32, device=DEV); done = torch.full((n,), 9, dtype=torch.uint8, device=DEV)
    stats = torch.zeros(6, dtype=torch.int64, device=DEV)
    acts = torch.from_numpy(inputs.pong_actions(steps, n, seed + 1)).to(DEV) if external else None
    p = stack = None
    if check_oracle:
        p = orc.Pong(n, seed, max_score=max_score); p.reset()
        stack = np.zeros((n, 4, F, F), np.uint8); p.fill_stack(stack)
    stream = torch.cuda.current_stream().cuda_stream
    total = dict(episodes=0, length_sum=0, return_sum=0.0)
    for t in range(steps):
        a = None if acts is None else acts[t]
        b.env_step(h, a, ring_h, rew_h, done_h)
        rc = L.env_step_pixels_noalloc(n, seed, t, max_score, state.data_ptr(), None if a is None else a.data_ptr(),
                                       ring.data_ptr(), rew.data_ptr(), done.data_ptr(), stats.data_ptr(), stream)
        assert rc == b.ENV_OK, b.env_strerror(rc)
        torch.cuda.synchronize()
        assert_bit_equal(ring.cpu().numpy(), ring_h.cpu().numpy(), "ring after step %d" % t)
        assert_bit_equal(rew.cpu().numpy(), rew_h.cpu().numpy(), "reward step %d" % t)
        assert_bit_equal(done.cpu().numpy(), done_h.cpu().numpy(), "done step %d" % t)
        _, want_fields = split_state(b.env_get_state(h), n, 10)
        assert_bit_equal(state.cpu().numpy().view(np.uint32), want_fields, "state after step %d" % t)
        st = stats_of(stats)
        assert st["episodes"] == int(done.sum().item()) and st["nonfinite"] == 0
        for k in total:
            total[k] += st[k]
        if check_oracle:
            _, orew, odone = p.step(actions=None if acts is None else acts[t].cpu().numpy(), stack=stack)
            assert_bit_equal(np.ascontiguousarray(ring.cpu().numpy().transpose(1, 0, 2, 3)), stack, "ring vs oracle, step %d" % t)
            assert_bit_equal(rew.cpu().numpy(), orew, "reward vs oracle")
            assert_bit_equal(done.cpu().numpy(), odone, "done vs oracle")
    want = b.env_stats(h)
    b.env_destroy(h)
    assert total["episodes"] == want["episodes"] and total["length_sum"] == want["length_sum"]
    assert total["return_sum"] == want["return_sum"]
    if check_oracle:
        assert_bit_equal(state.cpu().numpy().view(np.uint32), pong_state_fields(p.envs()), "state vs oracle")
    return total["episodes"]


def test_two_calls_in_a_row_the_second_smaller():
    # first a batch that spans many pages and a ragged tail, then a smaller one with another seed:
    # what the first call left in the scratch array (cell blocks of environments beyond the second
    # batch, statistics) must not show
    ep1 = run_case(3000, 61, 40, 1, external=False, check_oracle=True)
    ep2 = run_case(777, 62, 40, 1, external=True, check_oracle=True)
    assert ep1 > 0 and ep2 > 0
    # and larger again, on a plane that is 4 KiB-aligned
    run_case(8192, 63, 5, 21, external=False, check_oracle=False)


def test_largest_batch_and_sizes_beyond_it():
    n = b.ENV_NOALLOC_MAX_ENVS
    run_case(n, 64, 2, 1, external=False, check_oracle=False)      # long plane: four pages per workgroup
    L = b.lib()
    state = torch.zeros((10, 64), dtype=torch.int32, device=DEV)
    ring = torch.zeros((4, 64, F, F), dtype=torch.uint8, device=DEV)
    rew = torch.zeros(64, dtype=torch.float32, device=DEV); done = torch.zeros(64, dtype=torch.uint8, device=DEV)
    args = (state.data_ptr(), None, ring.data_ptr(), rew.data_ptr(), done.data_ptr(), None, None)
    assert L.env_step_pixels_noalloc(n + 1, 1, 0, 21, *args) == b.ENV_E_TOO_LARGE
    assert "fixed" in b.env_strerror(b.ENV_E_TOO_LARGE)
    assert L.env_step_pixels_noalloc(0, 1, 0, 21, *args) == b.ENV_E_ARG
    assert L.env_step_pixels_noalloc(64, 1, 0, 0, *args) == b.ENV_E_ARG
    # buffers far too small for the batch (beyond the allocation they live in; a caching allocator's
    # allocation is its pool segment), NULL and host pointers are refused before anything is launched
    assert L.env_step_pixels_noalloc(60000, 1, 0, 21, *args) == b.ENV_E_ARG
    assert L.env_step_pixels_noalloc(64, 1, 0, 21, None, None, ring.data_ptr(), rew.data_ptr(), done.data_ptr(),
                                     None, None) == b.ENV_E_ARG
    host = np.zeros(64, np.float32)
    assert L.env_step_pixels_noalloc(64, 1, 0, 21, state.data_ptr(), None, ring.data_ptr(),
                                     host.ctypes.data_as(C.c_void_p), done.data_ptr(), None, None) == b.ENV_E_ARG
    torch.cuda.synchronize()
    assert int(ring.sum().item()) == 0 and int(done.sum().item()) == 0      # nothing was touched
    assert L.env_step_pixels_noalloc(64, 1, 0, 21, *args) == b.ENV_OK       # stats_dev = NULL is allowed
    torch.cuda.synchronize()
    assert int(ring[0].sum().item()) > 0 and int(ring[1:].sum().item()) == 0


def test_a_call_recorded_in_a_graph_replays():
    # the caller that cannot allocate: a captured step, replayed with direct work in between
    n, seed = 1500, 71
    L = b.lib()
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, None)
    ring_h = torch.zeros((4, n, F, F), dtype=torch.uint8, device=DEV)
    b.env_reset(h, ring_h)
    _, fields = split_state(b.env_get_state(h), n, 10)
    state0 = torch.from_numpy(fields.astype(np.int32)).to(DEV)
    state = state0.clone()
    ring = torch.zeros_like(ring_h)
    rew = torch.empty(n, dtype=torch.float32, device=DEV); done = torch.empty(n, dtype=torch.uint8, device=DEV)
    stats = torch.zeros(6, dtype=torch.int64, device=DEV)
    rew_h = torch.empty_like(rew); done_h = torch.empty_like(done)
    b.env_step(h, None, ring_h, rew_h, done_h)                              # step 0 on the handle
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        b.env_step_pixels_noalloc(n, seed, 0, 21, state, None, ring, rew, done, stats, stream=st)   # buffers become known
        st.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            b.env_step_pixels_noalloc(n, seed, 0, 21, state, None, ring, rew, done, stats, stream=st)
        for k in range(3):                                                  # every replay: step 0 from the same state
            state.copy_(state0); ring.zero_(); rew.fill_(3.0)
            g.replay()
            st.synchronize()
            assert_bit_equal(ring[0].cpu().numpy(), ring_h[0].cpu().numpy(), "slot 0, replay %d" % k)
            assert int(ring[1:].sum().item()) == 0
            assert_bit_equal(rew.cpu().numpy(), rew_h.cpu().numpy(), "reward, replay %d" % k)
            _, want = split_state(b.env_get_state(h), n, 10)
            assert_bit_equal(state.cpu().numpy().view(np.uint32), want, "state, replay %d" % k)
        del g
    b.env_destroy(h)
