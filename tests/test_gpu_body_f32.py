"""GPU: the articulated body computed in float32 (body_arithmetic = ENV_BODY_F32, the precision the
paper's case study states, App. A.1) against the CPU oracle, through the C-ABI.

This instantiation is an option, not the default: float32 arithmetic cannot meet the single-step
bar of 1e-5 per component on every environment (the float32 ORACLE misses it against the float64
one on 0.1-6 % of the environments, by the same margins), so what is asserted here is what float32
can deliver -- single steps as close to the float64 oracle as the float32 oracle is, bit-identical
fused and per-step launches, and 1000-step return statistics within 1 %."""
import math

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle.body_binding import Body                   # noqa: E402
from paper_2603_12145_amd import binding as b         # noqa: E402
from gpu_helpers import assert_bit_equal, tost_p       # noqa: E402
from test_gpu_body import bufs, blob_from_oracle_state, state_from_blob, rel_err   # noqa: E402

DEV = "cuda:0"


def cfg_of(solver):
    c = {"body_arithmetic": b.ENV_BODY_F32}
    if solver:
        c["contact_solver"] = b.ENV_CONTACT_NEWTON
    return c


@pytest.mark.parametrize("solver", [0, 1], ids=["penalty", "newton"])
@pytest.mark.parametrize("warm", [0, 60, 400])
def test_single_steps_are_as_close_to_float64_as_the_float32_oracle(warm, solver):
    n, seed = 4096, 4
    o = Body(n, seed, np.float64, solver=solver); o.reset()
    if warm:
        o.rollout(warm, nthreads=8, want_obs=False)
    s = o.get_state().astype(np.float32).astype(np.float64)
    o.set_state(s); o.step_count = warm
    o64, r64, d64 = o.rollout(1, nthreads=8)
    o32 = Body(n, seed, np.float32, solver=solver); o32.set_state(s.astype(np.float32)); o32.step_count = warm
    oo32, _, _ = o32.rollout(1, nthreads=8)
    h = b.env_create(b.ENV_BODY, n, seed, cfg_of(solver))
    b.env_set_state(h, blob_from_oracle_state(warm, s))
    obs, rew, done = bufs(1, n)
    b.env_step(h, None, obs[0], rew[0], done[0])
    torch.cuda.synchronize()
    b.env_destroy(h)
    g = obs[0].cpu().numpy()
    e_gpu = np.maximum(rel_err(g, o64[0]).max(axis=1), rel_err(rew[0].cpu().numpy(), r64[0]))
    e_orc = rel_err(oo32[0], o64[0]).max(axis=1)
    print("f32 kernel vs f64 oracle: median %.2e 99.9%% %.2e max %.2e, beyond 1e-5: %d | f32 oracle vs f64 oracle: "
          "median %.2e 99.9%% %.2e max %.2e, beyond 1e-5: %d"
          % (np.median(e_gpu), np.quantile(e_gpu, .999), e_gpu.max(), (e_gpu > 1e-5).sum(),
             np.median(e_orc), np.quantile(e_orc, .999), e_orc.max(), (e_orc > 1e-5).sum()))
    assert np.array_equal(done[0].cpu().numpy(), d64[0])
    assert np.median(e_gpu) < 3e-6
    # no worse than the float32 oracle's own distance from the float64 one, with a factor of 3 of slack
    assert np.quantile(e_gpu, .999) < 3 * max(np.quantile(e_orc, .999), 1e-5)
    assert e_gpu.max() < 5 * max(e_orc.max(), 1e-5)


@pytest.mark.parametrize("solver", [0, 1], ids=["penalty", "newton"])
def test_fused_equals_per_step_and_env_i_does_not_depend_on_the_batch(solver):
    seed, T = 8, 30
    outs = {}
    for n, fused in ((70, True), (70, False), (1000, True)):
        cfg = dict(cfg_of(solver), max_episode_steps=12)
        h = b.env_create(b.ENV_BODY, n, seed, cfg)
        b.env_reset(h, None)
        obs, rew, done = bufs(T, n)
        if fused:
            b.env_rollout(h, T, None, obs, rew, done)
        else:
            for t in range(T):
                b.env_step(h, None, obs[t], rew[t], done[t])
        torch.cuda.synchronize()
        st = b.env_stats(h)
        outs[(n, fused)] = (obs[:, :70].cpu().numpy(), rew[:, :70].cpu().numpy(), done[:, :70].cpu().numpy())
        b.env_destroy(h)
        assert st["episodes"] == 2 * n and st["nonfinite"] == 0
    for k in range(3):
        assert_bit_equal(outs[(70, True)][k], outs[(70, False)][k], "fused vs per-step, output %d" % k)
        assert_bit_equal(outs[(70, True)][k], outs[(1000, True)][k], "N = 70 vs N = 1000, output %d" % k)
    # and it is a different computation from the float64 default
    h = b.env_create(b.ENV_BODY, 70, seed, {"max_episode_steps": 12})
    b.env_reset(h, None)
    obs, rew, done = bufs(T, 70)
    b.env_rollout(h, T, None, obs, rew, done)
    torch.cuda.synchronize()
    b.env_destroy(h)
    assert not np.array_equal(obs.cpu().numpy(), outs[(70, True)][0])


@pytest.mark.parametrize("solver", [0, 1], ids=["penalty", "newton"])
def test_n8192_t1000_return_statistics(solver):
    n, seed, T = 8192, 4, 1000
    h = b.env_create(b.ENV_BODY, n, seed, cfg_of(solver))
    b.env_reset(h, None)
    obs, rew, done = bufs(T, n)
    b.env_rollout(h, T, None, obs, rew, done)
    torch.cuda.synchronize()
    st = b.env_stats(h)
    b.env_destroy(h)
    g = rew.sum(dim=0, dtype=torch.float64).cpu().numpy()
    assert st["nonfinite"] == 0 and st["episodes"] == n and bool(torch.isfinite(obs).all().item())
    del obs, rew, done
    o = Body(n, seed, np.float32, solver=solver); o.reset()
    _, orew, _ = o.rollout(T, nthreads=16, want_obs=False)
    r = orew.astype(np.float64).sum(0)

    def se_of_std(x):
        d = x - x.mean()
        return math.sqrt(max((d ** 4).mean() - x.var() ** 2, 0.0) / (4 * len(x) * x.var()))
    se_std = math.sqrt(se_of_std(g) ** 2 + se_of_std(r) ** 2)
    print("f32 kernel returns: mean %.3f sd %.2f | f32 oracle: mean %.3f sd %.2f" % (g.mean(), g.std(), r.mean(), r.std()))
    assert abs(g.mean() - r.mean()) < 0.01 * abs(r.mean())
    p_tost = tost_p(g.mean() - r.mean(), math.sqrt((g.var() + r.var()) / n), 0.01 * abs(r.mean()))
    print("two one-sided tests, margin 1 %% of the mean return: p = %.2g (8192 returns per side: reported, not asserted)" % p_tost)
    assert abs(g.std() - r.std()) < 3.0 * se_std          # two independent samples: see test_gpu_body.py


def test_only_the_body_has_the_option():
    import ctypes as C
    h = C.c_void_p()
    c = b.env_config_t(struct_size=C.sizeof(b.env_config_t), armature=-1, joint_damping=-1, friction_mu=-1,
                       body_arithmetic=b.ENV_BODY_F32)
    assert b.lib().env_create(C.byref(h), b.ENV_PONG, 64, 0, C.byref(c), None) == b.ENV_E_UNSUPPORTED
    c.body_arithmetic = 9
    assert b.lib().env_create(C.byref(h), b.ENV_BODY, 64, 0, C.byref(c), None) == b.ENV_E_ARG
