#!/usr/bin/env python3
"""Benchmark of the vectorised-environment hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--skip-extra] [--skip-cpu]

A "step" is one env_rollout launch of the headline workload: Pong, N = 65536 environments x
T = 1000 steps fused into one kernel (seed 2), writing obs[T,N,8] f32, reward[T,N] f32 and
done[T,N] u8 — Philox draws, dynamics, auto-reset, trajectory stores and episode statistics all
inside the launch.  Buffers are resident in HBM before the timed region.  One JSON line is printed.

`roofline` is for the rollout kernel: algorithmic bytes (37 B per env-step x N x T) divided by the
mean launch duration measured with HIP events on the launch stream, against 8 TB/s.
`cpu_baseline` times the CPU oracle (test infrastructure) on the same workload on the host cores.
`extra` carries the other hot-path rows (per-step launches, pixel render, rigid body) measured the
same way, and a plain fill kernel as the write-bandwidth yardstick.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
PONG_BYTES_PER_ENV_STEP = 37   # 32 obs + 4 reward + 1 done
CARTPOLE_BYTES_PER_ENV_STEP = 21   # 16 obs + 4 reward + 1 done
CARTPOLE_VALU_PER_ENV_STEP = 197   # SQ_INSTS_VALU per wavefront and step (profiles/cartpole_rollout_n65536_t1000.md: 196.8)
VALU_PEAK_TINSTR = 39.3            # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, lane-instructions per second / 1e12
FRAME_BYTES = 84 * 84          # one new frame per env-step
FP32_PEAK_TFLOPS = 157.3       # MI355X vector float32, packed operations counted
FP64_PEAK_TFLOPS = 78.6        # MI355X vector float64 (256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz)
BODY_NEWTON_FLOP_PER_ENV_STEP = 13540   # 5 substeps x (1526 outside the Newton loop + 1.05 solves per environment x 1126), counted in the kernel ISA; a wavefront executes max-over-lanes solves (3.0 on average), which is not counted as useful work
BODY_FLOP_PER_ENV_STEP = 9400   # 5 substeps x 1876 flops (FMA = 2) of a single-lane formulation, read off the compiled substep loop; the kernel's own count is SQ_INSTS_VALU = 918 (float64) / 739 (float32) vector instructions per lane and substep, two lanes per environment (profiles/body_rollout_n8192_t1000.md)


def _traffic(key):
    """Measured HBM bytes per launch (rocprofv3 --pmc, see profiles/), or None."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        return json.load(open(path)).get(key)
    except (OSError, ValueError):
        return None


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _mean_std(xs):
    m = sum(xs) / len(xs)
    v = sum((x - m) ** 2 for x in xs) / max(1, len(xs) - 1)
    return m, v ** 0.5


PREROLL_S = 0.08   # see preroll()
REPEATS = 5         # timed regions of the headline (the paper's protocol: five runs, mean +- std)


def preroll(fn, seconds=PREROLL_S):
    """Keeps the device busy with fn() for `seconds` and returns the number of launches made.

    After ANY idle period, however short (0.5 ms is enough, 5 ms does it fully), this device runs
    the next 30-35 ms of work on lower clocks: the same launch takes 0.41 ms, then up to 0.55 ms
    around the eighth launch, and settles at 0.378 ms only some seventy launches later.  A
    measurement that starts within that window times the power management, not the kernel, so
    every timed region here is preceded by this fixed-time run of the same launches with no idle
    gap in between (a synchronize and a few microseconds of host code do not count as idle; a
    buffer allocation or a host-side computation does).  What preceded the timed region is
    recorded in the JSON line."""
    import torch
    t_end = time.perf_counter() + seconds
    batch, launches = 4, 0
    while time.perf_counter() < t_end:
        t0 = time.perf_counter()
        for _ in range(batch):
            fn()
        torch.cuda.synchronize()
        launches += batch
        if time.perf_counter() - t0 < 0.004:
            batch = min(2 * batch, 4096)
    return launches


def time_launches(fn, steps, warmup, preroll_s=PREROLL_S, repeats=1):
    """Pre-roll (fixed time, see preroll), then fn() warmup + steps times; returns (wall seconds for
    the timed steps, list of per-launch milliseconds from HIP events recorded on the current
    stream).  repeats > 1: the timed region is repeated that many times back to back and a list of
    (wall, per-launch ms) pairs is returned instead."""
    import torch
    events = [(_events(steps), _events(steps)) for _ in range(repeats)]   # made before the device is warmed up
    if preroll_s > 0:
        preroll(fn, preroll_s)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    if repeats > 1:
        out = []
        for starts, ends in events:
            t0 = time.perf_counter()
            for k in range(steps):
                starts[k].record()
                fn()
                ends[k].record()
            torch.cuda.synchronize()
            out.append((time.perf_counter() - t0, starts, ends))
        return [(w, [s.elapsed_time(e) for s, e in zip(ss, ee)]) for w, ss, ee in out]
    starts, ends = events[0]
    t0 = time.perf_counter()
    for k in range(steps):
        starts[k].record()
        fn()
        ends[k].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, [s.elapsed_time(e) for s, e in zip(starts, ends)]


def bench_pong_rollout(b, torch, n, T, seed, steps, warmup, repeats=1):
    """repeats > 1: the timed region of `steps` launches is taken that many times back to back; the
    first one is the result, `runs` lists env-steps/s and mean launch ms of every one."""
    dev = "cuda:0"
    h = b.env_create(b.ENV_PONG, n, seed, None)
    obs = torch.empty((T, n, 8), dtype=torch.float32, device=dev)
    rew = torch.empty((T, n), dtype=torch.float32, device=dev)
    done = torch.empty((T, n), dtype=torch.uint8, device=dev)
    b.env_reset(h, None)
    fn = lambda: b.env_rollout(h, T, None, obs, rew, done)
    if repeats > 1:
        regions = time_launches(fn, steps, warmup, repeats=repeats)
    else:
        regions = [time_launches(fn, steps, warmup)]
    stats = b.env_stats(h)
    b.env_destroy(h)
    del obs, rew, done
    import ctypes as C
    b.lib().mi355env_pace_choice.argtypes = [C.c_int64]
    pace = b.lib().mi355env_pace_choice(n)          # what the library measured for this batch size, if anything
    wall, ms = regions[0]
    mean_ms, std_ms = _mean_std(ms)
    return dict(wall=wall, mean_ms=mean_ms, std_ms=std_ms, min_ms=min(ms), max_ms=max(ms),
                env_steps=n * T * steps, episodes=stats["episodes"], pace_choice_gbs=pace,
                runs=[dict(env_steps_per_s=n * T * steps / w, launch_ms_mean=_mean_std(m)[0]) for w, m in regions])


def bench_pong_per_step(b, torch, n, seed, launches, kind="pong"):
    """One env_step launch per step, the same buffers every step (kind: "pong" or "cartpole")."""
    dev = "cuda:0"
    env_kind, obs_dim, step_bytes = {"pong": (b.ENV_PONG, 8, 101), "cartpole": (b.ENV_CARTPOLE, 4, 61)}[kind]
    h = b.env_create(env_kind, n, seed, None)
    obs = torch.empty((n, obs_dim), dtype=torch.float32, device=dev)
    rew = torch.empty(n, dtype=torch.float32, device=dev)
    done = torch.empty(n, dtype=torch.uint8, device=dev)
    b.env_reset(h, None)
    L = b.lib()

    def loop(fn):
        preroll(fn)
        t0 = time.perf_counter()
        for _ in range(launches):
            fn()
        t1 = time.perf_counter()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, t1 - t0

    # the binding call as a user makes it, same buffers every step: launched without kernel arguments
    # from the second call on, so the host's share (marshalling included) hides behind the device
    wall, host_enqueue = loop(lambda: b.env_step(h, None, obs, rew, done))
    # the same with the arguments marshalled once
    wall_prepared, _ = loop(b.PreparedStep(h, None, obs, rew, done))
    # and with the step kernel that takes its descriptor as a kernel argument: bound by the host's
    # launch path
    assert L.mi355env_tune_step_kernel(2) == 0
    wall_args, host_args = loop(lambda: b.env_step(h, None, obs, rew, done))
    wall_args_prepared, _ = loop(b.PreparedStep(h, None, obs, rew, done))
    assert L.mi355env_tune_step_kernel(1) == 0
    b.env_destroy(h)
    # the same loop with an empty kernel: what a launch costs from this process on this stream
    import ctypes as C
    L.mi355env_bench_empty.argtypes = [C.c_void_p]
    s = torch.cuda.current_stream().cuda_stream
    empty, _ = loop(lambda: L.mi355env_bench_empty(s))
    # the same launches recorded once in a HIP graph (device-resident step counter) and replayed
    per_graph = 100
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        hg = b.env_create(env_kind, n, seed, {"step_counter": b.ENV_STEP_COUNTER_DEVICE}, stream=st)
        b.env_reset(hg, None)
        b.env_step(hg, None, obs, rew, done)
        st.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            for _ in range(per_graph):
                b.env_step(hg, None, obs, rew, done)
        warm = preroll(g.replay)
        st.synchronize()
        reps = max(1, launches // per_graph)
        t0 = time.perf_counter()
        for _ in range(reps):
            g.replay()
        st.synchronize()
        graph_wall = time.perf_counter() - t0
        graph_steps = b.env_step_count(hg)
        del g
        b.env_destroy(hg)
    assert graph_steps == 1 + per_graph * (warm + reps), graph_steps   # the capture itself runs nothing
    graph_us = 1e6 * graph_wall / (reps * per_graph)
    return dict(workload="%s N=%d, one env_step launch per step" % ("pong vector obs" if kind == "pong" else kind, n),
                graph_replay_us_per_launch=graph_us, graph_env_steps_per_s=n / (graph_us * 1e-6),
                graph_launches_per_graph=per_graph,
                us_per_launch=1e6 * wall / launches, env_steps_per_s=n * launches / wall,
                us_per_launch_host_enqueue=1e6 * host_enqueue / launches,
                us_per_launch_prepared_call=1e6 * wall_prepared / launches,
                with_kernel_arguments=dict(us_per_launch=1e6 * wall_args / launches,
                                           us_per_launch_host_enqueue=1e6 * host_args / launches,
                                           us_per_launch_prepared_call=1e6 * wall_args_prepared / launches),
                bound="dispatch latency", launches=launches,
                empty_kernel_us_per_launch=1e6 * empty / launches, ratio_to_empty_launch=wall / empty,
                hbm_gbs=n * step_bytes / (wall / launches) / 1e9)   # state read and written, obs, reward, done


def bench_launch_costs(b, torch, launches=20000):
    """What a launch costs on this runtime, loops enqueued from C++ (mi355env_bench_launch_loop): an
    empty kernel, a 16 KiB store whose descriptor travels as kernel arguments, and the same store
    by a kernel without a kernel-argument segment.  Host time to enqueue and time until drained."""
    import ctypes as C
    f = b.lib().mi355env_bench_launch_loop
    f.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    dst = torch.empty(16384, dtype=torch.uint8, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    out = {}
    for _ in range(2):                                   # the first round warms the device up
        for kind, name in ((0, "empty"), (1, "store_16k_with_arguments"), (2, "store_16k_no_argument_segment")):
            host, total = C.c_double(), C.c_double()
            rc = f(kind, launches, dst.data_ptr(), dst.numel(), st, C.byref(host), C.byref(total))
            if rc != 0:
                raise RuntimeError("mi355env_bench_launch_loop -> %d" % rc)
            out[name] = dict(host_us_per_launch=host.value, us_per_launch=total.value)
    out["launches"] = launches
    return out


def bench_pixels(b, torch, n, seed, launches, warmup=20, layout="slot_major", device_counter=False,
                 delta=False, external=False):
    """external: the actions come from a device buffer, as they do behind a policy (nothing to look
    ahead to: the step is a dynamics launch and the renderer)."""
    dev = "cuda:0"
    code = {"slot_major": b.ENV_PIXELS_SLOT_MAJOR, "env_major": b.ENV_PIXELS_ENV_MAJOR,
            "ordered": b.ENV_PIXELS_ORDERED}[layout]
    delta = delta or layout == "ordered"
    cfg = {"pixel_layout": code}
    if device_counter:      # one launch per step that a HIP graph can replay (no staged lookahead)
        cfg["step_counter"] = b.ENV_STEP_COUNTER_DEVICE
    if delta:               # opt-in contract: the ring is shared state, a step rewrites only changed pixels
        cfg["pixel_update"] = b.ENV_PIXELS_DELTA
    h = b.env_create(b.ENV_PONG_PIXELS, n, seed, cfg)
    ring = torch.zeros((4, n, 84, 84) if layout == "slot_major" else (n, 4, 84, 84),
                       dtype=torch.uint8, device=dev)
    rew = torch.empty(n, dtype=torch.float32, device=dev)
    done = torch.empty(n, dtype=torch.uint8, device=dev)
    b.env_reset(h, ring)
    act = torch.randint(0, 3, (n,), dtype=torch.uint8, device=dev) if external else None
    preroll(lambda: b.env_step(h, act, ring, rew, done))
    for _ in range(warmup):
        b.env_step(h, act, ring, rew, done)
    torch.cuda.synchronize()
    # a step is one or two small launches: time blocks of 50 steps between one pair of events, so
    # that the event records do not sit between the launches they measure
    block, blocks_ms = 50, []
    t0 = time.perf_counter()
    done_steps = 0
    while done_steps < launches:
        k = min(block, launches - done_steps)
        s, e = _events(2)
        s.record()
        for _ in range(k):
            b.env_step(h, act, ring, rew, done)
        e.record()
        blocks_ms.append((s, e, k))
        done_steps += k
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    graph = {}
    if device_counter:
        per_graph = 20
        st = torch.cuda.Stream()
        st.wait_stream(torch.cuda.current_stream())
        b.env_set_stream(h, st)
        with torch.cuda.stream(st):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                for _ in range(per_graph):
                    b.env_step(h, act, ring, rew, done)
            preroll(g.replay)
            st.synchronize()
            reps = max(1, launches // per_graph)
            tg = time.perf_counter()
            for _ in range(reps):
                g.replay()
            st.synchronize()
            graph_us = 1e6 * (time.perf_counter() - tg) / (reps * per_graph)
            del g
        graph = dict(graph_replay_us_per_step=graph_us,
                     graph_replay_gbs=n * FRAME_BYTES / (graph_us * 1e-6) / 1e9)
    b.env_destroy(h)
    mean_ms = sum(s.elapsed_time(e) for s, e, _ in blocks_ms) / launches
    gbs = n * FRAME_BYTES / (mean_ms * 1e-3) / 1e9
    shape = {"slot_major": "a 4-slot ring (u8[4,N,84,84])", "env_major": "a 4-slot ring (u8[N,4,84,84])",
             "ordered": "an ordered stack (u8[N,4,84,84], newest frame last, all four channels kept current)"}[layout]
    out = dict(workload="pong pixels N=%d, 84x84 u8 frame into %s, one env_step "
                        "call per step%s" % (n, shape,
                                            (", actions from a device buffer" if external else "")
                                            + (", step counter in device memory" if device_counter else "")
                                            + (", delta updates of the slot" if delta else "")),
               **graph,
               env_steps_per_s=n * launches / wall, us_per_step_events=mean_ms * 1e3,
               us_per_step_wall=1e6 * wall / launches, launches=launches)
    if delta:
        # only changed pixels are written, so the frame's 7056 bytes are not this path's traffic and
        # no bandwidth roofline applies: the rate is reported beside the full-write figure instead
        out["bound"] = "scattered partial-line writes (a few dozen bytes per environment), not a stream"
        out["whole_frame_equivalent_gbs"] = gbs
    else:
        out["roofline"] = dict(bound="hbm", achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS,
                               traffic=_traffic("pixel_fused_step_n%d" % n)
                               if layout == "slot_major" and not device_counter and not external else None)
        if out["roofline"]["traffic"] is None:
            out["roofline"]["traffic_note"] = "no counter run for this variant; the full-write variants move 1.03 x the frame bytes"
    return out


def bench_fill(b, torch, nbytes, launches=50):
    """Write bandwidth of two trivial fill kernels: a grid-stride loop, and one 4 KiB page per
    workgroup (the best launch shape found on this device)."""
    import ctypes as C
    L = b.lib()
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    s = torch.cuda.current_stream().cuda_stream
    out = dict(workload="plain 16-byte fill of %d MiB" % (nbytes >> 20))
    for name, fn in (("grid_stride", L.mi355env_bench_fill), ("page_per_workgroup", L.mi355env_bench_fill_pages)):
        fn.argtypes = [C.c_void_p, C.c_size_t, C.c_uint32, C.c_void_p]
        wall, ms = time_launches(lambda: fn(buf.data_ptr(), nbytes, 0, s), launches, 10)
        mean_ms, _ = _mean_std(ms)
        out[name + "_gbs"] = nbytes / (mean_ms * 1e-3) / 1e9
    out["gbs"] = max(out["grid_stride_gbs"], out["page_per_workgroup_gbs"])
    out["frac_of_peak"] = out["gbs"] / HBM_PEAK_GBS
    return out


def bench_store_floor(b, torch, n, T, launches=30):
    """The rollout's trajectory stores with no computation behind them (same buffers, same launch
    shape): issued as fast as they can be, and paced (every wavefront sleeps k x 64 cycles per step;
    the best k is what the memory system can do for obs[T,N,8] + reward[T,N] + done[T,N])."""
    import ctypes as C
    L = b.lib()
    L.mi355env_bench_trajectory_stores_paced.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                                         C.c_int32, C.c_void_p]
    dev = "cuda:0"
    obs = torch.empty((T, n, 8), dtype=torch.float32, device=dev)
    rew = torch.empty((T, n), dtype=torch.float32, device=dev)
    done = torch.empty((T, n), dtype=torch.uint8, device=dev)
    s = torch.cuda.current_stream().cuda_stream

    def timed(sleep, launches, warmup):
        wall, ms = time_launches(lambda: L.mi355env_bench_trajectory_stores_paced(
            obs.data_ptr(), rew.data_ptr(), done.data_ptr(), n, T, sleep, s), launches, warmup)
        return _mean_std(ms)

    mean_ms, std_ms = timed(0, launches, 20)
    gbs = PONG_BYTES_PER_ENV_STEP * n * T / (mean_ms * 1e-3) / 1e9
    paced = {k: timed(k, 10, 3)[0] for k in (9, 10, 11, 12, 13, 14)}
    best = min(paced, key=paced.get)
    best_gbs = PONG_BYTES_PER_ENV_STEP * n * T / (paced[best] * 1e-3) / 1e9
    return dict(workload="stores of the Pong rollout only, N=%d x T=%d" % (n, T), ms_per_launch=mean_ms,
                ms_std=std_ms, gbs=gbs, frac_of_peak=gbs / HBM_PEAK_GBS,
                paced_ms_per_launch={str(k): v for k, v in paced.items()}, best_pace_sleep_units=best,
                best_paced_ms=paced[best], best_paced_gbs=best_gbs, best_paced_frac_of_peak=best_gbs / HBM_PEAK_GBS)


def bench_copy(b, torch, nbytes, launches=20):
    """Plain device-to-device copy of known size: calibrates the HBM byte counters."""
    import ctypes as C
    L = b.lib()
    L.mi355env_bench_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    src = torch.ones(nbytes, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    s = torch.cuda.current_stream().cuda_stream
    wall, ms = time_launches(lambda: L.mi355env_bench_copy(dst.data_ptr(), src.data_ptr(), nbytes, s),
                             launches, 3)
    mean_ms, _ = _mean_std(ms)
    return dict(workload="plain 16-byte copy of %d MiB (reads and writes that many bytes)" % (nbytes >> 20),
                gbs_each_way=nbytes / (mean_ms * 1e-3) / 1e9)


def bench_body(b, torch, n, T, seed, steps, newton=False, f32=False):
    dev = "cuda:0"
    cfg = {}
    if newton:
        cfg["contact_solver"] = b.ENV_CONTACT_NEWTON
    if f32:
        cfg["body_arithmetic"] = b.ENV_BODY_F32
    h = b.env_create(b.ENV_BODY, n, seed, cfg or None)
    obs = torch.empty((T, n, 17), dtype=torch.float32, device=dev)
    rew = torch.empty((T, n), dtype=torch.float32, device=dev)
    done = torch.empty((T, n), dtype=torch.uint8, device=dev)
    b.env_reset(h, None)
    wall, ms = time_launches(lambda: b.env_rollout(h, T, None, obs, rew, done), steps, 1)
    st = b.env_stats(h)
    b.env_destroy(h)
    mean_ms, std_ms = _mean_std(ms)
    if f32:
        # the same flops in float32, against the published float32 vector peak (which assumes packed
        # operations; they are switched off in this build, so the unpacked issue rate, half of it, is
        # the ceiling this code can reach)
        per = BODY_NEWTON_FLOP_PER_ENV_STEP if newton else BODY_FLOP_PER_ENV_STEP
        flops = per * n * T / (mean_ms * 1e-3) / 1e12
        return dict(workload="articulated body%s, float32 arithmetic (opt-in), N=%d x T=%d fused rollout"
                             % (", Newton contact model" if newton else "", n, T),
                    dtype="f32", env_steps_per_s=n * T * steps / wall, ms_per_launch=mean_ms,
                    nonfinite=st["nonfinite"], episodes=st["episodes"],
                    roofline=dict(bound="alu", achieved=flops, peak=FP32_PEAK_TFLOPS, unit="TFLOP/s",
                                  frac=flops / FP32_PEAK_TFLOPS, frac_of_unpacked_rate=flops / FP64_PEAK_TFLOPS,
                                  traffic=None))
    if newton:
        flops = BODY_NEWTON_FLOP_PER_ENV_STEP * n * T / (mean_ms * 1e-3) / 1e12
        return dict(workload="articulated body, Newton contact model, N=%d x T=%d fused rollout" % (n, T),
                    dtype="f64 in-step arithmetic, f32 state and I/O",
                    env_steps_per_s=n * T * steps / wall, ms_per_launch=mean_ms,
                    nonfinite=st["nonfinite"], episodes=st["episodes"],
                    roofline=dict(bound="alu", achieved=flops, peak=FP64_PEAK_TFLOPS, unit="TFLOP/s",
                                  frac=flops / FP64_PEAK_TFLOPS, traffic=None))
    flops = BODY_FLOP_PER_ENV_STEP * n * T / (mean_ms * 1e-3) / 1e12
    return dict(workload="articulated body N=%d x T=%d fused rollout" % (n, T), dtype="f64 in-step arithmetic, f32 state and I/O",
                env_steps_per_s=n * T * steps / wall, ms_per_launch=mean_ms,
                nonfinite=st["nonfinite"], episodes=st["episodes"],
                roofline=dict(bound="alu", achieved=flops, peak=FP64_PEAK_TFLOPS, unit="TFLOP/s",
                              frac=flops / FP64_PEAK_TFLOPS, traffic=_traffic("body_rollout_n%d_t%d" % (n, T))))


def bench_cartpole(b, torch, n, T, seed, steps):
    dev = "cuda:0"
    h = b.env_create(b.ENV_CARTPOLE, n, seed, None)
    obs = torch.empty((T, n, 4), dtype=torch.float32, device=dev)
    rew = torch.empty((T, n), dtype=torch.float32, device=dev)
    done = torch.empty((T, n), dtype=torch.uint8, device=dev)
    b.env_reset(h, None)
    wall, ms = time_launches(lambda: b.env_rollout(h, T, None, obs, rew, done), steps, 20)
    st = b.env_stats(h)
    b.env_destroy(h)
    mean_ms, std_ms = _mean_std(ms)
    gbs = CARTPOLE_BYTES_PER_ENV_STEP * n * T / (mean_ms * 1e-3) / 1e9
    tinstr = CARTPOLE_VALU_PER_ENV_STEP * n * T / (mean_ms * 1e-3) / 1e12
    # bound by vector-instruction issue, not by its 21 B per env-step: the roofline is the issue rate
    # (197 = the instructions one wavefront per 64 environments needs per step; batches up to 65536 run
    # two wavefronts per 64 environments, which issue a few more between them and share a SIMD better)
    return dict(workload="cart-pole N=%d x T=%d fused rollout, in-kernel Philox actions" % (n, T), dtype="f32",
                env_steps_per_s=n * T * steps / wall, ms_per_launch=mean_ms, episodes=st["episodes"],
                hbm_gbs=gbs, hbm_frac=gbs / HBM_PEAK_GBS,
                roofline=dict(bound="alu", achieved=tinstr, peak=VALU_PEAK_TINSTR, unit="T lane-instructions/s",
                              frac=tinstr / VALU_PEAK_TINSTR, traffic=None))


def bench_external_actions(b, torch, n, T, steps):
    """Fused rollouts that read their actions from a caller's buffer [T, N] (uint8) instead of
    drawing them in the kernel: Pong and cart-pole, same shapes as the in-kernel-action lines."""
    from paper_2603_12145_amd import inputs
    dev = "cuda:0"
    out = {}
    for name, kind, dim, acts in (("pong", b.ENV_PONG, 8, inputs.pong_actions(T, n, 11)),
                                  ("cartpole", b.ENV_CARTPOLE, 4, inputs.cartpole_actions(T, n, 12))):
        h = b.env_create(kind, n, 2, None)
        obs = torch.empty((T, n, dim), dtype=torch.float32, device=dev)
        rew = torch.empty((T, n), dtype=torch.float32, device=dev)
        done = torch.empty((T, n), dtype=torch.uint8, device=dev)
        act = torch.from_numpy(acts).to(dev)
        b.env_reset(h, None)
        wall, ms = time_launches(lambda: b.env_rollout(h, T, act, obs, rew, done), steps, 20)
        b.env_destroy(h)
        mean_ms, _ = _mean_std(ms)
        out[name] = dict(ms_per_launch=mean_ms, env_steps_per_s=n * T * steps / wall)
        del obs, rew, done, act
    out["workload"] = "env_rollout with external actions, N=%d x T=%d" % (n, T)
    return out


def bench_body_sweep(b, torch, steps=3):
    """Both body kernels over N (not part of the default run): one table row per size."""
    rows = []
    for newton in (False, True):
        for n, T in ((8192, 400), (16384, 200), (32768, 200), (65536, 100), (131072, 100), (262144, 50),
                     (524288, 25), (1048576, 12)):
            r = bench_body(b, torch, n, T, 4, steps, newton=newton)
            rows.append(dict(model="newton" if newton else "penalty", n=n, T=T, ms_per_launch=r["ms_per_launch"],
                             env_steps_per_s=r["env_steps_per_s"], tflops=r["roofline"]["achieved"],
                             frac=r["roofline"]["frac"]))
    return rows


def bench_policy_loop(b, torch, n, policy_kind, steps, steps_per_graph):
    """Policy-in-the-loop rollout: a PyTorch policy reads obs and writes actions, env_step consumes
    them, all on one stream; timed as direct calls and as a replayed HIP graph (device step counter)."""
    dev = "cuda:0"
    torch.manual_seed(0)
    if policy_kind == "mlp":
        net = torch.nn.Sequential(torch.nn.Linear(8, 64), torch.nn.Tanh(), torch.nn.Linear(64, 64),
                                  torch.nn.Tanh(), torch.nn.Linear(64, 3)).to(dev)
        hidden = None
    else:   # GRU cell with ~2M parameters, bf16 weights
        net = torch.nn.GRUCell(8, 800).to(dev).to(torch.bfloat16)
        head = torch.nn.Linear(800, 3).to(dev).to(torch.bfloat16)
        hidden = torch.zeros((n, 800), dtype=torch.bfloat16, device=dev)
    params = sum(p.numel() for p in net.parameters())
    s = torch.cuda.Stream()
    out = {}
    with torch.no_grad(), torch.cuda.stream(s):
        for mode in ("direct", "graph"):
            cfg = {"step_counter": b.ENV_STEP_COUNTER_DEVICE} if mode == "graph" else None
            h = b.env_create(b.ENV_PONG, n, 1, cfg, stream=s)
            obs = torch.empty((n, 8), dtype=torch.float32, device=dev)
            rew = torch.empty(n, dtype=torch.float32, device=dev)
            done = torch.empty(n, dtype=torch.uint8, device=dev)
            act = torch.zeros(n, dtype=torch.uint8, device=dev)
            b.env_reset(h, obs)
            if hidden is not None:
                hidden.zero_()

            def one_step():
                if hidden is None:
                    logits = net(obs)
                else:
                    hidden.copy_(net(obs.to(torch.bfloat16), hidden))
                    logits = head(hidden)
                act.copy_(logits.argmax(dim=1).to(torch.uint8))
                b.env_step(h, act, obs, rew, done)

            preroll(one_step)
            s.synchronize()
            if mode == "direct":
                t0 = time.perf_counter()
                for _ in range(steps):
                    one_step()
                s.synchronize()
                wall = time.perf_counter() - t0
                done_steps = steps
            else:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=s):
                    for _ in range(steps_per_graph):
                        one_step()
                preroll(g.replay)
                s.synchronize()
                reps = max(1, steps // steps_per_graph)
                t0 = time.perf_counter()
                for _ in range(reps):
                    g.replay()
                s.synchronize()
                wall = time.perf_counter() - t0
                done_steps = reps * steps_per_graph
                del g
            out[mode] = dict(us_per_step=1e6 * wall / done_steps, env_steps_per_s=n * done_steps / wall)
            b.env_destroy(h)
    return dict(workload="Pong N=%d, %s policy (%d parameters) -> argmax -> env_step, one stream"
                         % (n, policy_kind, params),
                steps_per_graph=steps_per_graph, direct=out["direct"], graph=out["graph"],
                speedup_from_graph=out["direct"]["us_per_step"] / out["graph"]["us_per_step"])


def cpu_baseline(n, T, seed, budget_s=10.0):
    """The oracle as it stands on the host threads allotted to the box: whole passes over the headline
    workload (same N, T, seed), repeated until about budget_s seconds of wall time are spent, plus one
    single-thread pass over an eighth of the environments."""
    import numpy as np
    from oracle import oracle as orc
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")), 16)
    out = (np.zeros((T, n, 8), np.float32), np.zeros((T, n), np.float32), np.zeros((T, n), np.uint8))
    p = orc.Pong(n, seed)
    p.reset()
    p.rollout(10, nthreads=cores, out=tuple(a[:10] for a in out))       # warm-up, touches code paths
    p = orc.Pong(n, seed)
    p.reset()
    passes, spent = 0, 0.0
    while passes < 1 or (spent < budget_s and passes < 200):
        t0 = time.perf_counter()
        p.rollout(T, nthreads=cores, out=out)
        spent += time.perf_counter() - t0
        passes += 1
    n1 = max(1, n // 8)
    out1 = (np.zeros((T, n1, 8), np.float32), np.zeros((T, n1), np.float32),
            np.zeros((T, n1), np.uint8))
    q = orc.Pong(n1, seed)
    q.reset()
    t0 = time.perf_counter()
    q.rollout(T, nthreads=1, out=out1)
    single = time.perf_counter() - t0
    return dict(value=n * T * passes / spent, unit="env-steps/s", cores=cores, kind="oracle",
                sample="Pong N=%d x T=%d, %d consecutive passes of the headline workload (%.1f s), "
                       "%d threads; single thread on N=%d: %.3g env-steps/s"
                       % (n, T, passes, spent, cores, n1, n1 * T / single),
                single_thread_value=n1 * T / single)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--n", type=int, default=65536, help="environments (headline: 65536)")
    ap.add_argument("--T", type=int, default=1000)
    ap.add_argument("--skip-extra", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--only", default="", help="run only this extra workload (profiling aid)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU only (environments shard by index with no "
              "per-step traffic; no multi-GPU figure is produced). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_12145_amd import binding as b
    b.lib()  # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)

    if args.only:
        fn = {"pixels": lambda: bench_pixels(b, torch, 16384, 3, args.steps),
              "pixels_device_counter": lambda: bench_pixels(b, torch, 16384, 3, args.steps, device_counter=True),
              "pixels_external": lambda: [bench_pixels(b, torch, 16384, 3, args.steps, external=True),
                                          bench_pixels(b, torch, 16384, 3, args.steps, external=True, device_counter=True)],
              "pixels_delta": lambda: [bench_pixels(b, torch, 16384, 3, args.steps, delta=True),
                                       bench_pixels(b, torch, 16384, 3, args.steps, delta=True, layout="env_major"),
                                       bench_pixels(b, torch, 16384, 3, args.steps, layout="ordered"),
                                       bench_pixels(b, torch, 16384, 3, args.steps, delta=True, device_counter=True),
                                       bench_pixels(b, torch, 16384, 3, args.steps, layout="ordered",
                                                    device_counter=True)],
              "per_step": lambda: bench_pong_per_step(b, torch, 4096, 1, args.steps),
              "launch_costs": lambda: bench_launch_costs(b, torch),
              "cartpole_per_step": lambda: bench_pong_per_step(b, torch, 4096, 1, args.steps, kind="cartpole"),
              "sweep": lambda: {"n%d" % nn: bench_pong_rollout(b, torch, nn, 1000, 2, args.steps, 10)
                                for nn in (16384, 131072, 262144)},
              "sweep_large": lambda: {"n524288": bench_pong_rollout(b, torch, 524288, 250, 2, args.steps, 3)},
              "pixels_large": lambda: [bench_pixels(b, torch, 32768, 3, args.steps),
                                       bench_pixels(b, torch, 262144, 3, max(20, args.steps // 5))],
              "body": lambda: bench_body(b, torch, 8192, 1000, 4, args.steps),
              "body_f32": lambda: [bench_body(b, torch, 8192, 1000, 4, args.steps, f32=True),
                                   bench_body(b, torch, 262144, 100, 4, args.steps, f32=True)],
              "body_sweep": lambda: bench_body_sweep(b, torch, args.steps),
              "body_newton": lambda: [bench_body(b, torch, 8192, 1000, 4, args.steps, newton=True),
                                      bench_body(b, torch, 262144, 100, 4, args.steps, newton=True)],
              "policy": lambda: [bench_policy_loop(b, torch, 4096, "mlp", 2000, 50),
                                 bench_policy_loop(b, torch, 65536, "mlp", 2000, 50),
                                 bench_policy_loop(b, torch, 4096, "gru", 1000, 50)],
              "cartpole": lambda: bench_cartpole(b, torch, 65536, 1000, 2, args.steps),
              "external_actions": lambda: bench_external_actions(b, torch, 65536, 1000, args.steps),
              "store_floor": lambda: bench_store_floor(b, torch, 65536, 1000, args.steps),
              "fill": lambda: bench_fill(b, torch, 1 << 30, args.steps),
              "copy": lambda: bench_copy(b, torch, 1 << 30, args.steps)}[args.only]
        print(json.dumps(fn()))
        return

    n, T, seed = args.n, args.T, 2
    # Yardsticks first: what the device does for a plain fill and for the rollout's own stores with
    # nothing behind them.  They also leave the device busy right up to the headline's own pre-roll.
    yard = {}
    if not args.skip_extra:
        yard["fill_yardstick"] = bench_fill(b, torch, 1 << 30)
        yard["trajectory_stores_only"] = bench_store_floor(b, torch, n, T)
    r = bench_pong_rollout(b, torch, n, T, seed, args.steps, args.warmup, repeats=REPEATS)
    value = r["env_steps"] / r["wall"]
    achieved = PONG_BYTES_PER_ENV_STEP * n * T / (r["mean_ms"] * 1e-3) / 1e9
    traffic = _traffic("pong_rollout_n%d_t%d" % (n, T))
    run_values = [x["env_steps_per_s"] for x in r["runs"]]
    run_mean, run_std = _mean_std(run_values)
    line = {
        "metric": "env-steps/sec on 1 MI355X (Pong N=65536 fused rollout) + % of HBM roofline",
        "value": value, "unit": "env-steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * r["wall"] / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "Pong fused env_rollout, N=%d envs x T=%d steps per launch, seed 2, "
                               "in-kernel Philox actions, obs[T,N,8] f32 + reward[T,N] f32 + done[T,N] u8"
                               % (n, T),
                   "n_envs": n, "T": T, "env_steps_per_step": n * T},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "pong_rollout_kernel", "launch_ms_mean": r["mean_ms"],
                     "launch_ms_std": r["std_ms"], "launch_ms_cv": r["std_ms"] / r["mean_ms"],
                     "algorithmic_bytes_per_launch": PONG_BYTES_PER_ENV_STEP * n * T,
                     # the library's own one-time measurement for this batch size on this device: the write rate
                     # its paced loop is held to (GB/s), -1 = the plain loop won, 0 = nothing measured
                     "pace_choice_gbs": r["pace_choice_gbs"]},
        # the paper's throughput protocol (Table 2 caption): mean +- std over five runs, CV below 3 %.
        # `value` is the first of them; the other four follow it back to back.
        "runs": {"n": len(run_values), "steps_each": args.steps, "env_steps_per_s": run_values,
                 "mean": run_mean, "std": run_std, "cv": run_std / run_mean,
                 "launch_ms_mean": [x["launch_ms_mean"] for x in r["runs"]]},
        "before_timed_region": ("fill and trajectory-store yardsticks (extra), then " if yard else "")
                               + "%.0f ms of the same env_rollout launches (device clocks settle 30-35 ms after "
                                 "any idle period), then the %d warm-up launches of the flag, no idle gap"
                                 % (1e3 * PREROLL_S, args.warmup),
        "device": {"name": props.name, "cus": props.multi_processor_count,
                   "hbm_gib": round(props.total_memory / 2 ** 30, 1)},
    }
    if not args.skip_cpu:
        line["cpu_baseline"] = cpu_baseline(n, T, seed)
    if not args.skip_extra:
        extra = dict(yard)
        floor = extra["trajectory_stores_only"]
        floor["rollout_vs_unpaced_stores"] = floor["ms_per_launch"] / r["mean_ms"]
        floor["rollout_vs_best_paced_stores"] = floor["best_paced_ms"] / r["mean_ms"]
        extra["config1_per_step"] = bench_pong_per_step(b, torch, 4096, 1, 10000)
        extra["launch_costs"] = bench_launch_costs(b, torch)
        extra["cartpole_per_step_n4096"] = bench_pong_per_step(b, torch, 4096, 1, 10000, kind="cartpole")
        extra["config3_pixels"] = bench_pixels(b, torch, 16384, 3, 500)
        extra["config3_pixels_external_actions"] = bench_pixels(b, torch, 16384, 3, 500, external=True)
        extra["config3_pixels_external_actions_device_counter"] = bench_pixels(b, torch, 16384, 3, 500, external=True,
                                                                               device_counter=True)
        for nn, st in ((32768, 300), (262144, 60)):      # the same step on larger batches (context, not the target)
            extra["pixels_n%d" % nn] = bench_pixels(b, torch, nn, 3, st)
        extra["config3_pixels_env_major"] = bench_pixels(b, torch, 16384, 3, 500, layout="env_major")
        extra["config3_pixels_device_counter"] = bench_pixels(b, torch, 16384, 3, 500, device_counter=True)
        extra["config3_pixels_delta_updates"] = bench_pixels(b, torch, 16384, 3, 500, delta=True)
        extra["config3_pixels_ordered_stack"] = bench_pixels(b, torch, 16384, 3, 500, layout="ordered")
        for nn in (16384, 262144):
            rr = bench_pong_rollout(b, torch, nn, T, seed, max(3, args.steps // 6), 3)
            gbs = PONG_BYTES_PER_ENV_STEP * nn * T / (rr["mean_ms"] * 1e-3) / 1e9
            extra["config2_n%d" % nn] = dict(env_steps_per_s=rr["env_steps"] / rr["wall"], pace_choice_gbs=rr["pace_choice_gbs"],
                                             ms_per_launch=rr["mean_ms"], ms_min=rr["min_ms"],
                                             ms_max=rr["max_ms"], hbm_gbs=gbs, frac=gbs / HBM_PEAK_GBS,
                                             traffic=_traffic("pong_rollout_n%d_t%d" % (nn, T)))
        extra["config4_body"] = bench_body(b, torch, 8192, 1000, 4, 2)
        extra["config4_body_n262144_t100"] = bench_body(b, torch, 262144, 100, 4, 2)
        extra["body_newton_n8192_t1000"] = bench_body(b, torch, 8192, 1000, 4, 2, newton=True)
        extra["config4_body_f32"] = bench_body(b, torch, 8192, 1000, 4, 2, f32=True)
        extra["config4_body_f32_n262144_t100"] = bench_body(b, torch, 262144, 100, 4, 2, f32=True)
        extra["cartpole_n65536_t1000"] = bench_cartpole(b, torch, 65536, 1000, 2, 5)
        extra["external_actions_n65536_t1000"] = bench_external_actions(b, torch, 65536, 1000, 5)
        extra["policy_in_loop_mlp_n4096"] = bench_policy_loop(b, torch, 4096, "mlp", 2000, 50)
        extra["policy_in_loop_gru2m_n4096"] = bench_policy_loop(b, torch, 4096, "gru", 1000, 50)
        line["extra"] = extra
    print(json.dumps(line))


if __name__ == "__main__":
    main()
