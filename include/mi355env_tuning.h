/* mi355env — measurement knobs and yardstick kernels of libmi355env.so.
 *
 * Not part of the environment boundary (include/mi355env.h): these exist so that the benchmark and
 * the tests can time a launch shape against another, force a code path that the library would
 * otherwise choose from N, and measure what the device does for a plain fill, copy or empty
 * launch.  All mi355env_tune_* settings are PROCESS-WIDE: they change which kernel every handle of
 * the process launches from its next call on, they are plain globals without locks, and they must
 * not be called while another thread is inside any call on any handle.  They never change a
 * result, only the launch shape.  A program that is not measuring has no reason to call them; a
 * test that does restores the defaults when it ends (0 / the documented default of each knob).
 * Return ENV_OK (0) or ENV_E_ARG (-1) unless stated.
 */
#ifndef MI355ENV_TUNING_H
#define MI355ENV_TUNING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Pong / cart-pole rollout: threads per workgroup (64, 128, 256; 0 = default 256) and whether
 * workgroups are remapped so that each XCD owns a contiguous eighth of the environments (default 1). */
int mi355env_tune_rollout(int threads_per_block, int xcd_remap);

/* Pong rollout: steps per chunk of the main loop (the Philox blocks of a chunk are drawn while the
 * previous chunk's steps run): 2, 4 or 8; 0 = chosen from N (default: 8 up to N = 53248, 2 above).
 * Only the full-wavefront, in-kernel-action, raw-observation loop with direct stores that is not
 * paced (below) has the three variants; the paced loop uses 2, the loops with external actions 8, every other loop 4. */
int mi355env_tune_rollout_chunk(int steps);

/* Pong rollout, small batches: 0 = default (for N <= 16384 and T >= 32, in-kernel actions and raw
 * observations, every 64 environments get a second wavefront that draws their Philox blocks and
 * hands them over through LDS), 1 = never, 2 = for any N and T.  Results are identical. */
int mi355env_tune_rollout_split(int mode);

/* Pong env_step (and env_rollout with T = 1): 1 = default, a kernel that holds the step and nothing
 * else, launched without kernel arguments (its launch descriptor kept in device memory) from the
 * second call in a row that passes the same buffers, for handles with the host step counter and
 * N <= 16384, at most four handles per device at a time; 2 = that kernel, always launched with
 * arguments; 0 = the rollout kernel's T = 1 path.  Results are identical. */
int mi355env_tune_step_kernel(int on);
/* How many env_step calls of this process have been launched without kernel arguments so far
 * (for tests that have to know which of the two launches they exercised). */
unsigned long long mi355env_resident_step_launches(void);

/* Cart-pole rollout, batches of at most one wavefront per SIMD: 0 = default (for N <= 65536 and
 * T >= 32 with in-kernel actions, every 64 environments get a second wavefront that draws their
 * Philox blocks and hands them over through LDS), 1 = never, 2 = for any N and T.  Results are
 * identical. */
int mi355env_tune_cartpole_split(int mode);

/* Pacing of the same loop.  gb_per_s > 0: every full wavefront runs the paced loop (two steps per
 * chunk, episode statistics brought up to date once per chunk instead of in every step) and starts
 * a chunk no sooner than 2 * N * 37 B / gb_per_s after the previous one, by the constant 100 MHz
 * clock, whatever N; 0 = chosen by the library (default), -1 = never paced.  The library's choice
 * for N = 61440 ... 262144: the first env_rollout of at least 256 steps for a batch size on a
 * device measures, on scratch state, the plain loop against the paced loop at a few rates around
 * a table's (6600 GB/s up to N = 65536, 5800 up to 131072, 5600 up to 262144) and keeps the fastest
 * for the rest of the process, the paced loop only if it wins by 1 % (about 60 ms, once; that call
 * synchronises the stream); shorter rollouts and calls under stream capture use the table; other
 * batch sizes are never paced; with external actions only N = 98305 ... 262144 is.
 * Results are identical. */
int mi355env_tune_rollout_pace(int gb_per_s);

/* 1 (default) = measure as just described, 0 = always take the table's rate. */
int mi355env_tune_measure_pace(int on);
/* What the measurement found for n environments on the current device: the rate in GB/s, -1 = not
 * paced, 0 = nothing measured yet for that batch size. */
int mi355env_pace_choice(int64_t n);

/* Pong rollout observation stores: 0 = direct (two 16-byte stores per lane), 1 = through LDS, one
 * 4 KiB page per store instruction, wherever a 256-thread workgroup is full, 2 = chosen from N
 * (default: paged above N = 262144, where the loop is not paced). */
int mi355env_tune_paged_stores(int mode);

/* Wave-tile pixel renderer (env-major ring, env_rollout frames): environments per wavefront
 * (4, 8, 16, 32 or 64; 0 = default: 8 up to N = 12288, 16 above) and streaming (non-temporal)
 * stores (0 / 1). */
int mi355env_tune_pixels(int envs_per_wave, int streaming);

/* Pixel env_rollout (frame trajectory): 0 = one launch whose wavefronts each own a few environments
 * for all T steps, 1 = a dynamics pass stages a chunk of steps and the page renderer writes the
 * chunk's frames together (wherever the staging area allows: N <= 262144 and the step counter on the
 * host), 2 = chosen from N (default: chunked except for N = 16384 ... 24575). */
int mi355env_tune_frame_trajectory(int mode);

/* Slot-major pixel env_step: 0 = wave-tile renderer, 1 = page renderer as separate launches,
 * 2 = page renderer fused with the next step's dynamics in one launch (default). */
int mi355env_tune_plane_path(int mode);

/* Inspection, for a handle of ENV_PONG_PIXELS created with pixel_update = ENV_PIXELS_DELTA: how many
 * env_step calls since env_create rewrote only the changed pixels of their ring slot and how many
 * fell back to a full write of it.  `e` is the env_t* of include/mi355env.h; host pointers. */
int mi355env_pixel_update_counts(const void *e, int64_t *delta_steps, int64_t *full_steps);

/* Yardsticks, launched on hip_stream: dst[i] = value; dst = src; a kernel that does nothing.
 * Pointers are device memory, 16-byte aligned, bytes a multiple of 16 (else -1); -3 if the launch
 * fails. */
int mi355env_bench_fill(void *dst_dev, size_t bytes, uint32_t value, void *hip_stream);
/* The same fill as one 4 KiB page per 256-thread workgroup, one store per thread, no loop. */
int mi355env_bench_fill_pages(void *dst_dev, size_t bytes, uint32_t value, void *hip_stream);
int mi355env_bench_copy(void *dst_dev, const void *src_dev, size_t bytes, void *hip_stream);
int mi355env_bench_empty(void *hip_stream);
/* A loop of `launches` launches enqueued from C++ with nothing in between, to tell the host's share
 * of a launch from the device's.  kind 0: an empty kernel; 1: workgroups of 256 threads store
 * bytes / 4 words, descriptor passed as kernel arguments; 2: the same store, descriptor read from
 * device memory by a kernel without a kernel-argument segment.  dst_dev: device memory of `bytes`
 * bytes (a multiple of 1024, at most 1 MiB; ignored for kind 0).  *host_us_out: host time per
 * launch until the last one is enqueued; *total_us_out: per launch until the stream has drained.
 * Synchronises the stream before and after.  Returns 0, -1 (arguments) or -3 (HIP error). */
int mi355env_bench_launch_loop(int kind, int launches, void *dst_dev, size_t bytes, void *hip_stream,
                               double *host_us_out, double *total_us_out);
/* The trajectory stores of the fused Pong rollout without any computation: constant values into
 * obs_dev float32[T][n][8] (16-byte aligned), reward_dev float32[T][n], done_dev uint8[T][n], in the
 * rollout's launch shape.  Its duration is the floor the memory system sets for that layout. */
int mi355env_bench_trajectory_stores(void *obs_dev, void *reward_dev, void *done_dev, int64_t n, int32_t T,
                                     void *hip_stream);
/* The same with every wavefront put to sleep for sleep x 64 cycles after each step (sleep = 0, or
 * 8..15; else -1).  Unpaced, wavefronts drift apart over the rows of the trajectory and the memory
 * system does worse than when they all write the same row at the rate it drains at: the best
 * paced time, not the unpaced one, is what the memory system can do for this layout. */
int mi355env_bench_trajectory_stores_paced(void *obs_dev, void *reward_dev, void *done_dev, int64_t n, int32_t T,
                                           int32_t sleep, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MI355ENV_TUNING_H */
