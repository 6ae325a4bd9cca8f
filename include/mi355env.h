/* mi355env — vectorised environment step / reset / rollout on one MI355X (gfx950).
 *
 * C ABI of the hot path that generated "performance environments" exist to accelerate: stepping N
 * independent environments in lock-step, resetting them, and running a T-step rollout fused into
 * one kernel launch (paper: section 1 — simulation is 50-90 % of RL wall-clock; App. B.1 items 3-5
 * — batch a single-instance step, one launch per batch step, fuse the rollout loop into one kernel;
 * App. B.1 items 6-7 — small dtypes, pre-allocated output buffers; App. B.2 item 8 — one call for
 * all environments, zero-copy buffers).
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory owned by the caller (e.g. a PyTorch tensor's
 *    data_ptr()), row-major, exactly the documented shape, alive until the stream has run the call.
 *    Every pointer named *_host / host_* is HOST memory owned by the caller.
 *  - The library owns only its SoA state, the episode-statistics block and, for ENV_PONG_PIXELS,
 *    its staging buffers (a second state buffer, about 100 B/env of staged step results and cell
 *    blocks, 3 MB for frame trajectories; with delta updates 60 B/env more), all allocated by
 *    env_create and freed by env_destroy.  step / reset / rollout never allocate.
 *  - step / reset / rollout enqueue work on the handle's stream and return without waiting;
 *    stats / get_state / set_state synchronise that stream.
 *  - All functions return ENV_OK (0) or a negative error code; on error no output buffer is
 *    touched.  No C++ exception crosses this boundary.
 *  - One handle must not be used from two threads at once.  A handle belongs to the device that
 *    was current in env_create; calls made with another device current return ENV_E_STATE.
 *  - Device pointers are checked for residency and size (the range must lie inside one device
 *    allocation) before anything is launched.  A handle remembers the last eight (pointer, size)
 *    pairs that passed and does not ask the driver about them again: a buffer that is freed and
 *    replaced by a smaller one at the same address is the caller's to keep track of.
 *  - Random draws come from Philox4x32-10 with key = (seed lo, seed hi) and
 *    counter = (env index, step lo, step hi, stream); `step` counts env steps since env_create and
 *    is never rewound, so results do not depend on N nor on how a rollout is cut into calls.
 *  - Auto-reset: done[t,i] = 1 marks the transition that ended an episode; the observation stored
 *    at that index is already the first observation of the next episode, the reward is the final
 *    transition's.
 */
#ifndef MI355ENV_H
#define MI355ENV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mi355env env_t; /* opaque handle */

enum {
  ENV_PONG = 0,        /* Pong, obs = float32[8]: ball x, y, vx, vy, agent y, opponent y, scores  */
  ENV_PONG_PIXELS = 1, /* same dynamics, obs = ring of four rendered 84x84 uint8 frames per env   */
  ENV_BODY = 2,        /* planar 7-link articulated body, obs = float32[17], action float32[6]    */
  ENV_CARTPOLE = 3     /* cart-pole, obs = float32[4]: x, xdot, theta, thetadot; action uint8     */
};

enum {
  ENV_OK = 0,
  ENV_E_ARG = -1,      /* bad argument: NULL, non-positive size, misaligned or non-device pointer */
  ENV_E_ALLOC = -2,    /* device allocation failed                                                */
  ENV_E_HIP = -3,      /* a HIP runtime call or kernel launch failed                              */
  ENV_E_STATE = -4,    /* call order: step/rollout before the first env_reset; capture on a handle
                          with a host step counter; current device is not the handle's            */
  ENV_E_UNSUPPORTED = -5, /* operation not available for this environment kind                    */
  ENV_E_TOO_LARGE = -6   /* size beyond the fixed maximum of env_step_pixels_noalloc              */
};
/* There is no status code for a state that left the finite range: step / rollout return before the
 * kernel has run, so a device-side condition cannot be their return value.  Such an environment is
 * re-initialised inside the kernel (done = 1, reward = 0) and counted in env_stats_t.nonfinite. */

/* Optional configuration (NULL = defaults).  struct_size = sizeof(env_config_t) as compiled by the
 * caller; fields beyond struct_size keep their defaults.  A zero/negative value in a field means
 * "default" unless stated. */
typedef struct env_config_t {
  uint32_t struct_size;
  int32_t max_score;          /* Pong: points that end an episode (default 21)                    */
  int32_t max_episode_steps;  /* truncation length: body (default 1000), cart-pole (default 500)  */
  float armature;             /* body: rotor inertia added to the 6 joint diagonals; <0 = default */
  float joint_damping;        /* body: viscous joint damping; <0 = default                        */
  float friction_mu;          /* body: Coulomb friction coefficient; <0 = default                 */
  int32_t pixel_layout;       /* pixels: ENV_PIXELS_* below; 0 = default (slot-major)             */
  int32_t step_counter;       /* ENV_STEP_COUNTER_* below; 0 = default (host)                     */
  int32_t obs_scaling;        /* ENV_OBS_* below; 0 = default (raw)                               */
  int32_t contact_solver;     /* body: ENV_CONTACT_* below; 0 = default (penalty)                 */
  int32_t pixel_update;       /* pixels: ENV_PIXELS_FULL / ENV_PIXELS_DELTA below; 0 = default    */
  int32_t body_arithmetic;    /* body: ENV_BODY_F64 / ENV_BODY_F32 below; 0 = default (float64)   */
} env_config_t;

/* Arithmetic inside a step of ENV_BODY (other kinds: ENV_E_UNSUPPORTED for F32).  State, actions,
 * observations and rewards are float32 in memory either way.
 *   f64  a step is computed in float64 from the float32 state and rounded back at its end
 *        (default).  This is what meets the single-step bar of 1e-5 per component against a
 *        float64 reference: the 9x9 system is conditioned like 10^2, and float32 arithmetic alone
 *        leaves an error of that size.
 *   f32  the same formulas in float32 (the precision the paper's case study states, App. A.1):
 *        fewer registers and a full-rate reciprocal square root, 1.3x (N = 8192) to 1.7x (N >= 262144)
 *        the speed.  Single steps then agree with a float64 reference to 1e-6 at the median
 *        environment and beyond 1e-5 on 0.3-6 % of them (worst seen 2e-4, as for any float32
 *        evaluation of these formulas); return statistics of long rollouts agree within 1 %.
 *        Every contact / joint-limit decision is taken in float32. */
enum { ENV_BODY_F64 = 1, ENV_BODY_F32 = 2 };

/* Ground contact and joint limits of ENV_BODY (other kinds: ENV_E_UNSUPPORTED for NEWTON).
 *   penalty  explicit spring-damper normal force (k = 1e4, c = 100), friction c*vx clipped to
 *            +-mu*fn, joint limits by an M-orthogonal velocity projection (the paper's first solver
 *            revision for this case study, App. A.1);
 *   newton   the substep's acceleration minimises 1/2 (a-a0)^T M (a-a0) + sum_i D_i/2 min(0, J_i a -
 *            aref_i)^2 over soft one-sided rows: the two friction-pyramid edges J_z +- mu J_x of
 *            every contact point below the ground (aref = -b J v - k z - dJ/dt qdot, D = 1/0.02) and
 *            one row per joint at a limit (aref = -b J v, D = 1/0.5), k = 1/tc^2, b = 2/tc,
 *            tc = 0.02 s; solved by Newton's method on the active set with Cholesky
 *            factorisations, at most 8 passes (the paper's final revision: acceleration-space QP). */
enum { ENV_CONTACT_PENALTY = 1, ENV_CONTACT_NEWTON = 2 };

/* ENV_PONG only (other kinds: ENV_E_UNSUPPORTED).  ENV_OBS_NORMALIZED scales every observation
 * component inside the step kernel (paper App. B.1 item 8) by one float32 multiplication with the
 * reciprocal of its range: ball x * (1/158), ball y * (1/208), vx * (1/3), vy * (1/2),
 * both paddle y * (1/194), both scores * (1/max_score) - positions and scores in [0,1],
 * velocities in [-1,1].  Dynamics, rewards, done flags and the state blob are unchanged. */
enum { ENV_OBS_RAW = 1, ENV_OBS_NORMALIZED = 2 };

/* Where the handle's step counter (which keys every random draw) lives.
 *   host    the library passes it to each launch as a kernel argument (default, cheapest);
 *   device  each launch reads it from device memory and advances it there, so an env_step /
 *           env_rollout call recorded into a HIP graph (stream capture) can be replayed and every
 *           replay continues the sequence exactly as the same number of direct calls would
 *           (the policy-in-the-loop rollout: policy kernels and env_step in one captured graph).
 *           Before capturing, make one direct call with the same buffers (the pointer checks query
 *           the driver the first time they see a buffer; later calls with the same buffers do
 *           not).  Launches of one handle must not overlap.  env_step_count, env_get_state and
 *           env_reset read the device counter; the first two synchronise the stream.
 *           A handle with the host counter refuses env_step / env_rollout while its stream is
 *           capturing (ENV_E_STATE): replays would repeat the captured step index.
 *           ENV_PONG_PIXELS: a step is then two launches (the default path computes the next step
 *           under the render of this one in a single launch and alternates library buffers from
 *           the host, which a replayed graph cannot do): with in-kernel actions a one-workgroup
 *           launch that moves the counter, then the same fused launch with buffers and ring slot
 *           derived from the counter; with external actions a dynamics launch, then the renderer.
 *           Results are the same bit for bit; a step takes about a quarter longer (22.5 against
 *           18 us at N = 16384). */
enum { ENV_STEP_COUNTER_HOST = 1, ENV_STEP_COUNTER_DEVICE = 2 };

/* Layout of the four frames of ENV_PONG_PIXELS in obs_dev of env_reset / env_step.  The first two
 * are a ring: the frame after the step with index s goes to slot s mod 4, the other slots keep what
 * they hold, and the consumer reads the slots in rotated order.
 *   slot-major  uint8[4][N][84][84]  frame of slot k of environment i at ((k*N + i) * 7056);
 *               one step writes one contiguous plane of N frames (the dense stream HBM likes);
 *   env-major   uint8[N][4][84][84]  frame at ((i*4 + k) * 7056): each environment's four frames
 *               are adjacent (NCHW order), at the price of a 25 %-dense write stream per step;
 *   ordered     uint8[N][4][84][84]  a stack, not a ring: channel 3 is the newest frame, channel k
 *               the one 3-k steps older; every env_step moves the channels down by one and puts
 *               the new frame on top; env_reset fills all four with the initial frame; env_rollout
 *               (a frame trajectory) and env_set_state leave it alone.  A consumer can read it as
 *               it is.  Always maintained by delta updates (see ENV_PIXELS_DELTA below: the same
 *               rules about the buffer being shared state apply): each channel changes by one
 *               step's worth of pixels.  When the library cannot vouch for the contents it moves
 *               the channels physically instead (four steps, as above). */
enum { ENV_PIXELS_SLOT_MAJOR = 1, ENV_PIXELS_ENV_MAJOR = 2, ENV_PIXELS_ORDERED = 3 };

/* How env_step brings a ring slot of ENV_PONG_PIXELS up to date (other kinds: ENV_E_UNSUPPORTED for
 * DELTA).  The ring's contents after a step are the same either way.
 *   full   every step writes all 7056 bytes of every environment's newest frame (default): the
 *          slot's previous contents do not matter;
 *   delta  the slot still holds the frame written four steps earlier, which differs from the new one
 *          in a few dozen pixels: the step clears the pixels that went dark and sets the ones that
 *          lit up, and touches nothing else.  This makes the ring shared state: pass the same ring
 *          to every env_reset / env_step and do not write to it.  The library keeps the rectangles
 *          of the last five frames (60 B/env) and a record of which buffer they describe and from
 *          which step on; whenever it cannot vouch for the buffer (no env_reset with it yet,
 *          env_set_state, another buffer, steps taken through env_rollout in between) the next four
 *          steps write whole frames, after which delta updates resume.  Works with either step
 *          counter: with ENV_STEP_COUNTER_DEVICE the record lives in device memory and every
 *          launch, also a replayed one, decides for itself. */
enum { ENV_PIXELS_FULL = 1, ENV_PIXELS_DELTA = 2 };

/* Statistics of the episodes that ended since the counters were last cleared (the per-batch
 * episode bookkeeping a training loop logs; reduced on the device, one atomic set per wavefront). */
typedef struct env_stats_t {
  int64_t episodes;
  int64_t length_sum;
  double return_sum;
  double return_min; /* +inf when episodes == 0 */
  double return_max; /* -inf when episodes == 0 */
  int64_t nonfinite; /* body: environments re-initialised because their state left the finite range */
} env_stats_t;

/* Paper section 3.1 (problem statement): the unit being built is an environment whose step / reset
 * reproduce a reference's observations, rewards and termination signals for any seed and action
 * sequence; App. B.1 item 3 and App. B.2 item 8: one object, one call, for the whole batch.
 * Create N environments of `kind`.  seed keys every random draw.  hip_stream is a hipStream_t
 * (NULL = the null stream) on the current device; the handle keeps using it.  Allocates
 * state (Pong: 40 B/env, body: 80 B/env, cart-pole: 24 B/env) on the current device.  *out is set only on success. */
int env_create(env_t **out, int kind, int64_t n_envs, uint64_t seed, const env_config_t *cfg,
               void *hip_stream);

/* Counterpart of env_create (App. B.1 item 7 / App. B.2 item 2: buffers live as long as the
 * environment, nothing is allocated per step).
 * Free the handle and its device memory (synchronises the stream first).  NULL is ignored. */
void env_destroy(env_t *e);

/* Paper section 3.1 and App. B.3 (the interface that optimisation must not change: step, reset,
 * observation / reward shapes); App. B.1 item 4: reset, like step, is one launch for the batch.
 * Start a new episode in every environment, drawing the initial state from the reset streams at
 * the current step counter.  obs_dev (may be NULL): Pong float32[N,8]; body float32[N,17];
 * pixels: the ring (4*N*7056 bytes, layout per cfg.pixel_layout) — all four slots of every
 * environment receive the initial frame.  16-byte aligned (body: 4-byte). */
int env_reset(env_t *e, void *obs_dev);

/* Paper section 3.1 (per-step outputs: observation, reward, termination); App. B.1 items 3-4 (a
 * single-instance step batched over N, one launch per batch step); items 6-7 (uint8 flags and
 * actions, float32 only where arithmetic needs it, caller-provided output buffers).
 * Advance every environment by one step (one kernel launch).
 * actions_dev: Pong uint8[N] in {0 stay, 1 up, 2 down} (other values = stay); body float32[N,6],
 * clipped to [-1,1]; cart-pole uint8[N], 1 = push right, anything else = push left;
 * NULL = draw the actions from this step's Philox block inside the kernel.
 * obs_dev: Pong float32[N,8]; body float32[N,17]; cart-pole float32[N,4]; pixels: the ring — the frame after the step
 * with index s (s = steps taken before this call) is written to slot s mod 4, the other three
 * slots are left as they are.  reward_dev float32[N], done_dev uint8[N].
 * obs_dev must be 16-byte aligned (body: 4-byte), reward_dev 4-byte aligned.  None may be NULL.
 * Pong and cart-pole handles with the host step counter and N <= 16384: a call that passes the
 * buffers of the call before it is launched without kernel arguments, from a record of the call
 * that the library keeps in device memory (four such handles per device; others launch with
 * arguments); same results, and nothing for the caller to do or to avoid. */
int env_step(env_t *e, const void *actions_dev, void *obs_dev, float *reward_dev, uint8_t *done_dev);

/* Paper App. B.1 item 5 (the rollout loop fused into one kernel, no per-step dispatch) and App. A.1
 * "Puffer Pong" (a whole rollout as a single GPU kernel with no host-device transfer).
 * T steps fused into one kernel launch; state stays in registers between steps.
 * actions_dev: [T,N] (Pong uint8) / [T,N,6] (body float32) or NULL (in-kernel Philox draws).
 * obs_dev: float32[T,N,obs_dim] (Pong, body); pixels: uint8[T,N,84,84], frame t of the rollout.
 * reward_dev float32[T,N]; done_dev uint8[T,N].  Alignment as for env_step.  Equivalent, bit for
 * bit, to T calls of env_step (Pong; the body's obs/reward agree exactly as well, same kernels). */
int env_rollout(env_t *e, int32_t T, const void *actions_dev, void *obs_dev, float *reward_dev,
                uint8_t *done_dev);

/* Paper section 3.2, level 3 (episodes compared over matched seeds) needs episode returns and
 * lengths per batch; this is their device-side reduction read back.
 * Copy the episode statistics to *host_out; clear the device counters if reset_counters != 0.
 * Synchronises the stream. */
int env_stats(env_t *e, env_stats_t *host_out, int reset_counters);

/* Size in bytes of the state blob of get/set_state: 8 + 4 * fields * N, where the blob is
 * { uint64 step_counter; field_0[N]; field_1[N]; ... }, every field 4 bytes wide.
 * Pong / pixels (10 fields): ball x, y, vx, vy, agent y, opponent y (float32), agent score,
 * opponent score, episode return so far, episode length so far (int32).
 * Body (20 fields): q[9], v[9], episode return so far (float32), episode length so far (int32).
 * Cart-pole (6 fields): x, xdot, theta, thetadot, return so far (float32), length so far (int32). */
size_t env_state_bytes(const env_t *e);

/* Paper App. C (module translation prompt: all of a simulator's registers in one plain structure,
 * for saving and loading state) and section 3.2, level 3 (rollouts replayed from matched states).
 * Copy the state blob to / from host memory (bytes must equal env_state_bytes); both synchronise
 * the stream.  set_state also marks the handle as reset.  Rendered frames are not part of the
 * state.  Values are taken as they are, except that a negative zero in a float32 field of Pong is
 * stored as +0 (the game never produces one; the step's sign tests treat the two alike this way). */
int env_get_state(env_t *e, void *host_buf, size_t bytes);
int env_set_state(env_t *e, const void *host_buf, size_t bytes);

/* Shapes of the interface (App. B.3: fixed observation / reward shapes).
 * Floats (or bytes, for pixels: 4*84*84) per environment in obs_dev of env_step; <0 on bad kind. */
int env_obs_dim(int kind);
/* Elements per environment in actions_dev (Pong 1 x uint8, body 6 x float32). */
int env_action_dim(int kind);
int64_t env_num_envs(const env_t *e);
/* Env steps taken since env_create.  With the device step counter this synchronises the stream
 * (returns UINT64_MAX if that fails). */
uint64_t env_step_count(const env_t *e);

/* For the policy-in-the-loop rollout (paper section 4.1, throughput table, row "GRU Rollout (2M)":
 * policy and environment step in one device-side loop): env_step recorded on the stream a graph
 * capture runs on.
 * Enqueue all later work of the handle on another stream of the same device (e.g. the stream a
 * graph capture runs on).  The caller orders the two streams; nothing is synchronised here. */
int env_set_stream(env_t *e, void *hip_stream);

/* For callers that cannot allocate device memory: code running under a HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  One env_step of Pong with pixel observations on
 * the slot-major ring, as env_step does it for an ENV_PONG_PIXELS handle, but without a handle: the
 * caller owns the state, and what a handle would have allocated -- the partial episode statistics
 * and the 12 bytes per environment that the dynamics pass stages for the renderer -- lives in a
 * fixed array inside the library (800 KiB per device, held until the process ends), which limits
 * the batch to ENV_NOALLOC_MAX_ENVS environments (more: ENV_E_TOO_LARGE).  The call allocates and
 * frees nothing, takes no handle and synchronises nothing; it enqueues four small launches on
 * hip_stream (NULL = the null stream) of the current device.
 *   state_dev   in/out, uint32[10][n]: the fields of the Pong state blob (env_state_bytes above)
 *               without the leading step counter, e.g. copied from env_get_state
 *   step        index of this step = env steps taken before it; keys the random draws (with seed)
 *               and selects the ring slot, step mod 4
 *   actions_dev uint8[n] or NULL (in-kernel draws), as for env_step
 *   ring_dev    uint8[4][n][84][84], 16-byte aligned; only slot step mod 4 is written
 *   reward_dev  float32[n];  done_dev uint8[n]
 *   stats_dev   optional (NULL = none), 8-byte aligned DEVICE memory: receives the statistics of the
 *               episodes that ended in THIS step (nonfinite = 0)
 * Results are those of env_step on a handle in the same state, bit for bit.  All calls on one
 * device share the one array: calls that overlap in time on one device (two streams, two threads)
 * race on it; calls on one stream do not.  Device pointers are checked like env_step's and the
 * ranges that passed are remembered, so make one direct call with the same buffers before
 * recording a call in a graph. */
#define ENV_NOALLOC_MAX_ENVS 65536
int env_step_pixels_noalloc(int64_t n_envs, uint64_t seed, uint64_t step, int32_t max_score,
                            void *state_dev, const uint8_t *actions_dev, uint8_t *ring_dev,
                            float *reward_dev, uint8_t *done_dev, env_stats_t *stats_dev,
                            void *hip_stream);

/* Static string for a status code. */
const char *env_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* MI355ENV_H */
