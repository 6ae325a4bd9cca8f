// TEST INFRASTRUCTURE — CPU oracle. Not part of the product path; shares no code with the HIP library.
//
// Pong, one environment at a time, float32, in the fixed operation order below.  The paper names
// the workload (Table 1 "Puffer Pong"; App. A.1 "Puffer Pong": the whole rollout fused into one
// kernel; App. B.1 item 2: branchless collision logic) but prints no dynamics; the dynamics are the
// benchmark configuration's: field 160x210, paddles 4x16 at x=140 (agent) and x=16 (opponent),
// agent speed 4, opponent tracks ball y at speed <= 3, ball 2x2 served from the centre at +-3 x and
// uniform [-2,2) y, wall reflection, paddle hit vy = 0.2 * (ball centre - paddle centre), reward
// +-1 per point, episode ends at max_score (21) with auto-reset, obs = 8 float32.
//
// Conventions fixed here (the configuration is silent): x to the right, y DOWN; every stored
// position is the top-left corner of its rectangle; action 1 = up = -y, 2 = down = +y, anything
// else = stay.  Order inside a step: agent paddle, opponent paddle (sees the ball before it moves),
// ball move, walls, paddle hits (moved paddles, post-wall ball), scoring, re-serve, episode end.
//
// Build with -ffp-contract=off and without fast-math: results are compared bit for bit.
#include <cstdint>
#include <cstring>
#include <cstdlib>
#include <thread>
#include <vector>

extern "C" {
void oracle_draw_block(uint64_t seed, uint32_t env, uint64_t step, uint32_t stream, uint32_t out[4]);
int32_t oracle_pong_action(uint32_t w);
float oracle_pong_serve_vx(uint32_t w);
float oracle_pong_serve_vy(uint32_t w);
}

namespace {

const float FIELD_W = 160.0f, FIELD_H = 210.0f;
const float PADDLE_W = 4.0f, PADDLE_H = 16.0f;
const float BALL_SIZE = 2.0f;
const float AGENT_X = 140.0f, OPP_X = 16.0f;
const float AGENT_SPEED = 4.0f, OPP_SPEED = 3.0f;
const float PADDLE_Y_MAX = 194.0f;   // FIELD_H - PADDLE_H
const float BALL_Y_MAX = 208.0f;     // FIELD_H - BALL_SIZE
const float SERVE_X = 79.0f, SERVE_Y = 104.0f;  // centred 2x2 ball
const float PADDLE_START_Y = 97.0f;  // centred paddle
const int FRAME = 84;

}  // namespace

extern "C" {

struct oracle_pong_env {
  float bx, by, vx, vy, pa, po;
  int32_t sa, so;
  int32_t ep_ret, ep_len;
};

struct oracle_pong_stats {
  int64_t episodes;
  int64_t return_sum;
  int64_t length_sum;
  int32_t return_min;
  int32_t return_max;
};

struct oracle_pong {
  int64_t n;
  uint64_t seed;
  uint64_t step;
  int32_t max_score;
  int32_t normalize;   // 1: observations are scaled at the source (paper App. B.1 item 8)
  oracle_pong_env* env;
  oracle_pong_stats stats;
};

static void stats_clear(oracle_pong_stats* s) {
  s->episodes = 0; s->return_sum = 0; s->length_sum = 0;
  s->return_min = INT32_MAX; s->return_max = INT32_MIN;
}

static void stats_add_episode(oracle_pong_stats* s, int32_t ret, int32_t len) {
  s->episodes += 1; s->return_sum += ret; s->length_sum += len;
  if (ret < s->return_min) s->return_min = ret;
  if (ret > s->return_max) s->return_max = ret;
}

static void stats_merge(oracle_pong_stats* into, const oracle_pong_stats* from) {
  into->episodes += from->episodes; into->return_sum += from->return_sum;
  into->length_sum += from->length_sum;
  if (from->return_min < into->return_min) into->return_min = from->return_min;
  if (from->return_max > into->return_max) into->return_max = from->return_max;
}

// One transition of one environment.  `action` in {0,1,2}; serve_vx/serve_vy are this step's serve
// draws (used only if a point is scored).  Returns the reward; *done = 1 on the transition that
// ends an episode (the state left behind is already the first state of the next episode).
// If an episode ends, its return and length are written to *fin_ret / *fin_len.
float oracle_pong_step_one(oracle_pong_env* e, int32_t action, float serve_vx, float serve_vy,
                           int32_t max_score, uint8_t* done, int32_t* fin_ret, int32_t* fin_len) {
  // 1. agent paddle
  if (action == 1) e->pa = e->pa - AGENT_SPEED;
  else if (action == 2) e->pa = e->pa + AGENT_SPEED;
  if (e->pa < 0.0f) e->pa = 0.0f;
  if (e->pa > PADDLE_Y_MAX) e->pa = PADDLE_Y_MAX;

  // 2. opponent paddle follows the centre of the ball as it was before this step's ball move
  float d = (e->by + 1.0f) - (e->po + 8.0f);
  if (d < -OPP_SPEED) d = -OPP_SPEED;
  if (d > OPP_SPEED) d = OPP_SPEED;
  e->po = e->po + d;
  if (e->po < 0.0f) e->po = 0.0f;
  if (e->po > PADDLE_Y_MAX) e->po = PADDLE_Y_MAX;

  // 3. ball
  e->bx = e->bx + e->vx;
  e->by = e->by + e->vy;

  // 4. walls: mirror the position, flip vy
  if (e->by < 0.0f) { e->by = -e->by; e->vy = -e->vy; }
  if (e->by > BALL_Y_MAX) { e->by = (2.0f * BALL_Y_MAX) - e->by; e->vy = -e->vy; }

  // 5. paddle hits
  if (e->vx > 0.0f && e->bx + BALL_SIZE >= AGENT_X && e->bx <= AGENT_X + PADDLE_W &&
      e->by + BALL_SIZE >= e->pa && e->by <= e->pa + PADDLE_H) {
    e->vx = -e->vx;
    e->bx = AGENT_X - BALL_SIZE;
    e->vy = 0.2f * ((e->by + 1.0f) - (e->pa + 8.0f));
  } else if (e->vx < 0.0f && e->bx <= OPP_X + PADDLE_W && e->bx + BALL_SIZE >= OPP_X &&
             e->by + BALL_SIZE >= e->po && e->by <= e->po + PADDLE_H) {
    e->vx = -e->vx;
    e->bx = OPP_X + PADDLE_W;
    e->vy = 0.2f * ((e->by + 1.0f) - (e->po + 8.0f));
  }

  // 6. scoring
  float reward = 0.0f;
  if (e->bx < 0.0f) { reward = 1.0f; e->sa += 1; }
  else if (e->bx + BALL_SIZE > FIELD_W) { reward = -1.0f; e->so += 1; }

  // 7. re-serve after a point (paddles stay where they are)
  if (reward != 0.0f) {
    e->bx = SERVE_X; e->by = SERVE_Y; e->vx = serve_vx; e->vy = serve_vy;
  }

  // 8./9. bookkeeping, episode end and auto-reset
  e->ep_ret += (int32_t)reward;
  e->ep_len += 1;
  *done = 0;
  if (e->sa == max_score || e->so == max_score) {
    *done = 1;
    if (fin_ret) *fin_ret = e->ep_ret;
    if (fin_len) *fin_len = e->ep_len;
    e->sa = 0; e->so = 0; e->pa = PADDLE_START_Y; e->po = PADDLE_START_Y;
    e->ep_ret = 0; e->ep_len = 0;
  }
  return reward;
}

void oracle_pong_obs_one(const oracle_pong_env* e, float obs[8]) {
  obs[0] = e->bx; obs[1] = e->by; obs[2] = e->vx; obs[3] = e->vy;
  obs[4] = e->pa; obs[5] = e->po; obs[6] = (float)e->sa; obs[7] = (float)e->so;
}

// Observation normalised at the source (paper App. B.1 item 8: constant denominators computed
// once, the scaling done inside the step).  Each component is one float32 multiplication by the
// float32 reciprocal of its range: ball x / 158, ball y / 208 and paddle y / 194 land in [0, 1],
// vx / 3 is +-1, vy / 2 lies in [-1, 1] (serves are within +-2, paddle spin within +-1.8), the
// scores are divided by max_score.
void oracle_pong_obs_one_normalized(const oracle_pong_env* e, int32_t max_score, float obs[8]) {
  const float inv_score = 1.0f / (float)max_score;
  obs[0] = e->bx * (1.0f / 158.0f); obs[1] = e->by * (1.0f / 208.0f);
  obs[2] = e->vx * (1.0f / 3.0f); obs[3] = e->vy * 0.5f;
  obs[4] = e->pa * (1.0f / 194.0f); obs[5] = e->po * (1.0f / 194.0f);
  obs[6] = (float)e->sa * inv_score; obs[7] = (float)e->so * inv_score;
}

static void write_obs(const oracle_pong* h, const oracle_pong_env* e, float* obs) {
  if (h->normalize) oracle_pong_obs_one_normalized(e, h->max_score, obs);
  else oracle_pong_obs_one(e, obs);
}

// Initial state of an episode started by env_reset: draws come from reset stream 16.
void oracle_pong_reset_one(oracle_pong_env* e, uint64_t seed, uint32_t env, uint64_t step) {
  uint32_t w[4];
  oracle_draw_block(seed, env, step, 16u, w);
  e->bx = SERVE_X; e->by = SERVE_Y;
  e->vx = oracle_pong_serve_vx(w[1]);
  e->vy = oracle_pong_serve_vy(w[2]);
  e->pa = PADDLE_START_Y; e->po = PADDLE_START_Y;
  e->sa = 0; e->so = 0; e->ep_ret = 0; e->ep_len = 0;
}

// Conservative (any-overlap) rasterisation of the three rectangles onto an 84x84 grid:
// pixel (r,c) is 255 iff some rectangle [x0,x0+w) x [y0,y0+h) overlaps the cell
// [160c/84, 160(c+1)/84) x [210r/84, 210(r+1)/84); tested in float32 with one multiply per side.
void oracle_pong_render_one(const oracle_pong_env* e, uint8_t* frame) {
  const float rx[3] = {AGENT_X, OPP_X, e->bx};
  const float ry[3] = {e->pa, e->po, e->by};
  const float rw[3] = {PADDLE_W, PADDLE_W, BALL_SIZE};
  const float rh[3] = {PADDLE_H, PADDLE_H, BALL_SIZE};
  for (int r = 0; r < FRAME; ++r) {
    for (int c = 0; c < FRAME; ++c) {
      uint8_t lit = 0;
      for (int k = 0; k < 3; ++k) {
        const float left = rx[k] * 84.0f, right = (rx[k] + rw[k]) * 84.0f;
        const float top = ry[k] * 84.0f, bottom = (ry[k] + rh[k]) * 84.0f;
        if (left < FIELD_W * (float)(c + 1) && right > FIELD_W * (float)c &&
            top < FIELD_H * (float)(r + 1) && bottom > FIELD_H * (float)r)
          lit = 255;
      }
      frame[r * FRAME + c] = lit;
    }
  }
}

oracle_pong* oracle_pong_create(int64_t n, uint64_t seed, int32_t max_score) {
  oracle_pong* h = (oracle_pong*)calloc(1, sizeof(oracle_pong));
  h->n = n; h->seed = seed; h->step = 0; h->max_score = max_score;
  h->env = (oracle_pong_env*)calloc((size_t)(n > 0 ? n : 1), sizeof(oracle_pong_env));
  stats_clear(&h->stats);
  for (int64_t i = 0; i < n; ++i) oracle_pong_reset_one(&h->env[i], seed, (uint32_t)i, 0);
  return h;
}

void oracle_pong_destroy(oracle_pong* h) { if (h) { free(h->env); free(h); } }

oracle_pong_env* oracle_pong_envs(oracle_pong* h) { return h->env; }
uint64_t oracle_pong_step_count(const oracle_pong* h) { return h->step; }
void oracle_pong_set_step_count(oracle_pong* h, uint64_t step) { h->step = step; }
void oracle_pong_set_normalize(oracle_pong* h, int32_t on) { h->normalize = on ? 1 : 0; }

void oracle_pong_get_stats(oracle_pong* h, oracle_pong_stats* out, int32_t clear) {
  *out = h->stats;
  if (clear) stats_clear(&h->stats);
}

// (Re)start every environment at the current step counter; obs[N,8] may be NULL.
void oracle_pong_reset(oracle_pong* h, float* obs) {
  for (int64_t i = 0; i < h->n; ++i) {
    oracle_pong_reset_one(&h->env[i], h->seed, (uint32_t)i, h->step);
    if (obs) write_obs(h, &h->env[i], obs + 8 * i);
  }
}

// T steps of environments [lo,hi).  actions: uint8 [T,N] or NULL (draw word 0 of the step block).
// obs [T,N,8], reward [T,N], done [T,N]; stack: optional u8 [N,4,84,84] ring of frames, the frame
// after the step with index s going to slot s mod 4.
static void run_range(oracle_pong* h, int64_t lo, int64_t hi, int32_t T, const uint8_t* actions,
                      float* obs, float* reward, uint8_t* done, uint8_t* stack,
                      oracle_pong_stats* st) {
  const int64_t n = h->n;
  for (int32_t t = 0; t < T; ++t) {
    const uint64_t s = h->step + (uint64_t)t;
    for (int64_t i = lo; i < hi; ++i) {
      uint32_t w[4];
      oracle_draw_block(h->seed, (uint32_t)i, s, 0u, w);
      const int32_t a = actions ? (int32_t)actions[(int64_t)t * n + i] : oracle_pong_action(w[0]);
      uint8_t dn = 0; int32_t fr = 0, fl = 0;
      const float r = oracle_pong_step_one(&h->env[i], a, oracle_pong_serve_vx(w[1]),
                                           oracle_pong_serve_vy(w[2]), h->max_score, &dn, &fr, &fl);
      if (dn) stats_add_episode(st, fr, fl);
      if (obs) write_obs(h, &h->env[i], obs + ((int64_t)t * n + i) * 8);
      if (reward) reward[(int64_t)t * n + i] = r;
      if (done) done[(int64_t)t * n + i] = dn;
      if (stack) oracle_pong_render_one(&h->env[i], stack + ((size_t)i * 4 + (size_t)(s & 3)) * FRAME * FRAME);
    }
  }
}

void oracle_pong_rollout(oracle_pong* h, int32_t T, const uint8_t* actions, float* obs,
                         float* reward, uint8_t* done, uint8_t* stack, int32_t nthreads) {
  if (nthreads <= 1) {
    run_range(h, 0, h->n, T, actions, obs, reward, done, stack, &h->stats);
  } else {
    std::vector<std::thread> pool;
    std::vector<oracle_pong_stats> part((size_t)nthreads);
    for (int k = 0; k < nthreads; ++k) {
      stats_clear(&part[k]);
      const int64_t lo = h->n * k / nthreads, hi = h->n * (k + 1) / nthreads;
      pool.emplace_back(run_range, h, lo, hi, T, actions, obs, reward, done, stack, &part[k]);
    }
    for (auto& th : pool) th.join();
    for (int k = 0; k < nthreads; ++k) stats_merge(&h->stats, &part[k]);
  }
  h->step += (uint64_t)T;
}

// One step of the whole batch (actions uint8[N] or NULL, obs[N,8], reward[N], done[N]).
void oracle_pong_step(oracle_pong* h, const uint8_t* actions, float* obs, float* reward,
                      uint8_t* done, uint8_t* stack) {
  oracle_pong_rollout(h, 1, actions, obs, reward, done, stack, 1);
}

// Fill all four ring slots of every environment with the frame of its current state.
void oracle_pong_fill_stack(oracle_pong* h, uint8_t* stack) {
  for (int64_t i = 0; i < h->n; ++i) {
    uint8_t* base = stack + (size_t)i * 4 * FRAME * FRAME;
    oracle_pong_render_one(&h->env[i], base);
    for (int k = 1; k < 4; ++k) memcpy(base + k * FRAME * FRAME, base, FRAME * FRAME);
  }
}

}  // extern "C"
