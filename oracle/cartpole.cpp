// TEST INFRASTRUCTURE — CPU oracle. Not part of the product path; shares no code with the HIP library.
//
// CartPole, the third workload of the fused-rollout path (the paper's Table 8 lists a CartPole scan
// rollout; App. B.1 item 5 reports the 3.2x gain of fusing its loop).  Dynamics: the classic
// cart-pole of Barto, Sutton and Anderson (1983) in the usual benchmark parametrisation:
// cart 1.0 kg, pole 0.1 kg, half-length 0.5 m, g = 9.8, force +-10 N, Euler steps of 0.02 s,
// failure at |x| > 2.4 m or |theta| > 12 degrees, reward 1 per step, truncation at 500 steps.
//   temp      = (F + m_p l thetadot^2 sin theta) / (m_c + m_p)
//   thetaacc  = (g sin theta - cos theta temp) / (l (4/3 - m_p cos^2 theta / (m_c + m_p)))
//   xacc      = temp - m_p l thetaacc cos theta / (m_c + m_p)
// float32, one IEEE operation per source operation in the order written (build with
// -ffp-contract=off).  sin / cos use the fixed polynomials below (theta stays within +-0.21 rad
// until the episode ends), so that trajectories can be compared bit for bit with an implementation
// that evaluates the same polynomials in the same order.
#include <cstdint>
#include <cstdlib>
#include <thread>
#include <vector>

extern "C" {
void oracle_draw_block(uint64_t seed, uint32_t env, uint64_t step, uint32_t stream, uint32_t out[4]);
float oracle_u01(uint32_t w);
}

extern "C" {

struct oracle_cartpole_env { float x, xd, th, thd; int32_t ep_len; };
struct oracle_cartpole_stats { int64_t episodes, length_sum; int32_t length_min, length_max; };
struct oracle_cartpole {
  int64_t n; uint64_t seed, step; int32_t max_steps;
  oracle_cartpole_env* env;
  oracle_cartpole_stats stats;
};

// sin x = x (1 - x^2/6 + x^4/120 - x^6/5040), Horner in x^2
float oracle_cartpole_sin(float x) {
  const float x2 = x * x;
  float p = -(1.0f / 5040.0f);
  p = p * x2; p = p + (1.0f / 120.0f);
  p = p * x2; p = p - (1.0f / 6.0f);
  p = p * x2; p = p + 1.0f;
  return x * p;
}
// cos x = 1 - x^2/2 + x^4/24 - x^6/720 + x^8/40320, Horner in x^2
float oracle_cartpole_cos(float x) {
  const float x2 = x * x;
  float p = 1.0f / 40320.0f;
  p = p * x2; p = p - (1.0f / 720.0f);
  p = p * x2; p = p + (1.0f / 24.0f);
  p = p * x2; p = p - 0.5f;
  p = p * x2; p = p + 1.0f;
  return p;
}

// accelerations (xacc, thetaacc) at a state under force F
void oracle_cartpole_accel(float th, float thd, float force, float* xacc, float* thacc) {
  const float s = oracle_cartpole_sin(th), c = oracle_cartpole_cos(th);
  const float temp = (force + ((0.05f * thd) * thd) * s) / 1.1f;
  const float denom = 0.5f * ((4.0f / 3.0f) - ((0.1f * c) * c) / 1.1f);
  *thacc = (9.8f * s - c * temp) / denom;
  *xacc = temp - ((0.05f * *thacc) * c) / 1.1f;
}

void oracle_cartpole_reset_one(oracle_cartpole_env* e, uint64_t seed, uint32_t env, uint64_t step) {
  uint32_t w[4];
  oracle_draw_block(seed, env, step, 16u, w);
  e->x = -0.05f + 0.1f * oracle_u01(w[0]);
  e->xd = -0.05f + 0.1f * oracle_u01(w[1]);
  e->th = -0.05f + 0.1f * oracle_u01(w[2]);
  e->thd = -0.05f + 0.1f * oracle_u01(w[3]);
  e->ep_len = 0;
}

// One transition; action 1 pushes right, anything else left.  Returns 1 if the episode ended
// (failure or truncation); the state left behind is then the next episode's initial state.
int32_t oracle_cartpole_step_one(oracle_cartpole_env* e, int32_t action, int32_t max_steps, uint64_t seed,
                                 uint32_t env, uint64_t step, int32_t* fin_len) {
  const float force = (action == 1) ? 10.0f : -10.0f;
  float xacc, thacc;
  oracle_cartpole_accel(e->th, e->thd, force, &xacc, &thacc);
  e->x = e->x + 0.02f * e->xd;
  e->xd = e->xd + 0.02f * xacc;
  e->th = e->th + 0.02f * e->thd;
  e->thd = e->thd + 0.02f * thacc;
  e->ep_len += 1;
  const bool failed = e->x < -2.4f || e->x > 2.4f || e->th < -0.20943951f || e->th > 0.20943951f;
  if (failed || e->ep_len >= max_steps) {
    if (fin_len) *fin_len = e->ep_len;
    oracle_cartpole_reset_one(e, seed, env, step + 1);
    return 1;
  }
  return 0;
}

static void stats_clear(oracle_cartpole_stats* s) {
  s->episodes = 0; s->length_sum = 0; s->length_min = INT32_MAX; s->length_max = INT32_MIN;
}

oracle_cartpole* oracle_cartpole_create(int64_t n, uint64_t seed, int32_t max_steps) {
  oracle_cartpole* h = (oracle_cartpole*)calloc(1, sizeof(oracle_cartpole));
  h->n = n; h->seed = seed; h->step = 0; h->max_steps = max_steps;
  h->env = (oracle_cartpole_env*)calloc((size_t)(n > 0 ? n : 1), sizeof(oracle_cartpole_env));
  stats_clear(&h->stats);
  for (int64_t i = 0; i < n; ++i) oracle_cartpole_reset_one(&h->env[i], seed, (uint32_t)i, 0);
  return h;
}
void oracle_cartpole_destroy(oracle_cartpole* h) { if (h) { free(h->env); free(h); } }
oracle_cartpole_env* oracle_cartpole_envs(oracle_cartpole* h) { return h->env; }
uint64_t oracle_cartpole_step_count(const oracle_cartpole* h) { return h->step; }
void oracle_cartpole_set_step_count(oracle_cartpole* h, uint64_t s) { h->step = s; }
void oracle_cartpole_get_stats(oracle_cartpole* h, oracle_cartpole_stats* out, int32_t clear) {
  *out = h->stats;
  if (clear) stats_clear(&h->stats);
}

void oracle_cartpole_reset(oracle_cartpole* h, float* obs) {
  for (int64_t i = 0; i < h->n; ++i) {
    oracle_cartpole_reset_one(&h->env[i], h->seed, (uint32_t)i, h->step);
    if (obs) { obs[4 * i] = h->env[i].x; obs[4 * i + 1] = h->env[i].xd; obs[4 * i + 2] = h->env[i].th; obs[4 * i + 3] = h->env[i].thd; }
  }
}

static void run_range(oracle_cartpole* h, int64_t lo, int64_t hi, int32_t T, const uint8_t* actions,
                      float* obs, float* reward, uint8_t* done, oracle_cartpole_stats* st) {
  const int64_t n = h->n;
  for (int32_t t = 0; t < T; ++t) {
    const uint64_t s = h->step + (uint64_t)t;
    for (int64_t i = lo; i < hi; ++i) {
      uint32_t w[4];
      oracle_draw_block(h->seed, (uint32_t)i, s, 0u, w);
      const int32_t a = actions ? (int32_t)actions[(int64_t)t * n + i] : (int32_t)(w[0] >> 31);
      int32_t fin = 0;
      const int32_t d = oracle_cartpole_step_one(&h->env[i], a, h->max_steps, h->seed, (uint32_t)i, s, &fin);
      if (d) {
        st->episodes += 1; st->length_sum += fin;
        if (fin < st->length_min) st->length_min = fin;
        if (fin > st->length_max) st->length_max = fin;
      }
      const int64_t k = (int64_t)t * n + i;
      if (obs) { obs[4 * k] = h->env[i].x; obs[4 * k + 1] = h->env[i].xd; obs[4 * k + 2] = h->env[i].th; obs[4 * k + 3] = h->env[i].thd; }
      if (reward) reward[k] = 1.0f;
      if (done) done[k] = (uint8_t)d;
    }
  }
}

void oracle_cartpole_rollout(oracle_cartpole* h, int32_t T, const uint8_t* actions, float* obs, float* reward,
                             uint8_t* done, int32_t nthreads) {
  if (nthreads <= 1) {
    run_range(h, 0, h->n, T, actions, obs, reward, done, &h->stats);
  } else {
    std::vector<std::thread> pool;
    std::vector<oracle_cartpole_stats> part((size_t)nthreads);
    for (int k = 0; k < nthreads; ++k) {
      stats_clear(&part[(size_t)k]);
      pool.emplace_back(run_range, h, h->n * k / nthreads, h->n * (k + 1) / nthreads, T, actions, obs, reward,
                        done, &part[(size_t)k]);
    }
    for (auto& th : pool) th.join();
    for (auto& p : part) {
      h->stats.episodes += p.episodes; h->stats.length_sum += p.length_sum;
      if (p.length_min < h->stats.length_min) h->stats.length_min = p.length_min;
      if (p.length_max > h->stats.length_max) h->stats.length_max = p.length_max;
    }
  }
  h->step += (uint64_t)T;
}

}  // extern "C"
