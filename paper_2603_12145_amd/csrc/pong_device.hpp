// Pong transition for one environment held in the registers of one lane (gfx950, float32).
//
// Workload: the paper's "Puffer Pong" case study (Table 1; App. A.1) with the dynamics of the
// benchmark configuration: 160x210 field, 4x16 paddles at x=140 (agent) / x=16 (opponent), agent
// speed 4, opponent follows the ball centre at speed <= 3, 2x2 ball served from the centre at +-3
// in x and uniform [-2,2) in y, mirror reflection at the top/bottom walls, paddle hit sets
// vy = 0.2 * (ball centre - paddle centre), +-1 reward per point, episode ends at max_score.
// y grows downwards; every position is the top-left corner of its rectangle.
//
// The collision logic is written with selects only (paper App. B.1 item 2): a wavefront never
// diverges inside a step.  Compiled with -ffp-contract=off: every operation below is a single
// IEEE float32 operation in the order written, which is what makes trajectories reproducible
// bit for bit against a scalar CPU implementation.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "philox.hpp"

namespace envk {

constexpr int PONG_FIELDS = 10;  // bx by vx vy pa po | sa so ep_ret ep_len
constexpr int PONG_OBS = 8;
constexpr int PONG_FLOAT_FIELDS = 6;   // the first six fields are float32, the rest int32

struct PongLane {
  float bx, by, vx, vy, pa, po;
  int sa, so, ep_ret, ep_len;
};

struct PongEvent {
  float reward;
  bool done;
  int fin_ret, fin_len;  // valid when done
};

__device__ __forceinline__ float pong_serve_vx(uint32_t w) { return (w >> 31) ? 3.0f : -3.0f; }
__device__ __forceinline__ float pong_serve_vy(uint32_t w) { return -2.0f + 4.0f * unit_float(w); }
__device__ __forceinline__ int pong_action_from_word(uint32_t w) { return (int)__umulhi(w, 3u); }

// Bit-exactness notes for the branch-free forms below (all values are finite, never NaN):
//  * clamp(x, lo, hi) as min(max(x, lo), hi) equals the compare-and-assign form except for the
//    sign of a zero; a negative zero cannot reach a clamp (paddle positions are sums of
//    non-negative-zero terms, and x + (-x) rounds to +0).
//  * the top-wall mirror "if (by < 0) { by = -by; vy = -vy; }" is done on the sign bit: by is a sum
//    whose operands are never -0, so "sign bit set" and "by < 0" coincide.
//  * the bottom-wall mirror by = min(by, 416 - by): for by <= 208 the rounded 416 - by is >= 208,
//    for by > 208 it is < 208, so the minimum picks exactly what the comparison would.
__device__ __forceinline__ float clampf(float x, float lo, float hi) {
  return __builtin_fminf(__builtin_fmaxf(x, lo), hi);
}

// The agent's paddle displacement for an action code, and for an action drawn from a Philox word w:
// floor(3 w / 2^32) is 1 (up) from ceil(2^32 / 3) and 2 (down) from ceil(2^33 / 3), so two
// comparisons replace the quarter-rate multiply of pong_action_from_word.
__device__ __forceinline__ float pong_move_of_action(int action) {
  return (action == 1) ? -4.0f : ((action == 2) ? 4.0f : 0.0f);
}
__device__ __forceinline__ float pong_move_of_word(uint32_t w) {
  return (w >= 0xAAAAAAABu) ? 4.0f : ((w >= 0x55555556u) ? -4.0f : 0.0f);
}

// What one step does to paddles and ball, before any bookkeeping: s.bx, s.by, s.vx, s.vy are
// updated (a point re-serves the ball), the moved paddles and the point flags are returned.
struct PongFlight {
  float pa, po;           // paddles after their move (an episode end puts them back to 97)
  bool point_a, point_o;  // the agent / the opponent scored in this step
  float reward;
};

__device__ __forceinline__ PongFlight pong_flight(PongLane& s, const float move, uint32_t w_vx, uint32_t w_vy) {
  // agent paddle, then opponent paddle (which looks at the ball before it moves)
  const float pa = clampf(s.pa + move, 0.0f, 194.0f);
  const float chase = clampf((s.by + 1.0f) - (s.po + 8.0f), -3.0f, 3.0f);
  const float po = clampf(s.po + chase, 0.0f, 194.0f);

  // ball flight and wall mirrors
  float bx = s.bx + s.vx;
  const float by_raw = s.by + s.vy;
  const uint32_t top_sign = __float_as_uint(by_raw) & 0x80000000u;
  const float by_top = __uint_as_float(__float_as_uint(by_raw) ^ top_sign);
  float vy = __uint_as_float(__float_as_uint(s.vy) ^ top_sign);
  const bool under_bottom = by_top > 208.0f;
  float by = __builtin_fminf(by_top, 416.0f - by_top);
  vy = under_bottom ? -vy : vy;
  float vx = s.vx;

  // paddle faces: the ball must be travelling towards the paddle and overlap it
  // (bitwise & on purpose: no short-circuit branches inside the step)
  const float by_bottom = by + 2.0f, bx_right = bx + 2.0f;
  const bool rows_a = (by_bottom >= pa) & (by <= pa + 16.0f);
  const bool rows_o = (by_bottom >= po) & (by <= po + 16.0f);
  const bool hit_a = (vx > 0.0f) & (bx_right >= 140.0f) & (bx <= 144.0f) & rows_a;
  const bool hit_o = (vx < 0.0f) & (bx <= 20.0f) & (bx_right >= 16.0f) & rows_o;
  const bool hit = hit_a | hit_o;
  const float paddle_y = hit_a ? pa : po;
  const float spin = 0.2f * ((by + 1.0f) - (paddle_y + 8.0f));
  vx = hit ? -vx : vx;
  vy = hit ? spin : vy;
  bx = hit_a ? 138.0f : bx;
  bx = hit_o ? 20.0f : bx;

  // points and re-serve (paddles stay put)
  PongFlight f;
  f.pa = pa; f.po = po;
  f.point_a = bx < 0.0f;
  f.point_o = (!f.point_a) & (bx + 2.0f > 160.0f);
  const bool point = f.point_a | f.point_o;
  f.reward = f.point_a ? 1.0f : (f.point_o ? -1.0f : 0.0f);
  // both operands of every select are computed first: a call inside the conditional operator is
  // a branch to the compiler, which it may or may not turn back into a select
  const float serve_vx = pong_serve_vx(w_vx), serve_vy = pong_serve_vy(w_vy);
  s.bx = point ? 79.0f : bx;
  s.by = point ? 104.0f : by;
  s.vx = point ? serve_vx : vx;
  s.vy = point ? serve_vy : vy;
  return f;
}

__device__ __forceinline__ PongEvent pong_transition_move(PongLane& s, const float move, uint32_t w_vx,
                                                          uint32_t w_vy, int max_score) {
  const PongFlight f = pong_flight(s, move, w_vx, w_vy);
  PongEvent ev;
  ev.reward = f.reward;
  const int sa = s.sa + (f.point_a ? 1 : 0);
  const int so = s.so + (f.point_o ? 1 : 0);
  // episode bookkeeping and auto-reset
  const int ep_ret = s.ep_ret + (f.point_a ? 1 : 0) - (f.point_o ? 1 : 0);
  const int ep_len = s.ep_len + 1;
  ev.done = (sa == max_score) | (so == max_score);
  ev.fin_ret = ep_ret;
  ev.fin_len = ep_len;
  s.pa = ev.done ? 97.0f : f.pa;
  s.po = ev.done ? 97.0f : f.po;
  s.sa = ev.done ? 0 : sa;
  s.so = ev.done ? 0 : so;
  s.ep_ret = ev.done ? 0 : ep_ret;
  s.ep_len = ev.done ? 0 : ep_len;
  return ev;
}

// Episode bookkeeping of one lane for the length of a launch, kept in a form that costs three
// vector instructions per step instead of fourteen (return so far, length so far, and the five
// accumulators of the episode statistics).  R counts points (agent minus opponent) and is never
// put back to zero; R0 is its value when the lane's last episode ended, so the return so far is
// R - R0; the length so far after the launch's k-th step is k + len0.  What an episode's end adds to
// the statistics is taken from these later, at a flush (see pong_books_flush): its return is
// R0 - R0_seen, and the lengths of all episodes a lane finished in a launch add up to
// (length at the start) + (steps of the launch) - (length at the end), which needs no per-step work.
// A flush can tell episode ends apart only if at most one happened in the lane since the last
// flush.  An episode ends on a point, every point re-serves the ball from the centre at |vx| = 3,
// and from there it needs 27 steps to reach either edge: whatever state a lane was given, two
// episode ends are at least 27 steps apart, so a flush every 8 steps or fewer misses none.
// Unsigned arithmetic: differences are exact modulo 2^32.
struct PongBooks {
  uint32_t R, R0, R0_seen, len0;
  unsigned long long ended;   // wave-uniform: the lanes in which an episode ended since the last flush
};

__device__ __forceinline__ PongBooks pong_books_open(const PongLane& s) {
  return PongBooks{(uint32_t)s.ep_ret, 0u, 0u, (uint32_t)s.ep_len, 0ull};
}

// Step number `steps_taken` (1-based) of the launch.  s.ep_ret and s.ep_len are not maintained;
// pong_books_close puts them back.  Returns the step's reward and done flag.
__device__ __forceinline__ PongFlight pong_transition_booked(PongLane& s, PongBooks& b, const float move,
                                                             uint32_t w_vx, uint32_t w_vy, int max_score,
                                                             uint32_t steps_taken, bool& done) {
  const PongFlight f = pong_flight(s, move, w_vx, w_vy);
  const int sa = s.sa + (f.point_a ? 1 : 0);
  const int so = s.so + (f.point_o ? 1 : 0);
  b.R += f.point_a ? 1u : 0u;
  b.R -= f.point_o ? 1u : 0u;
  done = (sa == max_score) | (so == max_score);
  b.R0 = done ? b.R : b.R0;
  b.len0 = done ? 0u - steps_taken : b.len0;
  b.ended |= __ballot(done);
  s.pa = done ? 97.0f : f.pa;
  s.po = done ? 97.0f : f.po;
  s.sa = done ? 0 : sa;
  s.so = done ? 0 : so;
  return f;
}

// Wave-uniform branch; all lanes of the wavefront call it.  `counts` = the lane owns an environment.
template <class Episodes>
__device__ __forceinline__ void pong_books_flush(PongBooks& b, Episodes& le, bool counts) {
  if (b.ended == 0ull) return;
  if (__builtin_amdgcn_inverse_ballot_w64(b.ended) && counts) {   // the mask itself becomes the lanes' predicate
    const int fin_ret = (int)(b.R0 - b.R0_seen);
    le.count += 1;
    le.ret_sum_i += fin_ret;
    le.min_key = min(le.min_key, fin_ret);
    le.max_key = max(le.max_key, fin_ret);
    b.R0_seen = b.R0;
  }
  b.ended = 0ull;
}

// After `steps` steps: restores s.ep_ret / s.ep_len and adds the finished episodes' lengths.
template <class Episodes>
__device__ __forceinline__ void pong_books_close(PongLane& s, const PongBooks& b, Episodes& le, uint32_t steps,
                                                 bool counts) {
  const uint32_t len_end = steps + b.len0;
  le.length_sum += counts ? (int)((uint32_t)s.ep_len + steps - len_end) : 0;
  s.ep_ret = (int)(b.R - b.R0);
  s.ep_len = (int)len_end;
}

__device__ __forceinline__ PongEvent pong_transition(PongLane& s, int action, uint32_t w_vx,
                                                     uint32_t w_vy, int max_score) {
  return pong_transition_move(s, pong_move_of_action(action), w_vx, w_vy, max_score);
}

// First state of an episode started by env_reset: serve drawn from reset stream 16.
__device__ __forceinline__ PongLane pong_initial(uint64_t seed, uint32_t env, uint64_t step) {
  const Draw4 d = philox_draw(seed, env, step, 16u);
  PongLane s;
  s.bx = 79.0f; s.by = 104.0f;
  s.vx = pong_serve_vx(d.w1);
  s.vy = pong_serve_vy(d.w2);
  s.pa = 97.0f; s.po = 97.0f;
  s.sa = 0; s.so = 0; s.ep_ret = 0; s.ep_len = 0;
  return s;
}

// The 8-float observation as two 16-byte halves.  NORMALIZE: scaled at the source (paper App. B.1
// item 8) by one float32 multiplication per component with the reciprocal of its range
// (ball x 158, ball y 208, vx 3, vy 2, paddles 194, scores max_score).
template <bool NORMALIZE>
__device__ __forceinline__ void pong_observe(const PongLane& s, float inv_score, float4& lo, float4& hi) {
  if (NORMALIZE) {
    lo = make_float4(s.bx * (1.0f / 158.0f), s.by * (1.0f / 208.0f), s.vx * (1.0f / 3.0f), s.vy * 0.5f);
    hi = make_float4(s.pa * (1.0f / 194.0f), s.po * (1.0f / 194.0f), (float)s.sa * inv_score,
                     (float)s.so * inv_score);
  } else {
    lo = make_float4(s.bx, s.by, s.vx, s.vy);
    hi = make_float4(s.pa, s.po, (float)s.sa, (float)s.so);
  }
}

// SoA state: field f of environment i lives at state[f * n + i] (coalesced across a wavefront).
__device__ __forceinline__ PongLane pong_load(const uint32_t* __restrict__ state, int64_t n,
                                              int64_t i) {
  PongLane s;
  s.bx = __uint_as_float(state[0 * n + i]); s.by = __uint_as_float(state[1 * n + i]);
  s.vx = __uint_as_float(state[2 * n + i]); s.vy = __uint_as_float(state[3 * n + i]);
  s.pa = __uint_as_float(state[4 * n + i]); s.po = __uint_as_float(state[5 * n + i]);
  s.sa = (int)state[6 * n + i]; s.so = (int)state[7 * n + i];
  s.ep_ret = (int)state[8 * n + i]; s.ep_len = (int)state[9 * n + i];
  return s;
}

__device__ __forceinline__ void pong_store(uint32_t* __restrict__ state, int64_t n, int64_t i,
                                           const PongLane& s) {
  state[0 * n + i] = __float_as_uint(s.bx); state[1 * n + i] = __float_as_uint(s.by);
  state[2 * n + i] = __float_as_uint(s.vx); state[3 * n + i] = __float_as_uint(s.vy);
  state[4 * n + i] = __float_as_uint(s.pa); state[5 * n + i] = __float_as_uint(s.po);
  state[6 * n + i] = (uint32_t)s.sa; state[7 * n + i] = (uint32_t)s.so;
  state[8 * n + i] = (uint32_t)s.ep_ret; state[9 * n + i] = (uint32_t)s.ep_len;
}

__device__ __forceinline__ PongLane pong_idle_lane() {
  PongLane s;
  s.bx = 79.0f; s.by = 104.0f; s.vx = 0.0f; s.vy = 0.0f; s.pa = 97.0f; s.po = 97.0f;
  s.sa = 0; s.so = 0; s.ep_ret = 0; s.ep_len = 0;
  return s;
}

}  // namespace envk
