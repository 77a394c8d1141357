// Host-side policy: speculation utility and the test-and-set choice of K.
//
// Paper: Section 4 (utility = ETR / (t_spec_iter / t_base_iter), Theorem 1), Section 5.3
// (test phase of up to M trials of t iterations, then a set phase of S iterations at the best K;
// baseline time from the first few no-speculation iterations, refreshed rarely; K_start from recent
// history), Section 5.4 (utility < 1 -> K = 0 for the set phase; stop testing at K = 1), Section 5.5
// (double S whenever K drops to 0), Section 5.6 (hill climbing on the direction of utility change,
// three early exits), Section 6 (t = 4, T = 16, S = 16), Section 7.4 (K_start = 3).
//
// Pure host code: plain conditionals and double arithmetic, no device calls.  Built without
// floating-point contraction so that replaying a trace gives the same decisions everywhere.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "cascade_moe.h"

namespace {

enum Phase : int32_t { kBaseline = 0, kTest = 1, kSet = 2 };

struct Record {
  int32_t k;
  double u;
};

}  // namespace

struct cascade_ctrl {
  cascade_params p;
  Phase phase;
  int32_t cur_k;    // K of the running trial / set phase
  int32_t left;     // iterations left in the running baseline window / trial / set phase
  int32_t s_cur;    // current set-phase length (grows under back-off)
  int32_t prev_set_k;  // K of the previous set phase, -1 before the first
  int64_t iters, last_refresh, trial_iters;
  double t_base, last_u;
  // accumulators of the running window
  int64_t acc_tokens;
  double acc_time;
  std::vector<double> tail;  // last base_iters iteration times of a K = 0 set phase
  // running test phase
  std::vector<Record> trials;
  bool have_best;
  Record best;
  // utility records of the last two cycles (trials + speculative set phase), oldest first
  std::vector<Record> cycle_prev, cycle_last, cycle_cur;
};

namespace {

bool better(const Record& a, bool have, const Record& b) {  // is a better than the incumbent b?
  return !have || a.u > b.u || (a.u == b.u && a.k < b.k);
}

void begin_window(cascade_ctrl* c, Phase ph, int32_t k, int32_t len) {
  c->phase = ph;
  c->cur_k = k;
  c->left = len;
  c->acc_tokens = 0;
  c->acc_time = 0.0;
}

void enter_baseline(cascade_ctrl* c) { begin_window(c, kBaseline, 0, c->p.base_iters); }

int32_t pick_k_start(const cascade_ctrl* c) {
  if (c->prev_set_k == 0) return 1;  // after a disabled set phase each cycle restarts at K = 1
  bool have = false;
  Record b{0, 0.0};
  for (const std::vector<Record>* cyc : {&c->cycle_prev, &c->cycle_last})
    for (const Record& r : *cyc)
      if (r.k > 0 && better(r, have, b)) {
        b = r;
        have = true;
      }
  int32_t k = have ? b.k : c->p.k_start;
  if (k < 1) k = 1;
  if (k > c->p.k_max) k = c->p.k_max;
  return k;
}

void enter_test(cascade_ctrl* c) {
  c->cycle_cur.clear();
  c->trials.clear();
  c->have_best = false;
  begin_window(c, kTest, pick_k_start(c), c->p.t_trial);
}

void enter_set(cascade_ctrl* c, int32_t k_set) {
  const cascade_params& p = c->p;
  // Section 5.5: "double the set phase length S whenever K drops to 0"; its figure speaks of utility that is
  // "persistently" below 1.  backoff = 1 (default) lets the first disabled set phase keep S and doubles from the
  // second consecutive drop on; backoff = 2 takes the sentence literally (the first one already lasts 2 S).  Both
  // reproduce the section's worked example equally (20 trial iterations in the first 250 against 54 without).
  // Any set phase that speculates puts S back.
  if (k_set == 0 && p.backoff && (p.backoff == 2 || c->prev_set_k == 0)) {
    c->s_cur *= 2;
    if (p.s_max > 0 && c->s_cur > p.s_max) c->s_cur = p.s_max;
  } else {
    c->s_cur = p.s_set;
  }
  c->tail.clear();
  begin_window(c, kSet, k_set, c->s_cur);
}

double window_utility(const cascade_ctrl* c, int32_t n) {
  return cascade_utility((double)c->acc_tokens / (double)n, c->acc_time / (double)n, c->t_base);
}

void end_trial(cascade_ctrl* c) {
  const cascade_params& p = c->p;
  const Record cur{c->cur_k, window_utility(c, p.t_trial)};
  c->last_u = cur.u;
  c->trials.push_back(cur);
  c->cycle_cur.push_back(cur);
  if (better(cur, c->have_best, c->best)) {
    c->best = cur;
    c->have_best = true;
  }
  const size_t j = c->trials.size();
  bool done = (int32_t)j >= p.max_trials || !p.hillclimb;
  if (cur.k == 1 && cur.u < 1.0) done = true;  // nothing more conservative left to try
  if (j >= 3 && c->trials[j - 1].u < c->trials[j - 2].u && c->trials[j - 2].u < c->trials[j - 3].u) done = true;
  if (j >= 2 && std::fabs(cur.u - c->trials[j - 2].u) <= p.converge_frac * c->trials[j - 2].u) done = true;
  int32_t next = 0;
  if (!done) {
    if (j == 1) {
      next = cur.k + (cur.u >= 1.0 ? 1 : -1);
    } else {
      const Record& prev = c->trials[j - 2];
      const int32_t step = cur.k > prev.k ? 1 : -1;
      next = cur.u > prev.u ? cur.k + step : prev.k - step;  // keep climbing, or backtrack past prev-K
    }
    if (next < 1 || next > p.k_max) done = true;
    for (const Record& r : c->trials)
      if (r.k == next) done = true;
  }
  if (done)
    enter_set(c, c->best.u >= 1.0 ? c->best.k : 0);
  else
    begin_window(c, kTest, next, p.t_trial);
}

void end_set(cascade_ctrl* c) {
  const cascade_params& p = c->p;
  const int32_t k = c->cur_k;
  if (k > 0) {
    const Record r{k, window_utility(c, c->s_cur)};
    c->last_u = r.u;
    c->cycle_cur.push_back(r);
  } else if ((int32_t)c->tail.size() == p.base_iters) {
    double s = 0.0;  // a disabled set phase is itself a no-speculation measurement
    for (double v : c->tail) s += v;
    c->t_base = s / (double)p.base_iters;
    c->last_refresh = c->iters;
  }
  c->cycle_prev.swap(c->cycle_last);
  c->cycle_last = c->cycle_cur;
  c->prev_set_k = k;
  if (c->iters - c->last_refresh >= p.base_refresh)
    enter_baseline(c);
  else
    enter_test(c);
}

}  // namespace

extern "C" {

double cascade_utility(double tokens_per_iter, double t_verify, double t_base) {
  if (!(t_verify > 0.0) || !(t_base > 0.0)) return std::nan("");
  return tokens_per_iter / (t_verify / t_base);
}

void cascade_default_params(cascade_params* p) {
  if (!p) return;
  p->t_trial = 4;
  p->max_trials = 4;
  p->s_set = 16;
  p->k_max = 8;
  p->k_start = 3;
  p->base_iters = 4;
  p->base_refresh = 100;
  p->s_max = 0;
  p->converge_frac = 0.10;
  p->backoff = 1;
  p->hillclimb = 1;
}

cascade_ctrl* cascade_ctrl_create(const cascade_params* params) {
  cascade_params p;
  if (params)
    p = *params;
  else
    cascade_default_params(&p);
  if (p.t_trial < 1 || p.max_trials < 1 || p.s_set < 1 || p.k_max < 1 || p.base_iters < 1 || p.base_refresh < 1 ||
      p.k_start < 1 || p.k_start > p.k_max || p.s_max < 0 || !(p.converge_frac >= 0.0) || p.s_set > (1 << 24) ||
      p.s_max > (1 << 24) || p.backoff < 0 || p.backoff > 2)
    return nullptr;
  cascade_ctrl* c = new (std::nothrow) cascade_ctrl();
  if (!c) return nullptr;
  c->p = p;
  c->s_cur = p.s_set;
  c->prev_set_k = -1;
  c->iters = c->last_refresh = c->trial_iters = 0;
  c->t_base = std::nan("");
  c->last_u = std::nan("");
  c->have_best = false;
  c->best = Record{0, 0.0};
  enter_baseline(c);
  return c;
}

void cascade_ctrl_destroy(cascade_ctrl* c) { delete c; }

int32_t cascade_next_k(const cascade_ctrl* c) { return c ? c->cur_k : 0; }

moe_status cascade_observe(cascade_ctrl* c, int32_t k_used, int32_t tokens_emitted, double t_iter) {
  if (!c || k_used != c->cur_k || tokens_emitted < 1 || tokens_emitted > k_used + 1 || !(t_iter > 0.0) ||
      std::isinf(t_iter))
    return MOE_ERR_INVALID_ARG;
  c->iters += 1;
  c->acc_time += t_iter;
  c->acc_tokens += tokens_emitted;
  c->left -= 1;
  switch (c->phase) {
    case kBaseline:
      if (c->left == 0) {
        c->t_base = c->acc_time / (double)c->p.base_iters;
        c->last_refresh = c->iters;
        enter_test(c);
      }
      break;
    case kTest:
      c->trial_iters += 1;
      if (c->left == 0) end_trial(c);
      break;
    case kSet:
      c->tail.push_back(t_iter);
      if ((int32_t)c->tail.size() > c->p.base_iters) c->tail.erase(c->tail.begin());
      if (c->left == 0) end_set(c);
      break;
  }
  return MOE_OK;
}

void cascade_get_state(const cascade_ctrl* c, cascade_state* out) {
  if (!c || !out) return;
  out->phase = c->phase;
  out->cur_k = c->cur_k;
  out->s_cur = c->s_cur;
  out->trials_done = c->phase == kTest ? (int32_t)c->trials.size() : 0;
  out->iters = c->iters;
  out->trial_iters = c->trial_iters;
  out->t_base = c->t_base;
  out->last_utility = c->last_u;
}

}  // extern "C"
