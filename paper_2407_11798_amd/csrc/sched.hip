// Head-node run bookkeeping (Sections "State tracking", "Invalidation detection", "Cancellation
// back-propagation", "Reactive speculation"): host code only.  A queue of run records, the
// search for superfluous and invalidated runs after every sampling phase, the store that
// cancels a run, and the reactive confidence cutoff.
#include <deque>
#include <new>
#include <vector>

#include "../../include/pipeinfer.h"

namespace {

struct RunRecord {
  int32_t id = 0;
  bool speculative = false;
  std::vector<int32_t> assumed;  // tokens at positions assumed_pos0 .. the run builds on
  int32_t assumed_pos0 = 0;
  std::vector<int32_t> tokens, parent, positions;
  int32_t max_pos = 0;
  int32_t cancelled = 0;  // 0, PI_RUN_SUPERFLUOUS, PI_RUN_INVALIDATED
  volatile int32_t* cancel_word = nullptr;
};

}  // namespace

struct pi_sched {
  double base = 0, recovery = 0, decay = 0, cutoff = 0;
  std::vector<int32_t> accepted;
  std::deque<RunRecord> fifo;
  int32_t next_id = 0;
};

namespace {

// Position method: everything the run can predict is already decided.
bool superfluous(const pi_sched& s, const RunRecord& r) { return r.max_pos < (int32_t)s.accepted.size() - 1; }

// Token method: the tokens the run assumed, then some root-to-node path of its tree, agree
// with the accepted tokens wherever both are defined.
bool follows_accepted(const pi_sched& s, const RunRecord& r) {
  const int32_t A = (int32_t)s.accepted.size();
  for (size_t k = 0; k < r.assumed.size(); ++k) {
    const int64_t p = (int64_t)r.assumed_pos0 + (int64_t)k;
    if (p < A && s.accepted[(size_t)p] != r.assumed[k]) return false;
  }
  const int n = (int)r.tokens.size();
  std::vector<char> alive(n, 0), next(n, 0);
  int32_t level_pos = 0;
  bool any = false;
  for (int i = 0; i < n; ++i)
    if (r.parent[i] < 0) {
      alive[i] = 1;
      level_pos = r.positions[i];
      any = true;
    }
  while (any) {
    if (level_pos >= A) return true;  // beyond the accepted end: nothing to compare with
    bool matched = false;
    for (int i = 0; i < n; ++i) {
      alive[i] = alive[i] && r.tokens[i] == s.accepted[(size_t)level_pos];
      matched = matched || alive[i];
    }
    if (!matched) return false;
    any = false;
    for (int c = 0; c < n; ++c) {
      next[c] = r.parent[c] >= 0 && alive[r.parent[c]];
      any = any || next[c];
    }
    if (!any) return true;  // the matching path ends inside the accepted tokens
    alive.swap(next);
    ++level_pos;
  }
  return true;
}

}  // namespace

extern "C" {

int32_t pi_sched_create(double base_cutoff, double recovery, double decay, pi_sched** out) {
  if (!out) return PI_E_ARG;
  *out = nullptr;
  pi_sched* s = new (std::nothrow) pi_sched();
  if (!s) return PI_E_OOM;
  s->base = s->cutoff = base_cutoff;
  s->recovery = recovery;
  s->decay = decay;
  *out = s;
  return PI_OK;
}

int32_t pi_sched_free(pi_sched* s) {
  if (!s) return PI_E_ARG;
  delete s;
  return PI_OK;
}

int32_t pi_sched_begin_run(pi_sched* s, int32_t speculative, const int32_t* assumed, int32_t n_assumed,
                           int32_t assumed_pos0, const int32_t* tokens, const int32_t* parent,
                           const int32_t* positions, int32_t n, volatile int32_t* cancel_word, int32_t* run_id) {
  if (!s || !tokens || !parent || !positions || !run_id || n_assumed < 0 || (n_assumed > 0 && !assumed)) return PI_E_ARG;
  if (n < 1 || n > PI_MAX_BATCH) return PI_E_SHAPE;
  if (assumed_pos0 < 0) return PI_E_ARG;
  int32_t root_pos = -1;
  for (int i = 0; i < n; ++i) {
    if (positions[i] < 0 || parent[i] < -1 || parent[i] >= i) return PI_E_ARG;
    if (parent[i] < 0) {
      if (root_pos >= 0 && positions[i] != root_pos) return PI_E_ARG;
      root_pos = positions[i];
    } else if (positions[i] != positions[parent[i]] + 1) {
      return PI_E_ARG;
    }
  }
  RunRecord r;
  r.id = s->next_id++;
  r.speculative = speculative != 0;
  r.assumed.assign(assumed, assumed + n_assumed);
  r.assumed_pos0 = assumed_pos0;
  r.tokens.assign(tokens, tokens + n);
  r.parent.assign(parent, parent + n);
  r.positions.assign(positions, positions + n);
  r.max_pos = positions[0];
  for (int i = 1; i < n; ++i) r.max_pos = positions[i] > r.max_pos ? positions[i] : r.max_pos;
  r.cancel_word = cancel_word;
  s->fifo.push_back(std::move(r));
  *run_id = s->fifo.back().id;
  return PI_OK;
}

int32_t pi_sched_accept_tokens(pi_sched* s, const int32_t* tokens, int32_t n, int32_t run_completed, int32_t* ids,
                               int32_t* reasons, int32_t* signalled, int32_t cap, int32_t* n_found) {
  if (!s || n < 0 || (n > 0 && !tokens) || cap < 0 || !n_found) return PI_E_ARG;
  if (cap > 0 && (!ids || !reasons || !signalled)) return PI_E_ARG;
  s->accepted.insert(s->accepted.end(), tokens, tokens + n);
  if (run_completed) s->cutoff = s->base;
  int32_t found = 0;
  for (RunRecord& r : s->fifo) {
    if (r.cancelled) continue;
    if (superfluous(*s, r)) r.cancelled = PI_RUN_SUPERFLUOUS;
    else if (!follows_accepted(*s, r)) r.cancelled = PI_RUN_INVALIDATED;
    if (!r.cancelled) continue;
    if (r.speculative && r.cancel_word) *r.cancel_word = 1;  // the cancellation signal
    if (found < cap) {
      ids[found] = r.id;
      reasons[found] = r.cancelled;
      signalled[found] = r.speculative ? 1 : 0;
    }
    ++found;
  }
  *n_found = found;
  return PI_OK;
}

int32_t pi_sched_complete_run(pi_sched* s, int32_t run_id, int32_t* state) {
  if (!s) return PI_E_ARG;
  for (auto it = s->fifo.begin(); it != s->fifo.end(); ++it)
    if (it->id == run_id) {
      if (state) *state = it->cancelled;
      s->fifo.erase(it);
      return PI_OK;
    }
  return PI_E_ARG;
}

int32_t pi_sched_want_speculation(const pi_sched* s, double confidence, int32_t* yes) {
  if (!s || !yes) return PI_E_ARG;
  *yes = confidence >= s->cutoff ? 1 : 0;
  return PI_OK;
}

int32_t pi_sched_on_speculated(pi_sched* s) {
  if (!s) return PI_E_ARG;
  s->cutoff = s->cutoff + s->recovery;
  return PI_OK;
}

int32_t pi_sched_on_speculation_stopped(pi_sched* s, int32_t logits_waiting) {
  if (!s) return PI_E_ARG;
  if (!logits_waiting) s->cutoff = s->cutoff - s->decay;
  return PI_OK;
}

int32_t pi_sched_state(const pi_sched* s, double* cutoff, int32_t* n_accepted, int32_t* ids, int32_t cap,
                       int32_t* n_runs) {
  if (!s || cap < 0 || (cap > 0 && !ids)) return PI_E_ARG;
  if (cutoff) *cutoff = s->cutoff;
  if (n_accepted) *n_accepted = (int32_t)s->accepted.size();
  int32_t k = 0;
  for (const RunRecord& r : s->fifo) {
    if (k < cap) ids[k] = r.id;
    ++k;
  }
  if (n_runs) *n_runs = k;
  return PI_OK;
}

}  // extern "C"
