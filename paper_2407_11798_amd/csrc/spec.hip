// Continuous asynchronous speculation on one GPU: the head node's loop behind the C ABI.
//
// What the paper's head node does (Sections "Asynchronous Speculation", "Continuous Speculation",
// "Pipelined KV Cache Multibuffering", "Early Inference Cancellation"), with the one GPU's stream in
// the role of the pipeline: verification runs are queued back to back and executed in order; while
// the oldest has not finished the head node keeps issuing further micro-batches of draft tokens,
// each a run with a sequence partition, a record and a cancel word of its own and each building on
// the entries of the one before it; when a result arrives it is sampled (greedy), the accepted
// entries join every sequence, and every queued run that the new tokens contradict is cancelled
// through its cancel word, which the stage kernel polls at every layer boundary.  Several
// consecutive runs can share one pass over the weights (pi_stage_forward_multi).
//
// Host code only: it sequences the library's own entry points (pi_sched_*, pi_kvmeta_*,
// pi_stage_forward_multi, pi_verify_greedy_chained) on one stream; every decision about runs comes
// from the run bookkeeping, every array is produced by the library's kernels.
#include <algorithm>
#include <cstring>
#include <deque>
#include <memory>
#include <new>
#include <vector>

#include "pi_internal.h"

namespace {

constexpr int kMaxRuns = 8;  // runs per weight pass the buffers are laid out for
// offsets in a pass's result words: [0:2] status of the pass, [2] place status, [3] inexpressible
// pairs, [kGS + 2k ..] status of run k, [kRES + 2k ..] verification result of run k,
// [kPATH + first token of run k ..] its accepted path
constexpr int kGS = 8, kRES = 24, kPATH = 40, kOUT = 56;

struct Pass;

// tokens[0 .. m-1] is the chain (positions start .. start+m-1); an optional last token is the
// alternative for position start + alt_at, a sibling of the chain token there.
struct Run {
  bool speculative = false;
  int start = 0, m = 0, n = 0, alt_at = -1;
  std::vector<int32_t> tokens, parent, positions;
  uint32_t seq = 0, seq_alt = 0;  // the chain's partition (a bit) and the alternative leaf's
  int32_t id = -1;
  bool cancelled = false;
  Pass* pass = nullptr;
  int k = 0, first = 0;  // index in its pass; index of its first token in the pass

  Run(bool spec, const std::vector<int32_t>& chain, int start_, uint32_t seq_, bool has_alt, int32_t alt, int alt_at_)
      : speculative(spec), start(start_), m((int)chain.size()), alt_at(has_alt ? alt_at_ : -1), tokens(chain), seq(seq_) {
    for (int i = 0; i < m; ++i) {
      parent.push_back(i - 1);
      positions.push_back(start + i);
    }
    if (has_alt) {
      tokens.push_back(alt);
      parent.push_back(alt_at_ - 1);
      positions.push_back(start + alt_at_);
    }
    n = (int)tokens.size();
  }
  // per token the partitions it belongs to: the chain's, plus the alternative's for the chain tokens
  // above the fork; the alternative leaf has its own only
  uint32_t node_seq(int i) const {
    if (i < m) return seq | (i < alt_at ? seq_alt : 0u);
    return seq_alt;
  }
};

struct Pass {
  int32_t *tokens = nullptr, *positions = nullptr, *parent = nullptr, *slots = nullptr, *out = nullptr;
  uint32_t *cell_seq = nullptr, *sees_seq = nullptr;
  uint64_t* mask = nullptr;
  float* logits = nullptr;
  int32_t* out_host = nullptr;      // pinned
  int32_t* cancel = nullptr;        // pinned + mapped: the runs' cancel words
  int32_t* cancel_dev = nullptr;    // the same words as the device sees them
  int32_t* h_in = nullptr;          // pinned [5][PI_MAX_BATCH]: tokens, positions, cell_seq, sees_seq, parent
  hipEvent_t event = nullptr;
  std::vector<std::shared_ptr<Run>> runs;
};

}  // namespace

struct pi_spec {
  pi_model* model = nullptr;
  pi_kv* kv = nullptr;
  pi_kvmeta* meta = nullptr;
  pi_sched* sched = nullptr;
  hipStream_t stream = nullptr;
  pi_spec_config cfg{};
  int L = 0, vocab = 0, max_pos = 0, n_cells = 0;
  uint32_t all_seq = 0;
  int dense = 0;                   // canonical cells 0 .. dense-1 are a dense prefix
  std::vector<int32_t> accepted;   // prompt tokens are not known here: placeholders
  int first_generated = 0;
  std::vector<Pass*> all_passes, free_passes;
  std::deque<Pass*> fifo;          // passes in flight, oldest first
  std::shared_ptr<Run> tail;       // last run issued, while the chain it ends is intact
  int issued_cells = 0;            // window cells handed out since the last compaction
  int32_t* compact_out = nullptr;  // device int32[2]
  bool cutoff_stop = false;
  pi_spec_stats stats{};
  int32_t error = PI_OK;           // first error met inside the loop
};

namespace {

#define SPEC_TRY(call)              \
  do {                              \
    const int32_t st__ = (call);    \
    if (st__ != PI_OK) return st__; \
  } while (0)

int32_t hip_st(hipError_t e) { return e == hipSuccess ? PI_OK : (e == hipErrorOutOfMemory ? PI_E_OOM : PI_E_HIP); }

void free_pass(Pass* p) {
  if (!p) return;
  for (void* d : {(void*)p->tokens, (void*)p->positions, (void*)p->parent, (void*)p->slots, (void*)p->out,
                  (void*)p->cell_seq, (void*)p->sees_seq, (void*)p->mask, (void*)p->logits})
    if (d) (void)hipFree(d);
  for (void* h : {(void*)p->out_host, (void*)p->cancel, (void*)p->h_in})
    if (h) (void)hipHostFree(h);
  if (p->event) (void)hipEventDestroy(p->event);
  delete p;
}

int32_t make_pass(int vocab, Pass** out) {
  Pass* p = new (std::nothrow) Pass();
  if (!p) return PI_E_OOM;
  const size_t nb = PI_MAX_BATCH;
  hipError_t e = hipMalloc((void**)&p->tokens, nb * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&p->positions, nb * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&p->parent, nb * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&p->slots, nb * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&p->cell_seq, nb * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&p->sees_seq, nb * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&p->mask, nb * 8);
  if (e == hipSuccess) e = hipMalloc((void**)&p->logits, nb * (size_t)vocab * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&p->out, kOUT * 4);
  if (e == hipSuccess) e = hipMemset(p->out, 0, kOUT * 4);
  if (e == hipSuccess) e = hipHostMalloc((void**)&p->out_host, kOUT * 4, hipHostMallocDefault);
  if (e == hipSuccess) e = hipHostMalloc((void**)&p->cancel, kMaxRuns * 4, hipHostMallocMapped);
  if (e == hipSuccess) e = hipHostMalloc((void**)&p->h_in, 5 * nb * 4, hipHostMallocDefault);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&p->event, hipEventDisableTiming);
  if (e == hipSuccess) {
    memset(p->cancel, 0, kMaxRuns * 4);
    memset(p->h_in, 0, 5 * nb * 4);
    void* dev = nullptr;
    const int32_t st = pi_mapped_device_pointer(p->cancel, &dev);
    if (st != PI_OK) {
      free_pass(p);
      return st;
    }
    p->cancel_dev = (int32_t*)dev;
  }
  if (e != hipSuccess) {
    free_pass(p);
    return hip_st(e);
  }
  *out = p;
  return PI_OK;
}

// Speculated tokens between the accepted end and `start` (what a run at `start` builds on): the
// tokens of the intact chain of runs in flight and of this pass so far.
std::vector<int32_t> assumed_tokens(const pi_spec* s, int start, const std::vector<std::shared_ptr<Run>>& extra) {
  const int A = (int)s->accepted.size();
  std::vector<int32_t> out;
  const auto take = [&](const Run& r) {
    if (r.cancelled) return;
    for (int k = 0; k < r.m; ++k)  // the chain: what later runs build on
      if (A <= r.start + k && r.start + k < start) out.push_back(r.tokens[k]);
  };
  for (const Pass* p : s->fifo)
    for (const auto& r : p->runs) take(*r);
  for (const auto& r : extra) take(*r);
  return out;
}

// The runs of the next weight pass: the non-speculative run if nothing in flight covers the accepted
// end, then micro-batches of draft tokens while their confidence clears the cutoff (which rises with
// each one).
int32_t plan_pass(pi_spec* s, std::vector<std::shared_ptr<Run>>* runs) {
  int n_tok = 0;
  s->cutoff_stop = false;
  std::shared_ptr<Run> last = s->tail;
  if (!last) {
    // Nothing to build on.  If a run in flight that still stands has a node at the accepted end (a tree
    // whose alternative leaf continues the accepted tokens where its chain does not), that run will
    // supply the entry of the accepted end and the token after it: wait for it.  A non-speculative run
    // for the same position would put a second canonical entry there.
    const int end_pos = (int)s->accepted.size() - 1;
    for (const Pass* p : s->fifo)
      for (const auto& r : p->runs)
        if (!r->cancelled)
          for (int i = 0; i < r->n; ++i)
            if (r->positions[i] == end_pos) return PI_OK;
    last = std::make_shared<Run>(false, std::vector<int32_t>{s->accepted.back()}, (int)s->accepted.size() - 1, s->all_seq,
                                 false, 0, -1);
    runs->push_back(last);
    n_tok = 1;
  }
  const int rpp = s->cfg.runs_per_pass, mb = s->cfg.micro_batch;
  while ((int)runs->size() < rpp && n_tok + 1 <= PI_MAX_BATCH && s->issued_cells + n_tok + 1 <= PI_WINDOW) {
    const int start = last->start + last->m;
    std::vector<int32_t> batch;
    const int room = std::min({mb, PI_MAX_BATCH - n_tok, PI_WINDOW - s->issued_cells - n_tok});
    while ((int)batch.size() < room) {
      int32_t tok = 0, yes = 0;
      double conf = 0.0;
      SPEC_TRY(s->cfg.draft(s->cfg.ctx, start + (int)batch.size(), &tok, &conf));
      SPEC_TRY(pi_sched_want_speculation(s->sched, conf, &yes));
      if (!yes) break;
      batch.push_back(tok);
    }
    if (batch.empty()) {
      s->cutoff_stop = room > 0;
      s->stats.cutoff_stops += room > 0 ? 1 : 0;
      break;
    }
    SPEC_TRY(pi_sched_on_speculated(s->sched));
    bool has_alt = false;
    int32_t alt = 0;
    int alt_at = -1;
    const int spare = std::min(PI_MAX_BATCH - n_tok, PI_WINDOW - s->issued_cells - n_tok) - (int)batch.size();
    if (s->cfg.alternative && spare >= 1) {
      for (int j = 0; j + 1 < (int)batch.size(); ++j) {  // at least two positions above the chain's end
        int32_t a = 0;
        const int32_t got = s->cfg.alternative(s->cfg.ctx, start + j, &a);
        if (got < 0) return got;
        if (got > 0 && a != batch[j]) {
          has_alt = true;
          alt = a;
          alt_at = j;
          break;
        }
      }
    }
    last = std::make_shared<Run>(true, batch, start, 0u, has_alt, alt, alt_at);
    runs->push_back(last);
    n_tok += last->n;
  }
  return PI_OK;
}

int32_t issue(pi_spec* s, const std::vector<std::shared_ptr<Run>>& runs) {
  if (s->dense + PI_WINDOW > s->n_cells) return PI_E_SHAPE;  // the window does not fit the cache
  int last_pos = 0;
  for (const auto& r : runs) last_pos = std::max(last_pos, r->start + r->n - 1);
  if (last_pos >= s->max_pos) return PI_E_ARG;  // a position reaches the model's rotary table
  Pass* P = s->free_passes.back();
  s->free_passes.pop_back();
  hipStream_t st = s->stream;
  // a run whose status word already says "cancelled" stays cancelled: start every pass clean
  hipError_t e = hipMemsetAsync(P->out, 0, kOUT * 4, st);
  if (e != hipSuccess) return hip_st(e);
  const int nb = PI_MAX_BATCH;
  int n_tot = 0, first = 0;
  for (const auto& r : runs) n_tot += r->n;
  std::shared_ptr<Run> prev = s->tail;
  std::vector<std::pair<int, uint32_t>> copies;
  int32_t group_of_token[PI_MAX_BATCH];
  for (int k = 0; k < (int)runs.size(); ++k) {
    Run& r = *runs[k];
    r.pass = P;
    r.k = k;
    r.first = first;
    if (r.speculative) {
      int32_t sid = 0;
      SPEC_TRY(pi_kvmeta_seq_acquire(s->meta, &sid));  // PI_E_FULL: out of sequence partitions
      r.seq = 1u << sid;
      if (r.alt_at >= 0) {
        int32_t sid2 = 0;
        SPEC_TRY(pi_kvmeta_seq_acquire(s->meta, &sid2));
        r.seq_alt = 1u << sid2;
        s->stats.tree_runs += 1;
      }
      if (prev && prev->speculative) {
        // early sharing: every branch of this run builds on the chain of the run before
        int src = 0;
        while (!((prev->seq >> src) & 1u)) ++src;
        copies.emplace_back(src, r.seq | r.seq_alt);
      }
    }
    for (int i = 0; i < r.n; ++i) {
      const uint32_t q = r.node_seq(i);
      P->h_in[0 * nb + first + i] = r.tokens[i];
      P->h_in[1 * nb + first + i] = r.positions[i];
      P->h_in[2 * nb + first + i] = (int32_t)q;
      // a non-speculative run's entry belongs to every sequence at once (it is known to be right),
      // but the run itself reads the canonical sequence only: never another run's speculation
      P->h_in[3 * nb + first + i] = r.speculative ? (int32_t)q : 1;
      P->h_in[4 * nb + first + i] = r.parent[i];
      group_of_token[first + i] = k;
    }
    P->cancel[k] = 0;
    first += r.n;
    prev = runs[k];
  }
  void* dsts[5] = {P->tokens, P->positions, P->cell_seq, P->sees_seq, P->parent};
  for (int j = 0; j < 5; ++j) {
    e = hipMemcpyAsync(dsts[j], P->h_in + j * nb, nb * 4, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return hip_st(e);
  }
  SPEC_TRY(pi_kvmeta_place(s->meta, n_tot, P->positions, P->cell_seq, s->dense, P->slots, P->out + 2, st));
  for (const auto& c : copies) SPEC_TRY(pi_kvmeta_seq_cp(s->meta, c.first, c.second, 0, PI_POS_MAX, st));
  SPEC_TRY(pi_kvmeta_build_mask(s->meta, n_tot, P->positions, P->sees_seq, s->dense, s->dense, P->mask, P->out + 3, st));
  pi_run_desc desc;
  desc.n = n_tot;
  desc.tokens = P->tokens;
  desc.positions = P->positions;
  desc.slots = P->slots;
  desc.mask = P->mask;
  desc.prefix_len = s->dense;
  desc.window_base = s->dense;
  pi_group_desc groups;
  groups.n_groups = (int)runs.size();
  groups.group_of_token = group_of_token;
  // (a non-speculative run is never cancelled -- its entries are what later runs build on -- because
  // the bookkeeping never stores into its word)
  groups.cancel_flags = P->cancel_dev;
  groups.group_status = P->out + kGS;
  SPEC_TRY(pi_stage_forward_multi(s->model, s->kv, &desc, &groups, 0, s->L, nullptr, nullptr, P->logits, P->out, st));
  prev = s->tail;
  for (int k = 0; k < (int)runs.size(); ++k) {
    const Run& r = *runs[k];
    const int a = r.first;
    int32_t* res = P->out + kRES + 2 * k;
    const int32_t* gst = P->out + kGS + 2 * k;
    const int32_t* par = r.alt_at >= 0 ? P->parent + a : nullptr;  // a chain needs no parent array
    if (!prev) {
      SPEC_TRY(pi_verify_greedy_chained(P->tokens + a, par, r.n, P->logits + (size_t)a * s->vocab, s->vocab, r.tokens[0],
                                        nullptr, 0, gst, P->out + kPATH + a, res, st));
    } else {
      // the run before counts as accepted whole when its chain was: the chain is its only path of that length
      const int32_t* pres = prev->pass->out + kRES + 2 * prev->k;
      SPEC_TRY(pi_verify_greedy_chained(P->tokens + a, par, r.n, P->logits + (size_t)a * s->vocab, s->vocab, 0, pres, prev->m,
                                        gst, P->out + kPATH + a, res, st));
    }
    if (r.speculative)
      SPEC_TRY(pi_kvmeta_accept(s->meta, r.n, P->positions + a, P->cell_seq + a, P->out + kPATH + a, res, st));
    prev = runs[k];
  }
  e = hipMemcpyAsync(P->out_host, P->out, kOUT * 4, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipEventRecord(P->event, st);
  if (e != hipSuccess) return hip_st(e);
  std::vector<std::shared_ptr<Run>> done;
  for (int k = 0; k < (int)runs.size(); ++k) {
    Run& r = *runs[k];
    const std::vector<int32_t> assumed = assumed_tokens(s, r.start, done);
    SPEC_TRY(pi_sched_begin_run(s->sched, r.speculative ? 1 : 0, assumed.empty() ? nullptr : assumed.data(), (int)assumed.size(),
                                r.start - (int)assumed.size(), r.tokens.data(), r.parent.data(), r.positions.data(), r.n,
                                P->cancel + k, &r.id));
    done.push_back(runs[k]);
    s->stats.runs += 1;
    (r.speculative ? s->stats.speculative : s->stats.non_speculative) += 1;
    if (r.speculative) s->stats.tokens_speculated += r.n;
  }
  P->runs = runs;
  s->fifo.push_back(P);
  s->tail = runs.back();
  s->issued_cells += n_tot;
  s->stats.passes += 1;
  return PI_OK;
}

int32_t process_head(pi_spec* s) {
  Pass* P = s->fifo.front();
  s->fifo.pop_front();
  hipError_t e = hipEventSynchronize(P->event);
  if (e != hipSuccess) return hip_st(e);
  const int32_t* out = P->out_host;
  if (out[2] != PI_OK) return out[2];  // the window had no room for the pass's entries
  if (out[3] != 0) return PI_E_STATE;  // the mask form could not express what the metadata says
  if (out[0] != PI_OK && out[0] != PI_CANCELLED) return out[0];
  for (const auto& rp : P->runs) {
    Run& r = *rp;
    const int32_t status = out[kGS + 2 * r.k], layers_done = out[kGS + 2 * r.k + 1];
    const int32_t a = out[kRES + 2 * r.k], bonus = out[kRES + 2 * r.k + 1];
    int32_t state = 0;
    SPEC_TRY(pi_sched_complete_run(s->sched, r.id, &state));
    const bool counted = state == 0 && status == PI_OK && a >= 1;
    if (state != 0) s->stats.discarded += 1;
    if (status == PI_CANCELLED) {
      s->stats.cancelled += 1;
      s->stats.layers_skipped += s->L - layers_done;
    }
    if (counted) {
      // positions start .. start+a-1 hold the run's accepted tokens (the first of them is the accepted
      // end already), position start+a the target's own token
      const int32_t* path = out + kPATH + r.first;
      if ((int)s->accepted.size() != r.start + 1 || path[0] < 0 || path[0] >= r.n || s->accepted[r.start] != r.tokens[path[0]])
        return PI_E_STATE;
      std::vector<int32_t> fresh;
      for (int i = 1; i < a; ++i) {
        if (path[i] < 0 || path[i] >= r.n) return PI_E_STATE;
        fresh.push_back(r.tokens[path[i]]);
      }
      fresh.push_back(bonus);
      s->accepted.insert(s->accepted.end(), fresh.begin(), fresh.end());
      if (r.speculative) {
        s->stats.tokens_accepted_from_drafts += a;
        if (r.alt_at >= 0 && path[a - 1] == r.n - 1) s->stats.alternatives_accepted += 1;
      }
      int32_t ids[64], reasons[64], signalled[64], found = 0;
      SPEC_TRY(pi_sched_accept_tokens(s->sched, fresh.data(), (int)fresh.size(), 1, ids, reasons, signalled, 64, &found));
      const int nf = std::min(found, 64);
      const auto mark = [&](Run& q) {
        for (int j = 0; j < nf; ++j)
          if (ids[j] == q.id) q.cancelled = true;
      };
      for (const auto& q : P->runs) mark(*q);
      for (Pass* p2 : s->fifo)
        for (const auto& q : p2->runs) mark(*q);
    }
    if (r.speculative) {
      for (uint32_t bits : {r.seq, r.seq_alt}) {
        if (!bits) continue;
        int sid = 0;
        while (!((bits >> sid) & 1u)) ++sid;
        SPEC_TRY(pi_kvmeta_seq_release(s->meta, sid, s->stream));
      }
    }
  }
  // the chain can be continued only while its last run is in flight and still stands (a rejected token
  // takes every run built on it along, so the last run tells)
  if (s->tail && (s->tail->pass == P || s->tail->cancelled)) s->tail.reset();
  P->runs.clear();
  s->free_passes.push_back(P);
  return PI_OK;
}

int32_t compact(pi_spec* s) {
  SPEC_TRY(pi_kvmeta_compact(s->meta, s->kv, s->dense, s->compact_out, s->stream));
  int32_t r[2] = {0, 0};
  hipError_t e = hipMemcpyAsync(r, s->compact_out, 8, hipMemcpyDeviceToHost, s->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(s->stream);
  if (e != hipSuccess) return hip_st(e);
  if (r[0] != PI_OK) return r[0];
  s->dense = r[1];
  s->issued_cells = 0;
  s->tail.reset();
  s->stats.compactions += 1;
  return PI_OK;
}

bool head_ready(const pi_spec* s) { return !s->fifo.empty() && hipEventQuery(s->fifo.front()->event) == hipSuccess; }

}  // namespace

extern "C" {

int32_t pi_spec_create(pi_model* model, pi_kv* kv, const pi_spec_config* cfg, void* stream, pi_spec** out) {
  if (!model || !kv || !cfg || !out || !cfg->draft) return PI_E_ARG;
  *out = nullptr;
  if (cfg->micro_batch < 1 || cfg->micro_batch > 4 || cfg->depth < 1 || cfg->depth > 16 || cfg->runs_per_pass < 1 ||
      cfg->runs_per_pass > kMaxRuns || cfg->n_seq < 2 || cfg->n_seq > PI_MAX_SEQ || cfg->prefix_len < 0)
    return PI_E_ARG;
  const pi::ModelView mv = pi::model_view(model);
  const pi::KvView kvv = pi::kv_view(kv);
  if (cfg->prefix_len + PI_WINDOW > kvv.n_cells) return PI_E_SHAPE;
  pi_spec* s = new (std::nothrow) pi_spec();
  if (!s) return PI_E_OOM;
  s->model = model;
  s->kv = kv;
  s->stream = (hipStream_t)stream;
  s->cfg = *cfg;
  s->L = mv.n_layers;
  s->vocab = mv.vocab;
  s->max_pos = mv.max_pos;
  s->n_cells = kvv.n_cells;
  s->all_seq = cfg->n_seq >= 32 ? 0xffffffffu : (1u << cfg->n_seq) - 1u;
  s->dense = cfg->prefix_len;
  int32_t st = pi_kvmeta_alloc(kvv.n_cells, cfg->n_seq, &s->meta);
  if (st == PI_OK) st = pi_sched_create(cfg->base_cutoff, cfg->recovery, cfg->decay, &s->sched);
  if (st == PI_OK) st = pi_kvmeta_fill(s->meta, 0, cfg->prefix_len, 0, s->all_seq, stream);
  if (st == PI_OK) {
    s->accepted.assign((size_t)cfg->prefix_len, 0);
    s->accepted.push_back(cfg->first_token);
    int32_t ids[64], reasons[64], signalled[64], found = 0;
    st = pi_sched_accept_tokens(s->sched, s->accepted.data(), (int)s->accepted.size(), 0, ids, reasons, signalled, 64, &found);
    s->first_generated = cfg->prefix_len + 1;
  }
  for (int i = 0; st == PI_OK && i < cfg->depth + 2; ++i) {
    Pass* p = nullptr;
    st = make_pass(s->vocab, &p);
    if (st == PI_OK) {
      s->all_passes.push_back(p);
      s->free_passes.push_back(p);
    }
  }
  if (st == PI_OK) st = hip_st(hipMalloc((void**)&s->compact_out, 8));
  if (st != PI_OK) {
    pi_spec_free(s);
    return st;
  }
  *out = s;
  return PI_OK;
}

int32_t pi_spec_generate(pi_spec* s, int32_t n_tokens, int32_t* tokens_out) {
  if (!s || n_tokens < 0 || (n_tokens > 0 && !tokens_out)) return PI_E_ARG;
  if (s->error != PI_OK) return s->error;
  const size_t goal = (size_t)s->first_generated + (size_t)n_tokens;
  const auto fail = [&](int32_t st) {
    s->error = st;
    (void)hipStreamSynchronize(s->stream);
    return st;
  };
  while (s->accepted.size() < goal) {
    int32_t st = PI_OK;
    if (head_ready(s)) {  // logits are waiting: sample and verify
      if ((st = process_head(s)) != PI_OK) return fail(st);
      continue;
    }
    if (s->fifo.empty() && s->issued_cells + 2 + s->cfg.micro_batch > PI_WINDOW) {
      if ((st = compact(s)) != PI_OK) return fail(st);
      continue;
    }
    if ((int)s->fifo.size() < s->cfg.depth && !s->free_passes.empty() && s->issued_cells + 1 <= PI_WINDOW) {
      std::vector<std::shared_ptr<Run>> runs;
      if ((st = plan_pass(s, &runs)) != PI_OK) return fail(st);
      if (!runs.empty()) {
        if ((st = issue(s, runs)) != PI_OK) return fail(st);
        continue;
      }
      if (s->cutoff_stop) {  // speculation stopped for lack of confidence: one decay per stop
        if ((st = pi_sched_on_speculation_stopped(s->sched, head_ready(s) ? 1 : 0)) != PI_OK) return fail(st);
        if (s->fifo.empty()) continue;  // idle: the cutoff decays until speculation resumes
      }
    }
    if (!s->fifo.empty() && (st = process_head(s)) != PI_OK) return fail(st);  // nothing to issue: wait for the oldest pass
  }
  while (!s->fifo.empty()) {
    const int32_t st = process_head(s);
    if (st != PI_OK) return fail(st);
  }
  const hipError_t e = hipStreamSynchronize(s->stream);
  if (e != hipSuccess) return fail(hip_st(e));
  for (int32_t i = 0; i < n_tokens; ++i) tokens_out[i] = s->accepted[(size_t)s->first_generated + i];
  return PI_OK;
}

int32_t pi_spec_settle(pi_spec* s, int32_t* n_accepted, int32_t* dense_len) {
  if (!s) return PI_E_ARG;
  if (s->error != PI_OK) return s->error;
  while (!s->fifo.empty()) {
    const int32_t st = process_head(s);
    if (st != PI_OK) return s->error = st;
  }
  const int32_t st = compact(s);
  if (st != PI_OK) return s->error = st;
  if (n_accepted) *n_accepted = (int32_t)s->accepted.size();
  if (dense_len) *dense_len = s->dense;
  return PI_OK;
}

int32_t pi_spec_read_cells(const pi_spec* s, int32_t* pos_host, uint32_t* seq_host) {
  if (!s) return PI_E_ARG;
  return pi_kvmeta_read(s->meta, pos_host, seq_host);
}

int32_t pi_spec_get_stats(const pi_spec* s, pi_spec_stats* out) {
  if (!s || !out) return PI_E_ARG;
  *out = s->stats;
  return PI_OK;
}

int32_t pi_spec_free(pi_spec* s) {
  if (!s) return PI_E_ARG;
  (void)hipStreamSynchronize(s->stream);
  for (Pass* p : s->all_passes) free_pass(p);
  if (s->compact_out) (void)hipFree(s->compact_out);
  if (s->meta) (void)pi_kvmeta_free(s->meta);
  if (s->sched) (void)pi_sched_free(s->sched);
  delete s;
  return PI_OK;
}

}  // extern "C"
