"""Continuous asynchronous speculation on one GPU: a driver above the C ABI.

What the paper's head node does (Sections "Asynchronous Speculation", "Continuous Speculation",
"Pipelined KV Cache Multibuffering", "Early Inference Cancellation"), with the one GPU's
stream in the role of the pipeline: verification runs are queued back to back and executed in
order; while the oldest has not finished the head node keeps issuing further micro-batches of
draft tokens, each a run with a sequence partition, a record and a cancel word of its own and
each building on the entries of the one before it; when a result arrives it is sampled
(greedy), the accepted entries join every sequence, and every queued run that the new tokens
contradict is cancelled through its cancel word, which the stage kernel polls at every layer
boundary.  On one GPU several consecutive runs can also share one pass over the weights
(`runs_per_pass` > 1, pi_stage_forward_multi): they stay separate runs in every other respect.

This module only sequences calls: every decision about runs comes from the native
bookkeeping (pi_sched_*), every array is produced by the library's kernels, and nothing is
computed on the host beyond appending tokens to a list.  The draft model is an argument: any
callable position -> (token, confidence).

Token trees (Sections "Speculative Inference / Verification", "Continuous Speculation": trees
build on previous trees): with an `alternative` callable a speculative run is a small tree -- its
chain of draft tokens plus one leaf holding the draft model's second choice for one of the
chain's positions, a sibling of the chain token there.  The leaf hangs at least two positions
above the chain's end, so the chain is the only path of full depth: the next run builds on the
chain's last token and counts exactly when the whole chain was accepted.  Each of the tree's two
branches has a sequence partition of its own; a node belongs to the branches that pass through it.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as pi

_MAX_RUNS = 8       # runs per weight pass the buffers are laid out for
_GS, _RES, _PATH, _OUT = 8, 24, 40, 56   # offsets in a pass's result words: group status, results, paths; size


class _Pass:
    """Device and pinned buffers of one weight pass in flight (reused round robin)."""

    def __init__(self, vocab: int):
        dev, nb = "cuda", pi.PI_MAX_BATCH
        self.tokens = torch.zeros(nb, dtype=torch.int32, device=dev)
        self.positions = torch.zeros(nb, dtype=torch.int32, device=dev)
        self.parent = torch.zeros(nb, dtype=torch.int32, device=dev)     # parent node of each token inside its run
        self.cell_seq = torch.zeros(nb, dtype=torch.int32, device=dev)   # sequences each new entry belongs to
        self.sees_seq = torch.zeros(nb, dtype=torch.int32, device=dev)   # sequences each token reads
        self.slots = torch.zeros(nb, dtype=torch.int32, device=dev)
        self.mask = torch.zeros(nb, dtype=torch.int64, device=dev)
        self.logits = torch.zeros((nb, vocab), dtype=torch.float32, device=dev)
        # [0:2] status of the pass, [2] place status, [3] inexpressible pairs, [_GS + 2k ..] status of run k,
        # [_RES + 2k ..] verification result of run k, [_PATH + first token of run k ..] its accepted path
        self.out = torch.zeros(_OUT, dtype=torch.int32, device=dev)
        self.out_host = torch.zeros(_OUT, dtype=torch.int32, pin_memory=True)
        self.cancel = torch.zeros(_MAX_RUNS, dtype=torch.int32, pin_memory=True)
        self.cancel_dev = pi.mapped_device_pointer(self.cancel)
        self.event = torch.cuda.Event()
        self.h_in = torch.zeros((5, nb), dtype=torch.int32, pin_memory=True)  # tokens, positions, cell_seq, sees_seq, parent
        self.runs = []


class _Run:
    """tokens[0 .. m-1] is the chain (positions start .. start+m-1); an optional last token is the
    alternative for position start + alt_at, a sibling of the chain token there."""

    def __init__(self, speculative, tokens, start, seq, alt=None, alt_at=-1):
        self.speculative, self.start, self.seq = speculative, start, seq
        self.m = len(tokens)
        self.tokens = [int(t) for t in tokens] + ([int(alt)] if alt is not None else [])
        self.n = len(self.tokens)
        self.parent = list(range(-1, self.m - 1)) + ([alt_at - 1] if alt is not None else [])
        self.positions = list(range(start, start + self.m)) + ([start + alt_at] if alt is not None else [])
        self.alt_at = alt_at if alt is not None else -1
        self.seq_alt = 0      # the alternative leaf's partition (a bit), 0 if the run is a chain
        self.id = -1
        self.cancelled = False
        self.pass_ = None
        self.k = 0            # index in its pass
        self.first = 0        # index of its first token in the pass

    def node_seqs(self):
        """Per token the set of partitions it belongs to: the chain's partition, plus the
        alternative's for the chain tokens above the fork; the alternative leaf has its own only."""
        out = [self.seq | (self.seq_alt if i < self.alt_at else 0) for i in range(self.m)]
        return out + ([self.seq_alt] if self.alt_at >= 0 else [])


def _i32(v):
    return int(np.uint32(v).astype(np.int32))


class ContinuousSpeculation:
    """model/kv: the target and its cache, holding `prefix_len` canonical cells (positions
    0 .. prefix_len-1); first_token: the accepted token at position prefix_len whose entry
    is not in the cache yet; draft(pos) -> (token, confidence) for pos > prefix_len.
    depth: weight passes in flight; micro_batch: draft tokens per run (1..4); runs_per_pass:
    consecutive runs sharing one pass over the weights (1 = every run is a pass of its own)."""

    def __init__(self, model, kv, prefix_len: int, first_token: int, draft, depth: int = 3, micro_batch: int = 4,
                 base_cutoff: float = 0.3, recovery: float = 0.05, decay: float = 0.05, n_seq: int = 32,
                 runs_per_pass: int = 1, alternative=None):
        """alternative(pos) -> token or None: the draft model's second choice for position pos; when
        given, runs become trees (chain + one alternative leaf) where there is room."""
        assert 1 <= micro_batch <= 4 and depth >= 1 and 1 <= runs_per_pass <= _MAX_RUNS
        self.model, self.kv, self.draft, self.alternative = model, kv, draft, alternative
        self.depth, self.mb, self.rpp = depth, micro_batch, runs_per_pass
        self.L = model.shape.n_layers
        self.vocab = model.shape.vocab
        self.meta = pi.KVMeta(kv.n_cells, n_seq)
        self.all_seq = (1 << n_seq) - 1
        self.sched = pi.Scheduler(base_cutoff, recovery, decay)
        self.dense = prefix_len                       # canonical cells 0 .. dense-1 are a dense prefix
        self.meta.fill(0, prefix_len, 0, self.all_seq)
        self.accepted = [0] * prefix_len + [int(first_token)]    # prompt tokens are not known here: placeholders
        self.sched.accept_tokens(self.accepted, run_completed=False)
        self.first_generated = prefix_len + 1
        self.free = [_Pass(self.vocab) for _ in range(depth + 2)]
        self.fifo = []                                # passes in flight, oldest first
        self.tail = None                              # last run issued, while the chain it ends is intact
        self.issued_cells = 0                         # window cells handed out since the last compaction
        self.compact_out = torch.zeros(2, dtype=torch.int32, device="cuda")
        self._cutoff_stop = False
        self.stats = {"passes": 0, "runs": 0, "non_speculative": 0, "speculative": 0, "discarded": 0, "cancelled": 0,
                      "layers_skipped": 0, "tokens_speculated": 0, "tokens_accepted_from_drafts": 0, "compactions": 0,
                      "cutoff_stops": 0, "tree_runs": 0, "alternatives_accepted": 0}

    # ---- issuing ---------------------------------------------------------------------------
    def _runs_in_flight(self):
        return [r for p in self.fifo for r in p.runs]

    def _assumed(self, start, extra):
        """Speculated tokens between the accepted end and `start` (what a run at `start` builds
        on): the tokens of the intact chain of runs in flight and of this pass so far."""
        A = len(self.accepted)
        out = []
        for r in self._runs_in_flight() + extra:
            if not r.cancelled:
                for k, t in enumerate(r.tokens[:r.m]):       # the chain: what later runs build on
                    if A <= r.start + k < start:
                        out.append(t)
        return out

    def _plan_pass(self):
        """The runs of the next weight pass: the non-speculative run if nothing in flight covers
        the accepted end, then micro-batches of draft tokens while their confidence clears the
        cutoff (which rises with each one)."""
        runs, n_tok = [], 0
        self._cutoff_stop = False
        last = self.tail
        if last is None:
            runs.append(_Run(False, [self.accepted[-1]], len(self.accepted) - 1, self.all_seq))
            n_tok, last = 1, runs[0]
        while len(runs) < self.rpp and n_tok + 1 <= pi.PI_MAX_BATCH and self.issued_cells + n_tok + 1 <= pi.PI_WINDOW:
            start = last.start + last.m
            batch = []
            room = min(self.mb, pi.PI_MAX_BATCH - n_tok, pi.PI_WINDOW - self.issued_cells - n_tok)
            while len(batch) < room:
                tok, conf = self.draft(start + len(batch))
                if not self.sched.want_speculation(conf):
                    break
                batch.append(int(tok))
            if not batch:
                self._cutoff_stop = room > 0
                self.stats["cutoff_stops"] += 1 if room > 0 else 0
                break
            self.sched.on_speculated()
            alt, alt_at = None, -1
            spare = min(pi.PI_MAX_BATCH - n_tok, pi.PI_WINDOW - self.issued_cells - n_tok) - len(batch)
            if self.alternative is not None and spare >= 1:
                for j in range(len(batch) - 1):      # at least two positions above the chain's end
                    a = self.alternative(start + j)
                    if a is not None and int(a) != batch[j]:
                        alt, alt_at = int(a), j
                        break
            last = _Run(True, batch, start, 0, alt, alt_at)
            runs.append(last)
            n_tok += last.n
        return runs

    def _issue(self, runs):
        if self.dense + pi.PI_WINDOW > self.kv.n_cells:
            raise RuntimeError("KV cache too small: the window [%d, %d) does not fit %d cells"
                               % (self.dense, self.dense + pi.PI_WINDOW, self.kv.n_cells))
        last_pos = max(r.start + r.n - 1 for r in runs)
        if last_pos >= self.model.max_pos:
            raise RuntimeError("position %d reaches the model's rotary table (max_pos %d)" % (last_pos, self.model.max_pos))
        P = self.free.pop()
        P.out.zero_()     # a run whose status word already says "cancelled" stays cancelled: start every pass clean
        n_tot = sum(r.n for r in runs)
        first = 0
        prev = self.tail
        copies = []
        for k, r in enumerate(runs):
            r.pass_, r.k, r.first = P, k, first
            if r.speculative:
                sid = self.meta.acquire()
                assert sid is not None, "out of sequence partitions"
                r.seq = 1 << sid
                if r.alt_at >= 0:
                    sid2 = self.meta.acquire()
                    assert sid2 is not None, "out of sequence partitions"
                    r.seq_alt = 1 << sid2
                    self.stats["tree_runs"] += 1
                if prev is not None and prev.speculative:
                    # early sharing: every branch of this run builds on the chain of the run before
                    copies.append((prev.seq.bit_length() - 1, r.seq | r.seq_alt))
            seqs = np.asarray([_i32(q) for q in r.node_seqs()], dtype=np.int32)
            P.h_in[0, first:first + r.n] = torch.as_tensor(np.asarray(r.tokens, dtype=np.int32))
            P.h_in[1, first:first + r.n] = torch.as_tensor(np.asarray(r.positions, dtype=np.int32))
            P.h_in[2, first:first + r.n] = torch.as_tensor(seqs)
            # a non-speculative run's entry belongs to every sequence at once (it is known to be right),
            # but the run itself reads the canonical sequence only: never another run's speculation
            P.h_in[3, first:first + r.n] = torch.as_tensor(seqs) if r.speculative else 1
            P.h_in[4, first:first + r.n] = torch.as_tensor(np.asarray(r.parent, dtype=np.int32))
            P.cancel[k] = 0
            first += r.n
            prev = r
        for dst, src in ((P.tokens, 0), (P.positions, 1), (P.cell_seq, 2), (P.sees_seq, 3), (P.parent, 4)):
            dst.copy_(P.h_in[src], non_blocking=True)
        self.meta.place(n_tot, P.positions, P.cell_seq, self.dense, P.slots, P.out[2:3])
        for src_id, dst_mask in copies:
            self.meta.seq_cp(src_id, dst_mask)
        self.meta.build_mask(n_tot, P.positions, P.sees_seq, self.dense, self.dense, P.mask, P.out[3:4])
        desc = pi.Run.from_device(n_tot, P.tokens, P.positions, P.slots, P.mask, self.dense, self.dense)
        groups = [k for k, r in enumerate(runs) for _ in range(r.n)]
        # (a non-speculative run is never cancelled -- its entries are what later runs build on --
        # because the bookkeeping never stores into its word)
        pi.stage_forward_multi(self.model, self.kv, desc, groups, 0, self.L, logits_out=P.logits,
                               cancel_flags_ptr=P.cancel_dev, group_status=P.out[_GS:_GS + 2 * len(runs)],
                               run_status=P.out[0:2])
        prev = self.tail
        for k, r in enumerate(runs):
            a, b = r.first, r.first + r.n
            res = P.out[_RES + 2 * k:_RES + 2 * k + 2]
            gst = P.out[_GS + 2 * k:_GS + 2 * k + 2]
            par = P.parent[a:b] if r.alt_at >= 0 else None     # a chain needs no parent array
            if prev is None:
                pi.verify_greedy_chained(P.tokens[a:b], par, r.n, P.logits[a:b], self.vocab, r.tokens[0], None, 0, gst,
                                         P.out[_PATH + a:_PATH + b], res)
            else:
                # the run before counts as accepted whole when its chain was: the chain is its only path of that length
                pres = prev.pass_.out[_RES + 2 * prev.k:_RES + 2 * prev.k + 2]
                pi.verify_greedy_chained(P.tokens[a:b], par, r.n, P.logits[a:b], self.vocab, 0, pres, prev.m, gst,
                                         P.out[_PATH + a:_PATH + b], res)
            if r.speculative:
                self.meta.accept(r.n, P.positions[a:b], P.cell_seq[a:b], P.out[_PATH + a:_PATH + b], res)
            prev = r
        P.out_host.copy_(P.out, non_blocking=True)
        P.event.record()
        done = []
        for k, r in enumerate(runs):
            assumed = self._assumed(r.start, done)
            r.id = self.sched.begin_run(r.speculative, assumed, r.start - len(assumed), r.tokens, r.parent, r.positions,
                                        cancel_word_ptr=P.cancel.data_ptr() + 4 * k)
            done.append(r)
            self.stats["runs"] += 1
            self.stats["speculative" if r.speculative else "non_speculative"] += 1
            if r.speculative:
                self.stats["tokens_speculated"] += r.n
        P.runs = runs
        self.fifo.append(P)
        self.tail = runs[-1]
        self.issued_cells += n_tot
        self.stats["passes"] += 1

    # ---- results ---------------------------------------------------------------------------
    def _process_head(self):
        P = self.fifo.pop(0)
        P.event.synchronize()
        out = P.out_host.numpy()
        if int(out[2]) != pi.PI_OK or int(out[3]) != 0:
            raise RuntimeError("pass: place status %d, %d inexpressible pairs" % (int(out[2]), int(out[3])))
        if int(out[0]) not in (pi.PI_OK, pi.PI_CANCELLED):
            raise pi.PiError(int(out[0]), "stage forward")
        for r in P.runs:
            status, layers_done = int(out[_GS + 2 * r.k]), int(out[_GS + 2 * r.k + 1])
            a, bonus = int(out[_RES + 2 * r.k]), int(out[_RES + 2 * r.k + 1])
            state = self.sched.complete_run(r.id)
            counted = state == 0 and status == pi.PI_OK and a >= 1
            if state != 0:
                self.stats["discarded"] += 1
            if status == pi.PI_CANCELLED:
                self.stats["cancelled"] += 1
                self.stats["layers_skipped"] += self.L - layers_done
            if counted:
                # positions start .. start+a-1 hold the run's accepted tokens (the first of them is
                # the accepted end already), position start+a the target's own token
                path = [int(v) for v in out[_PATH + r.first:_PATH + r.first + a]]
                new = [r.tokens[i] for i in path[1:]] + [bonus]
                assert len(self.accepted) == r.start + 1 and self.accepted[r.start] == r.tokens[path[0]]
                self.accepted += new
                if r.speculative:
                    self.stats["tokens_accepted_from_drafts"] += a
                    if r.alt_at >= 0 and path[-1] == r.n - 1:
                        self.stats["alternatives_accepted"] += 1
                hit = {rid for rid, _, _ in self.sched.accept_tokens(new, run_completed=True)}
                for q in P.runs + self._runs_in_flight():
                    if q.id in hit:
                        q.cancelled = True
            if r.speculative:
                self.meta.release(r.seq.bit_length() - 1)
                if r.seq_alt:
                    self.meta.release(r.seq_alt.bit_length() - 1)
        # the chain can be continued only while its last run is in flight and still stands (a
        # rejected token takes every run built on it along, so the last run tells)
        if self.tail is not None and (self.tail.pass_ is P or self.tail.cancelled):
            self.tail = None
        P.runs = []
        self.free.append(P)

    def _compact(self):
        assert not self.fifo
        self.meta.compact(self.kv, self.dense, self.compact_out)
        st, dense = self.compact_out.cpu().tolist()
        if st != pi.PI_OK:
            raise pi.PiError(st, "pi_kvmeta_compact")
        self.dense, self.issued_cells, self.tail = dense, 0, None
        self.stats["compactions"] += 1

    # ---- the loop ----------------------------------------------------------------------------
    def generate(self, n_tokens: int):
        """Run until n_tokens have been generated after first_token; returns them."""
        goal = self.first_generated + n_tokens
        while len(self.accepted) < goal:
            if self.fifo and self.fifo[0].event.query():
                self._process_head()                       # logits are waiting: sample and verify
                continue
            if not self.fifo and self.issued_cells + 2 + self.mb > pi.PI_WINDOW:
                self._compact()
                continue
            if len(self.fifo) < self.depth and self.free and self.issued_cells + 1 <= pi.PI_WINDOW:
                runs = self._plan_pass()
                if runs:
                    self._issue(runs)
                    continue
                if self._cutoff_stop:                      # speculation stopped for lack of confidence: one decay per stop
                    waiting = bool(self.fifo) and self.fifo[0].event.query()
                    self.sched.on_speculation_stopped(waiting)
                    if not self.fifo:
                        continue                           # idle: the cutoff decays until speculation resumes
            if self.fifo:
                self._process_head()                       # nothing to issue: wait for the oldest pass
        while self.fifo:
            self._process_head()
        torch.cuda.synchronize()
        return self.accepted[self.first_generated:goal]

    def close(self):
        self.meta.free()
        self.sched.free()
