"""Continuous asynchronous speculation on one GPU: a driver above the C ABI.

What the paper's head node does (Sections "Asynchronous Speculation", "Continuous Speculation",
"Pipelined KV Cache Multibuffering", "Early Inference Cancellation"), with the one GPU's
stream in the role of the pipeline: verification runs are queued back to back and executed in
order; while the oldest has not finished the head node keeps issuing further micro-batches of
draft tokens, each in a sequence partition of its own and each building on the entries of the
one before it; when a result arrives it is sampled (greedy), the accepted entries join every
sequence, and every queued run that the new tokens contradict is cancelled through its cancel
word, which the stage kernel polls at every layer boundary.

This module only sequences calls: every decision about runs comes from the native
bookkeeping (pi_sched_*), every array is produced by the library's kernels, and nothing is
computed on the host beyond appending tokens to a list.  The draft model is an argument: any
callable position -> (token, confidence).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as pi


class _Slot:
    """Device and pinned buffers of one run in flight (reused round robin)."""

    def __init__(self, vocab: int, mb: int):
        dev = "cuda"
        self.tokens = torch.zeros(mb, dtype=torch.int32, device=dev)
        self.positions = torch.zeros(mb, dtype=torch.int32, device=dev)
        self.tok_seq = torch.zeros(mb, dtype=torch.int32, device=dev)
        self.slots = torch.zeros(mb, dtype=torch.int32, device=dev)
        self.mask = torch.zeros(mb, dtype=torch.int64, device=dev)
        self.logits = torch.zeros((mb, vocab), dtype=torch.float32, device=dev)
        # [0:2] run_status, [2:4] verification result, [4] place status, [5] inexpressible pairs, [8:8+mb] path
        self.out = torch.zeros(8 + mb, dtype=torch.int32, device=dev)
        self.out_host = torch.zeros(8 + mb, dtype=torch.int32, pin_memory=True)
        self.cancel = torch.zeros(1, dtype=torch.int32, pin_memory=True)
        self.cancel_dev = pi.mapped_device_pointer(self.cancel)
        self.event = torch.cuda.Event()
        self.h_tokens = torch.zeros(mb, dtype=torch.int32, pin_memory=True)
        self.h_positions = torch.zeros(mb, dtype=torch.int32, pin_memory=True)
        self.h_seq = torch.zeros(mb, dtype=torch.int32, pin_memory=True)
        self.canonical_only = torch.ones(mb, dtype=torch.int32, device=dev)      # sequence 0 alone


class _Run:
    def __init__(self, rid, slot, speculative, tokens, start, seq):
        self.id, self.slot, self.speculative = rid, slot, speculative
        self.tokens, self.start, self.seq = tokens, start, seq
        self.n = len(tokens)
        self.cancelled = False


class ContinuousSpeculation:
    """model/kv: the target and its cache, holding `prefix_len` canonical cells (positions
    0 .. prefix_len-1); first_token: the accepted token at position prefix_len whose entry
    is not in the cache yet; draft(pos) -> (token, confidence) for pos > prefix_len."""

    def __init__(self, model, kv, prefix_len: int, first_token: int, draft, depth: int = 3, micro_batch: int = 4,
                 base_cutoff: float = 0.3, recovery: float = 0.05, decay: float = 0.05, n_seq: int = 32):
        assert 1 <= micro_batch <= 4 and depth >= 1
        self.model, self.kv, self.draft = model, kv, draft
        self.depth, self.mb = depth, micro_batch
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
        self.free_slots = [_Slot(self.vocab, micro_batch) for _ in range(depth + 3)]
        self.fifo = []                                # runs in flight, oldest first
        self.tail = None                              # last run issued, while the chain it ends is intact
        self.issued_cells = 0                         # window cells handed out since the last compaction
        self.compact_out = torch.zeros(2, dtype=torch.int32, device="cuda")
        self.stats = {"runs": 0, "non_speculative": 0, "speculative": 0, "discarded": 0, "cancelled": 0, "layers_skipped": 0,
                      "tokens_speculated": 0, "tokens_accepted_from_drafts": 0, "compactions": 0, "cutoff_stops": 0}

    # ---- issuing ---------------------------------------------------------------------------
    def _issue(self, tokens, start, speculative):
        n = len(tokens)
        slot = self.free_slots.pop()
        prev = self.tail
        seq = self.all_seq
        if speculative:
            sid = self.meta.acquire()
            assert sid is not None, "out of sequence partitions"
            seq = 1 << sid
            if prev is not None and prev.speculative:
                self.meta.seq_cp(prev.seq.bit_length() - 1, seq)      # early sharing: build on the run before
        slot.h_tokens[:n] = torch.as_tensor(np.asarray(tokens, dtype=np.int32))
        slot.h_positions[:n] = torch.arange(start, start + n, dtype=torch.int32)
        slot.h_seq[:n] = int(np.uint32(seq).astype(np.int32))
        slot.tokens.copy_(slot.h_tokens, non_blocking=True)
        slot.positions.copy_(slot.h_positions, non_blocking=True)
        slot.tok_seq.copy_(slot.h_seq, non_blocking=True)
        slot.cancel[0] = 0
        self.meta.place(n, slot.positions, slot.tok_seq, self.dense, slot.slots, slot.out[4:5])
        # a non-speculative run's entry belongs to every sequence at once (it is known to be right),
        # but the run itself reads the canonical sequence only: never another run's speculation
        sees = slot.tok_seq if speculative else slot.canonical_only
        self.meta.build_mask(n, slot.positions, sees, self.dense, self.dense, slot.mask, slot.out[5:6])
        run_desc = pi.Run.__new__(pi.Run)
        run_desc.n, run_desc.tokens, run_desc.positions = n, slot.tokens, slot.positions
        run_desc.slots, run_desc.mask, run_desc.parent = slot.slots, slot.mask, None
        run_desc.prefix_len, run_desc.window_base = self.dense, self.dense
        # a non-speculative run is never cancelled: its entries are what later runs build on
        pi.stage_forward(self.model, self.kv, run_desc, 0, self.L, logits_out=slot.logits, run_status=slot.out[0:2],
                         cancel_flag_ptr=slot.cancel_dev if speculative else None)
        if prev is None:
            pi.verify_greedy_chained(slot.tokens, None, n, slot.logits, self.vocab, int(tokens[0]), None, 0,
                                     slot.out[0:2], slot.out[8:8 + n], slot.out[2:4])
        else:
            pi.verify_greedy_chained(slot.tokens, None, n, slot.logits, self.vocab, 0, prev.slot.out[2:4], prev.n,
                                     slot.out[0:2], slot.out[8:8 + n], slot.out[2:4])
        if speculative:
            self.meta.accept(n, slot.positions, slot.tok_seq, slot.out[8:8 + n], slot.out[2:4])
        slot.out_host.copy_(slot.out, non_blocking=True)
        slot.event.record()
        assumed = self.accepted_frontier(start)
        rid = self.sched.begin_run(speculative, assumed, start - len(assumed), tokens, list(range(-1, n - 1)),
                                   list(range(start, start + n)), cancel_word_ptr=slot.cancel.data_ptr())
        run = _Run(rid, slot, speculative, [int(t) for t in tokens], start, seq)
        self.fifo.append(run)
        self.tail = run
        self.issued_cells += n
        self.stats["runs"] += 1
        self.stats["speculative" if speculative else "non_speculative"] += 1
        if speculative:
            self.stats["tokens_speculated"] += n
        return run

    def accepted_frontier(self, start):
        """Speculated tokens between the accepted end and `start` (what a run at `start`
        builds on): the tokens of the intact chain of runs in flight."""
        A = len(self.accepted)
        out = []
        for r in self.fifo:
            if not r.cancelled:
                for k, t in enumerate(r.tokens):
                    if A <= r.start + k < start:
                        out.append(t)
        return out

    def _room(self, n):
        return len(self.fifo) < self.depth and self.issued_cells + n <= pi.PI_WINDOW and self.free_slots

    # ---- results ---------------------------------------------------------------------------
    def _process_head(self):
        run = self.fifo.pop(0)
        run.slot.event.synchronize()
        out = run.slot.out_host.numpy()
        status, layers_done, a, bonus, placed, bad = (int(out[i]) for i in range(6))
        state = self.sched.complete_run(run.id)
        if placed != pi.PI_OK or bad != 0:
            raise RuntimeError("run %d: place status %d, %d inexpressible pairs" % (run.id, placed, bad))
        if status not in (pi.PI_OK, pi.PI_CANCELLED):
            raise pi.PiError(status, "stage forward of run %d" % run.id)
        counted = state == 0 and status == pi.PI_OK and a >= 1
        if state != 0:
            self.stats["discarded"] += 1
        if status == pi.PI_CANCELLED:
            self.stats["cancelled"] += 1
            self.stats["layers_skipped"] += self.L - layers_done
        if counted:
            # positions start .. start+a-1 hold the run's accepted tokens (the first of them is the
            # accepted end already), position start+a the target's own token
            new = run.tokens[1:a] + [bonus]
            assert len(self.accepted) == run.start + 1 and self.accepted[run.start] == run.tokens[0]
            self.accepted += new
            if run.speculative:
                self.stats["tokens_accepted_from_drafts"] += a
            for rid, _, _ in self.sched.accept_tokens(new, run_completed=True):
                for r in self.fifo:
                    if r.id == rid:
                        r.cancelled = True
        if run.speculative:
            self.meta.release(run.seq.bit_length() - 1)
        # the chain can be continued only while its last run is in flight and still stands (a
        # rejected token takes every run built on it along, so the last run tells)
        if self.tail is run or (self.tail is not None and self.tail.cancelled):
            self.tail = None
        self.free_slots.append(run.slot)

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
            if self.fifo and self.fifo[0].slot.event.query():
                self._process_head()                       # logits are waiting: sample and verify
                continue
            if not self.fifo and self.issued_cells + 1 + self.mb > pi.PI_WINDOW:
                self._compact()
                continue
            if self.tail is None and self._room(1):
                # nothing in flight covers the accepted end: the non-speculative run
                self._issue([self.accepted[-1]], len(self.accepted) - 1, speculative=False)
                continue
            if self.tail is not None and self._room(self.mb):
                start = self.tail.start + self.tail.n
                batch = []
                while len(batch) < self.mb:
                    tok, conf = self.draft(start + len(batch))
                    if not self.sched.want_speculation(conf):
                        break
                    batch.append(int(tok))
                if batch:
                    self._issue(batch, start, speculative=True)
                    self.sched.on_speculated()
                    continue
                self.stats["cutoff_stops"] += 1
                waiting = bool(self.fifo) and self.fifo[0].slot.event.query()
                self.sched.on_speculation_stopped(waiting)
                if not waiting and not self.fifo:
                    continue                               # idle: the cutoff decays until speculation resumes
            if self.fifo:
                self._process_head()                       # nothing to issue: wait for the oldest run
        while self.fifo:
            self._process_head()
        torch.cuda.synchronize()
        return self.accepted[self.first_generated:goal]

    def close(self):
        self.meta.free()
        self.sched.free()
