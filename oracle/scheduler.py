"""CPU oracle for the head node's run bookkeeping.  TEST INFRASTRUCTURE ONLY.

A plain Python statement of what the head node tracks while several inference runs are in
flight, and of the decisions it takes after every verification.  Nothing here is shared with
the library; only tests, the smoke check and the benchmark's cpu_baseline leg may import it.

What the paper fixes (and where):
  * every run is described by a record created before the run starts and kept in a FIFO
    queue; the record is removed when the run completes
                      -- Sections "State tracking", "Cancellation back-propagation"
  * the record holds the run's speculated tokens and its lowest and highest token positions
                      -- Section "Invalidation detection"
  * a run whose highest position lies below the position of the last accepted token is
    superfluous; a run whose speculated sequence does not begin like the accepted tokens
    end is invalidated; both are looked for after every sampling phase, over the whole queue
                      -- Section "Invalidation detection"
  * such runs are cancelled by a signal that names the run; a non-speculative run is only
    marked: it is still evaluated in full and just its sampling is skipped
                      -- Sections "Cancellation back-propagation", "Performance
                         considerations and conflicts"
  * the confidence a draft token needs for speculation to go on starts at a base cutoff,
    rises by a recovery factor with every further speculation issued, returns to the base
    when a completed run is accepted, and falls by a decay factor whenever speculation
    stops for lack of confidence while no logits are waiting
                      -- Section "Reactive speculation"

Readings taken where the text leaves details open:
  * positions count tokens from 0; "the accepted end" is the position of the last accepted
    token, A - 1 for A accepted tokens;
  * superfluous is strict: a run whose highest position equals the accepted end still
    yields the prediction for the next position and is kept;
  * a run built on tokens that were themselves speculation when it started keeps those
    "assumed" tokens in its record (positions assumed_pos0 ..), so that rejecting an
    earlier run invalidates its descendants by the same token comparison;
  * a tree run matches iff some path from a root follows the accepted tokens for as long as
    the accepted sequence and the tree overlap; no constraint where they do not overlap;
  * method 1 is looked at first, then method 2; a run is reported once;
  * the cutoff is not clamped.
"""
from __future__ import annotations

SUPERFLUOUS = 1
INVALIDATED = 2


class RunRecord:
    def __init__(self, run_id, speculative, assumed, assumed_pos0, tokens, parent, positions):
        self.id = run_id
        self.speculative = bool(speculative)
        self.assumed = [int(t) for t in assumed]
        self.assumed_pos0 = int(assumed_pos0)
        self.tokens = [int(t) for t in tokens]
        self.parent = [int(p) for p in parent]
        self.positions = [int(p) for p in positions]
        self.cancelled = 0            # 0, SUPERFLUOUS or INVALIDATED
        self.signalled = False        # the cancellation signal was sent (speculative runs only)
        self.min_pos = min(self.positions + ([self.assumed_pos0] if self.assumed else []))
        self.max_pos = max(self.positions)


class OracleScheduler:
    def __init__(self, base_cutoff: float, recovery: float, decay: float):
        self.base, self.recovery, self.decay = float(base_cutoff), float(recovery), float(decay)
        self.cutoff = self.base
        self.accepted = []            # the canonical token sequence
        self.fifo = []                # run records, oldest first
        self.next_id = 0

    # ---- run records ----------------------------------------------------------------------
    def begin_run(self, speculative, assumed, assumed_pos0, tokens, parent, positions) -> int:
        rec = RunRecord(self.next_id, speculative, assumed, assumed_pos0, tokens, parent, positions)
        self.next_id += 1
        self.fifo.append(rec)
        return rec.id

    def complete_run(self, run_id: int):
        """The run's result has been dealt with: its record leaves the queue.  Returns the
        record's cancellation state."""
        for k, rec in enumerate(self.fifo):
            if rec.id == run_id:
                return self.fifo.pop(k).cancelled
        raise KeyError(run_id)

    # ---- the two detection methods --------------------------------------------------------
    def _superfluous(self, rec) -> bool:
        return rec.max_pos < len(self.accepted) - 1

    def _follows_accepted(self, rec) -> bool:
        A = len(self.accepted)
        for k, t in enumerate(rec.assumed):
            p = rec.assumed_pos0 + k
            if p < A and self.accepted[p] != t:
                return False
        # nodes that can still lie on the accepted path, level by level
        alive = [i for i in range(len(rec.tokens)) if rec.parent[i] < 0]
        while alive:
            p = rec.positions[alive[0]]
            if p >= A:
                return True                          # beyond the accepted end: nothing to compare
            alive = [i for i in alive if rec.tokens[i] == self.accepted[p]]
            if not alive:
                return False
            nxt = [c for c in range(len(rec.tokens)) if rec.parent[c] in alive]
            if not nxt:
                return True                          # the matching path ends inside the accepted tokens
            alive = nxt
        return True

    def accept_tokens(self, tokens, run_completed: bool = True):
        """Tokens join the accepted sequence (a sampling phase has ended); the queue is then
        searched.  Returns [(run id, reason, signal)] for the runs newly found superfluous
        or invalidated, oldest first; signal says whether the cancellation signal is sent
        (speculative runs) or the run is only marked (non-speculative runs)."""
        self.accepted += [int(t) for t in tokens]
        if run_completed:
            self.cutoff = self.base
        out = []
        for rec in self.fifo:
            if rec.cancelled:
                continue
            if self._superfluous(rec):
                rec.cancelled = SUPERFLUOUS
            elif not self._follows_accepted(rec):
                rec.cancelled = INVALIDATED
            if rec.cancelled:
                rec.signalled = rec.speculative
                out.append((rec.id, rec.cancelled, rec.signalled))
        return out

    # ---- reactive speculation ---------------------------------------------------------------
    def want_speculation(self, confidence: float) -> bool:
        return float(confidence) >= self.cutoff

    def on_speculated(self) -> None:
        self.cutoff = self.cutoff + self.recovery

    def on_speculation_stopped(self, logits_waiting: bool) -> None:
        if not logits_waiting:
            self.cutoff = self.cutoff - self.decay
