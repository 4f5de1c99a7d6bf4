"""CPU oracle for KV-cache cell metadata and sequence partitions.  TEST INFRASTRUCTURE ONLY.

A plain statement, in Python sets and loops, of the bookkeeping that lets several inference
runs share one KV cache: nothing here is shared with the HIP library, and only tests, the
smoke check and the benchmark's cpu_baseline leg may import it.

What the paper fixes (and where):
  * every cache cell carries metadata -- the position of its entry and the set of
    sequences it belongs to; cache changes are made by editing the metadata, and the
    attention mask is built from it                       -- Section "KV Cache"
  * sequence 0 is the canonical sequence; every speculative run gets a sequence
    identifier from a FIFO queue of free identifiers, and, together with the causal
    mask, sequence membership keeps runs from seeing each other's entries
                      -- Section "Pipelined KV Cache Multibuffering / Sequence partitions"
  * when a run ends, the entries of its accepted tokens are copied to the canonical
    sequence (the "buffer swap") and the partition is free again      -- same section
  * accepted entries are copied to all other sequences too, but only up to the position
    of the last accepted token       -- Section "Sequence acceptance and propagation"
  * a run may be given another sequence's entries before that sequence is verified, so
    it can continue from them     -- Section "Transactions and early cache entry sharing"

Readings taken where the paper leaves the bookkeeping open:
  * copying "to a sequence" only adds the identifier to the cell's set (no data moves);
  * a token of a run may belong to several sequences (a tree node shared by several
    branches, one identifier per branch): it sees cell c iff the two sets intersect and
    pos[c] <= the token's position;
  * new entries take the lowest free cells of a 64-cell window, in token order;
  * freeing a partition removes its identifier from every cell that is not canonical
    (a cell is canonical iff sequence 0 is in its set) and frees cells left in no sequence;
  * the attention kernel takes visibility as "a dense prefix that every token sees, plus
    a 64-bit word per token over the window", so the mask builder also counts what this
    form cannot express, and compaction moves canonical window cells down into the dense
    prefix, in position order, once no partition holds a cell of the window.
"""
from __future__ import annotations

import numpy as np

PI_OK = 0
PI_E_ARG = -1
PI_E_FULL = -7
PI_E_BUSY = -8
WINDOW = 64
CANONICAL = 0
POS_MAX = 2**31 - 1  # "no upper bound" for position ranges [p0, p1)


class OracleKVMeta:
    def __init__(self, n_cells: int, n_seq: int):
        assert 2 <= n_seq <= 32
        self.n_cells, self.n_seq = n_cells, n_seq
        self.pos = [-1] * n_cells                     # -1: the cell is free
        self.seq = [set() for _ in range(n_cells)]    # sequences the cell's entry belongs to
        self.free_ids = list(range(1, n_seq))         # FIFO of free partition identifiers
        self.held = set()

    # ---- sequence identifiers (FIFO) ------------------------------------------------------
    def acquire(self):
        """Identifier at the head of the queue, or None when every partition is in use."""
        if not self.free_ids:
            return None
        s = self.free_ids.pop(0)
        self.held.add(s)
        return s

    def release(self, s: int) -> None:
        """The run that held partition s is over: what it holds beside canonical entries is
        dropped, and s goes to the tail of the queue."""
        assert s in self.held
        for c in range(self.n_cells):
            if s in self.seq[c] and CANONICAL not in self.seq[c]:
                self.seq[c].discard(s)
                if not self.seq[c]:
                    self.pos[c] = -1
        self.held.discard(s)
        self.free_ids.append(s)

    # ---- cell edits -----------------------------------------------------------------------
    def fill(self, cell0: int, n: int, pos0: int, seqs) -> None:
        """Mark cells cell0.. as holding positions pos0.. in `seqs` (prefilled entries)."""
        for i in range(n):
            self.pos[cell0 + i] = pos0 + i
            self.seq[cell0 + i] = set(seqs)

    def place(self, positions, tok_seqs, window_base: int):
        """Cells for a run's new entries: token i gets the i-th lowest free cell of the
        window.  Returns (PI_OK, slots), or with nothing changed (PI_E_FULL, None), or
        (PI_E_ARG, None) for a token with a negative position, no sequence or an identifier
        the table does not have."""
        for p, ss in zip(positions, tok_seqs):
            if int(p) < 0 or len(ss) == 0 or any(not 0 <= s < self.n_seq for s in ss):
                return PI_E_ARG, None
        free =[c for c in range(window_base, min(window_base + WINDOW, self.n_cells)) if self.pos[c] < 0]
        n = len(positions)
        if len(free) < n:
            return PI_E_FULL, None
        slots = free[:n]
        for i, c in enumerate(slots):
            self.pos[c] = int(positions[i])
            self.seq[c] = set(tok_seqs[i])
        return PI_OK, slots

    def seq_cp(self, src: int, dst, p0: int = 0, p1: int = POS_MAX) -> None:
        """Entries of sequence src at positions [p0, p1) also become entries of every
        sequence in dst."""
        for c in range(self.n_cells):
            if src in self.seq[c] and p0 <= self.pos[c] < p1:
                self.seq[c] |= set(dst)

    def seq_rm(self, seqs, p0: int = 0, p1: int = POS_MAX) -> None:
        """Entries at positions [p0, p1) leave every sequence in seqs; a cell left in no
        sequence is free."""
        for c in range(self.n_cells):
            if self.pos[c] >= 0 and p0 <= self.pos[c] < p1:
                self.seq[c] -= set(seqs)
                if not self.seq[c]:
                    self.pos[c] = -1

    def accept(self, positions, tok_seqs, accepted_nodes) -> None:
        """The accepted path of a run becomes part of every sequence: the entries of the
        branch the last accepted token lies on (its lowest identifier), up to and
        including that token's position."""
        if len(accepted_nodes) == 0:
            return
        last = accepted_nodes[-1]
        src = min(tok_seqs[last])
        self.seq_cp(src, range(self.n_seq), 0, int(positions[last]) + 1)

    # ---- visibility -----------------------------------------------------------------------
    def visible(self, p: int, seqs, c: int) -> bool:
        return bool(self.seq[c] & set(seqs)) and self.pos[c] <= p

    def build_mask(self, positions, tok_seqs, prefix_len: int, window_base: int):
        """Window words for the attention kernel, and the number of (token, cell) pairs the
        kernel's form gets wrong: a prefix cell some token must not see, or a visible cell
        that lies neither in the prefix nor in the window."""
        n = len(positions)
        mask = np.zeros(n, dtype=np.uint64)
        bad = 0
        for i in range(n):
            word = 0
            for c in range(self.n_cells):
                vis = self.visible(int(positions[i]), tok_seqs[i], c)
                in_window = window_base <= c < window_base + WINDOW
                # prefix cells are always attended to; a window cell below prefix_len
                # (overlap) is attended to through the prefix, not through its bit
                if c < prefix_len:
                    bad += 0 if vis else 1
                elif in_window:
                    word |= (1 << (c - window_base)) if vis else 0
                else:
                    bad += 1 if vis else 0
            mask[i] = np.uint64(word)
        return mask, bad

    # ---- compaction -----------------------------------------------------------------------
    def compact(self, prefix_len: int, K: np.ndarray | None = None, V: np.ndarray | None = None):
        """Move the canonical cells of the window [prefix_len, prefix_len + 64) down to
        prefix_len, prefix_len + 1, ... in position order (metadata and, when given, the
        data K, V[layers, cells, ...] of every layer); cells that were moved away and not
        refilled are free, their data stays.  Refused (PI_E_BUSY, nothing changes) while a
        cell of the window belongs to partitions only, or when two canonical window cells
        hold the same position.  Returns (status, dense length)."""
        win = range(prefix_len, min(prefix_len + WINDOW, self.n_cells))
        live = [c for c in win if self.pos[c] >= 0]
        if any(CANONICAL not in self.seq[c] for c in live):
            return PI_E_BUSY, prefix_len
        if len({self.pos[c] for c in live}) != len(live):
            return PI_E_BUSY, prefix_len
        order = sorted(live, key=lambda c: self.pos[c])
        old_pos = {c: self.pos[c] for c in order}
        old_seq = {c: set(self.seq[c]) for c in order}
        if K is not None:
            oldK = {c: K[:, c].copy() for c in order}
            oldV = {c: V[:, c].copy() for c in order}
        for c in order:
            self.pos[c] = -1
            self.seq[c] = set()
        for k, c in enumerate(order):
            t = prefix_len + k
            self.pos[t] = old_pos[c]
            self.seq[t] = old_seq[c]
            if K is not None:
                K[:, t] = oldK[c]
                V[:, t] = oldV[c]
        return PI_OK, prefix_len + len(order)

    # ---- export ---------------------------------------------------------------------------
    def arrays(self):
        """pos[n_cells] int32 and seq[n_cells] uint32 (bit s set iff s is in the cell's set)."""
        pos = np.asarray(self.pos, dtype=np.int32)
        seq = np.asarray([sum(1 << s for s in ss) for ss in self.seq], dtype=np.uint32)
        return pos, seq
