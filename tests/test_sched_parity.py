"""The native run bookkeeping (pi_sched_*, host code of the library) against the CPU oracle:
same queues, same cancellations in the same order, same cutoff bit for bit, and the
cancellation signal lands in exactly the words of the speculative runs that were cancelled.
Needs no GPU."""
import ctypes

import numpy as np
import pytest

import synth
import paper_2407_11798_amd as pi
from oracle.scheduler import OracleScheduler


class Both:
    def __init__(self, base, rec, dec, n_words=512):
        self.o = OracleScheduler(base, rec, dec)
        self.g = pi.Scheduler(base, rec, dec)
        self.words = (ctypes.c_int32 * n_words)()
        self.want_words = [0] * n_words
        self.word_of = {}

    def begin(self, speculative, assumed, pos0, tokens, parent, positions):
        rid = self.o.begin_run(speculative, assumed, pos0, tokens, parent, positions)
        ptr = ctypes.addressof(self.words) + 4 * rid
        got = self.g.begin_run(speculative, assumed, pos0, tokens, parent, positions, cancel_word_ptr=ptr)
        assert got == rid
        self.word_of[rid] = rid
        return rid

    def accept(self, tokens, completed=True):
        want = self.o.accept_tokens(tokens, completed)
        got = self.g.accept_tokens(tokens, completed)
        assert got == want
        for rid, _, signalled in want:
            if signalled:
                self.want_words[rid] = 1
        assert list(self.words) == self.want_words
        return want

    def complete(self, rid):
        assert self.g.complete_run(rid) == self.o.complete_run(rid)

    def check(self):
        cutoff, na, ids = self.g.state()
        assert cutoff == self.o.cutoff                       # bit for bit: same operations in the same order
        assert na == len(self.o.accepted)
        assert ids == [r.id for r in self.o.fifo]


def test_worked_scenario_through_the_c_abi():
    b = Both(0.25, 0.125, 0.0625)
    b.accept([5, 6, 7], completed=False)
    r_ns = b.begin(False, [], 0, [7], [-1], [2])
    r0 = b.begin(True, [], 0, [10, 11], [-1, 0], [3, 4])
    r1 = b.begin(True, [10, 11], 3, [12, 13], [-1, 0], [5, 6])
    assert b.accept([10]) == [(r_ns, pi.PI_RUN_SUPERFLUOUS, False)]
    assert b.accept([99]) == [(r0, pi.PI_RUN_INVALIDATED, True), (r1, pi.PI_RUN_INVALIDATED, True)]
    assert list(b.words)[:3] == [0, 1, 1]                    # the non-speculative run is never signalled
    b.complete(r_ns)
    b.complete(r0)
    b.check()
    assert pi.lib().pi_sched_complete_run(b.g.handle, r0, None) == pi.PI_E_ARG


def test_cutoff_arithmetic_matches_bit_for_bit():
    b = Both(0.3, 0.07, 0.011)                               # not exactly representable on purpose
    for k in range(200):
        if k % 7 == 3:
            b.o.on_speculation_stopped(k % 2 == 0)
            b.g.on_speculation_stopped(k % 2 == 0)
        elif k % 31 == 30:
            b.accept([k], completed=True)
        else:
            b.o.on_speculated()
            b.g.on_speculated()
        for c in (0.1, 0.3, 0.5, 0.9, b.o.cutoff):
            assert b.g.want_speculation(c) == b.o.want_speculation(c)
        b.check()


def test_arguments_are_checked():
    L = pi.lib()
    out = ctypes.c_void_p()
    assert L.pi_sched_create(0.5, 0.0, 0.0, None) == pi.PI_E_ARG
    assert L.pi_sched_create(0.5, 0.0, 0.0, ctypes.byref(out)) == pi.PI_OK
    rid = ctypes.c_int32()
    tok = (ctypes.c_int32 * 3)(1, 2, 3)
    par_bad = (ctypes.c_int32 * 3)(-1, 1, 0)                 # a node may not be its own parent
    par = (ctypes.c_int32 * 3)(-1, 0, 0)
    pos_bad = (ctypes.c_int32 * 3)(4, 5, 6)                  # both children sit one below the root
    pos = (ctypes.c_int32 * 3)(4, 5, 5)
    args = lambda pa, po, n=3: L.pi_sched_begin_run(out, 1, None, 0, 0, tok, pa, po, n, None, ctypes.byref(rid))
    assert args(par_bad, pos) == pi.PI_E_ARG
    assert args(par, pos_bad) == pi.PI_E_ARG
    assert args(par, pos, 0) == pi.PI_E_SHAPE and args(par, pos, 17) == pi.PI_E_SHAPE
    assert args(par, pos) == pi.PI_OK and rid.value == 0
    assert L.pi_sched_accept_tokens(out, None, 1, 1, None, None, None, 0, None) == pi.PI_E_ARG
    assert L.pi_sched_free(out) == pi.PI_OK and L.pi_sched_free(None) == pi.PI_E_ARG


@pytest.mark.parametrize("seed,alpha,vocab", [(0, 0.5, 3), (1, 0.8, 5), (2, 0.3, 2), (3, 0.66, 50)])
def test_random_speculation_streams(seed, alpha, vocab):
    """A seeded ground-truth sequence; runs (chains and trees) whose tokens agree with it with
    probability alpha, each building on the speculation issued before it; sampling phases that
    accept one to three true tokens; completions in and out of order."""
    rng = np.random.default_rng(seed)
    G = rng.integers(0, vocab, size=400).tolist()
    b = Both(0.4, 0.05, 0.02)
    b.accept(G[:4], completed=False)
    A = 4
    frontier = []            # speculated tokens beyond the accepted end (positions A ..)
    live = []
    for step in range(250):
        op = int(rng.integers(0, 10))
        if op < 4 and len(live) < 12:
            n = int(rng.integers(1, 9))
            parent = synth.random_tree(seed, step, n) if rng.integers(2) else np.arange(-1, n - 1)
            start = A + len(frontier)
            depth = np.zeros(n, dtype=np.int64)
            for i in range(n):
                depth[i] = 0 if parent[i] < 0 else depth[parent[i]] + 1
            positions = (start + depth).tolist()
            tokens = [G[p] if rng.random() < alpha else int(rng.integers(0, vocab)) for p in positions]
            speculative = bool(rng.integers(0, 6))
            live.append(b.begin(speculative, list(frontier), A, tokens, parent.tolist(), positions))
            # the next run builds on the first branch of this one
            j, path = 0, []
            while j >= 0:
                path.append(tokens[j])
                kids = [c for c in range(n) if parent[c] == j]
                j = kids[0] if kids else -1
            frontier += path
            b.o.on_speculated()
            b.g.on_speculated()
        elif op < 7:
            k = int(rng.integers(1, 4))
            b.accept(G[A:A + k], completed=bool(rng.integers(2)))
            for t in G[A:A + k]:                              # speculation that was right stays the frontier
                if frontier and frontier[0] == t:
                    frontier.pop(0)
                else:
                    frontier = []
            A += k
        elif op < 9 and live:
            b.complete(live.pop(0 if rng.integers(3) else int(rng.integers(len(live)))))
        else:
            w = bool(rng.integers(2))
            b.o.on_speculation_stopped(w)
            b.g.on_speculation_stopped(w)
        b.check()
    assert sum(b.want_words) > 0                              # the stream did cancel speculative runs


def test_largest_batch_empty_sampling_phase_and_short_report_buffer():
    b = Both(0.5, 0.0, 0.0)
    b.accept([1, 2, 3], completed=False)
    parent = synth.random_tree(5, 1, 16, max_children=3, max_depth=6)
    depth = np.zeros(16, dtype=np.int64)
    for i in range(16):
        depth[i] = 0 if parent[i] < 0 else depth[parent[i]] + 1
    ids = [b.begin(True, [], 0, list(range(100, 116)), parent.tolist(), (3 + depth).tolist()) for _ in range(5)]
    assert b.accept([], completed=True) == []                       # nothing sampled: nothing to find
    # one wrong token takes all five runs; a report buffer of two still cancels all of them
    want = b.o.accept_tokens([7], True)
    got = b.g.accept_tokens([7], True, cap=2)
    assert [w[0] for w in want] == ids and got == want[:2]
    assert list(b.words)[:5] == [1] * 5
    b.check()
