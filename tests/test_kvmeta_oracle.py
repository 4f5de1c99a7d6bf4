"""Pins for the cell-metadata oracle: scenarios worked by hand from the paper's description
(Sections "KV Cache" and "Pipelined KV Cache Multibuffering"), the tree-attention
definition by brute force, and the decoder oracle on runs that share the cache."""
import numpy as np

import synth
import oracle
from oracle import from_synth, OracleKVMeta, PI_E_FULL, PI_E_BUSY

ALL4 = [0, 1, 2, 3]


def _table(m):
    pos, seq = m.arrays()
    return list(map(int, pos)), list(map(int, seq))


# ---- the double-buffer scenario, cell by cell ------------------------------------------------

def test_partition_as_back_buffer_then_swap_worked_by_hand():
    """Four canonical entries; run A (partition 1) speculates positions 4..6; run B
    (partition 2) is given A's entries early and continues at 7, 8.  A is verified with two
    of three tokens accepted: those two become canonical, A's third entry and everything
    of B go away, and the identifiers return to the queue in the order they were freed."""
    m = OracleKVMeta(16, 4)
    m.fill(0, 4, 0, ALL4)
    a, b = m.acquire(), m.acquire()
    assert (a, b) == (1, 2)
    st, slots_a = m.place([4, 5, 6], [[a]] * 3, window_base=4)
    assert st == 0 and slots_a == [4, 5, 6]
    assert _table(m) == ([0, 1, 2, 3, 4, 5, 6] + [-1] * 9, [15] * 4 + [2] * 3 + [0] * 9)
    # A sees the prefix and its own causal entries, nothing else
    mask, bad = m.build_mask([4, 5, 6], [[a]] * 3, prefix_len=4, window_base=4)
    assert list(map(int, mask)) == [0b1, 0b11, 0b111] and bad == 0

    m.seq_cp(a, [b])                       # early sharing: B may read what A wrote
    st, slots_b = m.place([7, 8], [[b]] * 2, window_base=4)
    assert slots_b == [7, 8]
    assert _table(m)[1] == [15] * 4 + [6] * 3 + [4] * 2 + [0] * 7
    mask, bad = m.build_mask([7, 8], [[b]] * 2, 4, 4)
    assert list(map(int, mask)) == [0b1111, 0b11111] and bad == 0
    # A still does not see B
    mask, bad = m.build_mask([4, 5, 6], [[a]] * 3, 4, 4)
    assert list(map(int, mask)) == [0b1, 0b11, 0b111] and bad == 0

    m.accept([4, 5, 6], [[a]] * 3, accepted_nodes=[0, 1])
    assert _table(m)[1] == [15] * 6 + [6] + [4] * 2 + [0] * 7      # only up to position 5
    m.release(a)
    assert _table(m)[1] == [15] * 6 + [4] * 3 + [0] * 7
    m.release(b)                                                   # B continued a rejected token
    assert _table(m) == ([0, 1, 2, 3, 4, 5] + [-1] * 10, [15] * 6 + [0] * 10)
    assert [m.acquire(), m.acquire(), m.acquire(), m.acquire()] == [3, 1, 2, None]


def test_rival_runs_holes_and_compaction_worked_by_hand():
    """Two runs speculate the same positions in different partitions; the second wins.  Its
    entries become canonical where they lie (cells 6, 7), a later run sees them through the
    window, and compaction moves them down to cells 4, 5 once no partition is in the way."""
    m = OracleKVMeta(16, 4)
    m.fill(0, 4, 0, ALL4)
    a, b = m.acquire(), m.acquire()
    assert m.place([4, 5], [[a]] * 2, 4)[1] == [4, 5]
    assert m.place([4, 5], [[b]] * 2, 4)[1] == [6, 7]
    mask, bad = m.build_mask([4, 5], [[b]] * 2, 4, 4)
    assert list(map(int, mask)) == [0b0100, 0b1100] and bad == 0     # B never sees A's cells
    m.accept([4, 5], [[b]] * 2, [0, 1])
    m.release(a)
    m.release(b)
    assert _table(m) == ([0, 1, 2, 3, -1, -1, 4, 5] + [-1] * 8, [15] * 4 + [0, 0, 15, 15] + [0] * 8)
    c = m.acquire()
    assert c == 3
    st, slots_c = m.place([6], [[c]], 4)
    assert slots_c == [4]                                            # lowest free cell
    mask, bad = m.build_mask([6], [[c]], 4, 4)
    assert list(map(int, mask)) == [0b1101] and bad == 0
    K = np.arange(2 * 16 * 3, dtype=np.float64).reshape(2, 16, 3)
    V = -K.copy()
    K0 = K.copy()
    assert m.compact(4, K, V) == (PI_E_BUSY, 4) and np.array_equal(K, K0)
    m.release(c)
    assert m.compact(4, K, V) == (0, 6)
    assert _table(m) == ([0, 1, 2, 3, 4, 5] + [-1] * 10, [15] * 6 + [0] * 10)
    assert np.array_equal(K[:, 4], K0[:, 6]) and np.array_equal(K[:, 5], K0[:, 7])
    assert np.array_equal(V[:, 4], -K0[:, 6]) and np.array_equal(V[:, 5], -K0[:, 7])
    untouched = [c for c in range(16) if c not in (4, 5)]
    assert np.array_equal(K[:, untouched], K0[:, untouched])         # vacated cells keep their data


def test_compaction_orders_by_position_and_refuses_duplicates():
    m = OracleKVMeta(80, 3)
    m.fill(0, 2, 0, [0, 1, 2])
    for cell, pos in ((40, 3), (7, 2), (65, 4)):                     # canonical entries out of order
        m.fill(cell, 1, pos, [0, 1, 2])
    K = np.arange(80, dtype=np.float64).reshape(1, 80, 1)
    V = K + 1000
    assert m.compact(2, K, V) == (0, 5)
    assert _table(m)[0][:6] == [0, 1, 2, 3, 4, -1]
    assert K[0, 2:5, 0].tolist() == [7.0, 40.0, 65.0] and V[0, 2:5, 0].tolist() == [1007.0, 1040.0, 1065.0]
    assert m.pos[40] == -1 and m.pos[65] == -1 and m.pos[7] == -1
    m.fill(10, 1, 9, [0, 1, 2])
    m.fill(11, 1, 9, [0, 1, 2])
    assert m.compact(5)[0] == PI_E_BUSY
    # a canonical cell beyond the window is not compaction's business
    m2 = OracleKVMeta(80, 3)
    m2.fill(70, 1, 0, [0, 1, 2])
    assert m2.compact(0) == (0, 0) and m2.pos[70] == 0


def test_window_full_and_what_the_mask_form_cannot_express():
    m = OracleKVMeta(96, 3)
    m.fill(0, 8, 0, [0, 1, 2])
    s = m.acquire()
    st, slots = m.place(list(range(8, 70)), [[s]] * 62, 8)
    assert st == 0 and slots == list(range(8, 70))
    assert m.place([70, 71, 72], [[s]] * 3, 8) == (PI_E_FULL, None)  # two cells left, three asked
    assert m.pos[70] == -1 and m.pos[71] == -1
    # a visible entry that lies behind the window, and a prefix cell that a token must not see
    m.fill(90, 1, 5, [s])
    m.seq_rm([s], 3, 4)                                              # partition s loses position 3
    mask, bad = m.build_mask([69, 8], [[s], [s]], prefix_len=8, window_base=8)
    assert bad == 2 + 2                                              # per token: cell 90 and cell 3
    assert int(mask[0]) == (1 << 62) - 1 and int(mask[1]) == 1
    # overlap of prefix and window: the bit stays clear, the prefix already covers the cell
    mask, bad = m.build_mask([8], [[0]], prefix_len=8, window_base=4)
    assert int(mask[0]) == 0 and bad == 0


# ---- tree attention by brute force -------------------------------------------------------------

def _ancestors_or_self(parent, i):
    out = set()
    while i >= 0:
        out.add(i)
        i = int(parent[i])
    return out


def test_tree_mask_from_sequences_equals_ancestor_definition():
    """Each branch of a speculation tree is a sequence; a node carries the identifiers of
    all branches through it.  Membership plus position order must give exactly the tree
    mask: a node sees its ancestors and itself, never another branch."""
    for seed in range(12):
        n = 5 + seed
        parent = synth.random_tree(seed, 3, n)
        nl = synth.n_leaves(parent)
        m = OracleKVMeta(128, 32)
        T = 20
        m.fill(0, T, 0, range(32))
        # cells of some other run are already in the window, in a partition of their own
        other = m.acquire()
        taken = [T + 1, T + 2, T + 9]
        for c in taken:
            m.fill(c, 1, T, [other])
        ids = [m.acquire() for _ in range(nl)]
        seqs = synth.tree_sequences(parent, ids)
        run = synth.tree_run(parent, T, T)
        st, slots = m.place(run["positions"], seqs, T)
        assert st == 0 and not set(slots) & set(taken) and slots == sorted(slots)
        mask, bad = m.build_mask(run["positions"], seqs, T, T)
        assert bad == 0
        for i in range(n):
            want = sum(1 << (slots[j] - T) for j in _ancestors_or_self(parent, i))
            assert int(mask[i]) == want, (seed, i)


# ---- invariants under random edits ---------------------------------------------------------------

def test_invariants_under_random_edit_sequences():
    rng = np.random.default_rng(7)
    for trial in range(20):
        m = OracleKVMeta(96, 8)
        T = 16
        m.fill(0, T, 0, range(8))
        held = []
        queue = list(range(1, 8))        # what a FIFO of identifiers must hand out next
        for step in range(60):
            op = rng.integers(0, 5)
            if op == 0 and len(held) < 7:
                s = m.acquire()
                assert s == (queue.pop(0) if queue else None)
                if s is not None:
                    held.append(s)
            elif op == 1 and held:
                s = held[rng.integers(len(held))]
                k = int(rng.integers(1, 6))
                p0 = T + int(rng.integers(0, 6))
                m.place([p0 + i for i in range(k)], [[s]] * k, T)
            elif op == 2 and len(held) >= 2:
                src, dst = rng.choice(held, 2, replace=False)
                before = _table(m)
                m.seq_cp(int(src), [int(dst)], T, T + 4)
                gained = [c for c in range(96) if (_table(m)[1][c] ^ before[1][c])]
                assert all(before[1][c] >> int(src) & 1 and T <= before[0][c] < T + 4 for c in gained)
            elif op == 3 and held:
                s = held[rng.integers(len(held))]
                m.seq_rm([s], T + 2)
            elif op == 4 and held:
                s = held.pop(rng.integers(len(held)))
                m.release(s)
                queue.append(s)
                assert all(s not in m.seq[c] or 0 in m.seq[c] for c in range(96))
            pos, seq = _table(m)
            assert all((p < 0) == (q == 0) for p, q in zip(pos, seq))      # free <=> in no sequence
            assert all(seq[c] == 255 and pos[c] == c for c in range(T))     # canonical prefix untouched


# ---- runs that share the cache, through the decoder oracle -----------------------------------------

def _tiny(seed=0):
    sh = synth.SHAPES["tiny"]
    return sh, from_synth.model_from_seed(sh, seed, 0.1)


def _run_from_meta(m, positions, seqs, prefix_len, window_base):
    st, slots = m.place(positions, seqs, window_base)
    assert st == 0
    mask, bad = m.build_mask(positions, seqs, prefix_len, window_base)
    assert bad == 0
    return {"positions": np.asarray(positions, dtype=np.int32), "slots": np.asarray(slots, dtype=np.int32),
            "mask": mask, "prefix_len": prefix_len, "window_base": window_base, "n": len(positions)}


def test_chained_runs_equal_one_linear_batch():
    """Run B continues run A's speculation before A is verified (early entry sharing): its
    logits must be those of the last four tokens of one eight-token causal batch."""
    sh, model = _tiny()
    T = 12
    kv = from_synth.kv_synthetic(sh, 3, 64, T)
    toks = synth.tokens_host(sh, 5, 8, synth.T_DRAFT)
    whole = oracle.stage_forward(model, kv.clone(), synth.linear_run(8, T), 0, sh.n_layers, tokens=toks)["logits"]

    m = OracleKVMeta(64, 4)
    m.fill(0, T, 0, ALL4)
    a, b = m.acquire(), m.acquire()
    k2 = kv.clone()
    run_a = _run_from_meta(m, [T, T + 1, T + 2, T + 3], [[a]] * 4, T, T)
    la = oracle.stage_forward(model, k2, run_a, 0, sh.n_layers, tokens=toks[:4])["logits"]
    m.seq_cp(a, [b])
    run_b = _run_from_meta(m, [T + 4, T + 5, T + 6, T + 7], [[b]] * 4, T, T)
    lb = oracle.stage_forward(model, k2, run_b, 0, sh.n_layers, tokens=toks[4:])["logits"]
    assert np.allclose(la, whole[:4], rtol=1e-11, atol=1e-12)
    assert np.allclose(lb, whole[4:], rtol=1e-11, atol=1e-12)
    # without the early copy B would not see A: its logits must then differ
    m2 = OracleKVMeta(64, 4)
    m2.fill(0, T, 0, ALL4)
    a2, b2 = m2.acquire(), m2.acquire()
    k3 = kv.clone()
    ra = _run_from_meta(m2, [T, T + 1, T + 2, T + 3], [[a2]] * 4, T, T)
    oracle.stage_forward(model, k3, ra, 0, sh.n_layers, tokens=toks[:4])
    rb = _run_from_meta(m2, [T + 4, T + 5, T + 6, T + 7], [[b2]] * 4, T, T)
    lb2 = oracle.stage_forward(model, k3, rb, 0, sh.n_layers, tokens=toks[4:])["logits"]
    assert np.max(np.abs(lb2 - whole[4:])) > 1e-3


def test_winner_left_in_place_equals_winner_moved_to_canonical_cells():
    """A rival run's accepted entries stay in their window cells and are seen through the
    mask; the next run's logits must equal those computed after the data-moving commit
    (copy to canonical cells), and after compaction of the metadata-kept cache."""
    sh, model = _tiny()
    T = 12
    kv = from_synth.kv_synthetic(sh, 3, 64, T)
    ta = synth.tokens_host(sh, 6, 2, synth.T_DRAFT)
    tb = synth.tokens_host(sh, 7, 2, synth.T_DRAFT)
    tc = synth.tokens_host(sh, 8, 3, synth.T_DRAFT)

    # data-moving reference: B alone, committed by rollback, then C on a dense prefix
    kr = kv.clone()
    rb = synth.linear_run(2, T)
    oracle.stage_forward(model, kr, rb, 0, sh.n_layers, tokens=tb)
    oracle.kv_rollback(kr, rb["slots"], [0, 1])
    ref = oracle.stage_forward(model, kr, synth.linear_run(3, T + 2), 0, sh.n_layers, tokens=tc)["logits"]

    m = OracleKVMeta(64, 4)
    m.fill(0, T, 0, ALL4)
    a, b = m.acquire(), m.acquire()
    km = kv.clone()
    run_a = _run_from_meta(m, [T, T + 1], [[a]] * 2, T, T)
    oracle.stage_forward(model, km, run_a, 0, sh.n_layers, tokens=ta)
    run_b = _run_from_meta(m, [T, T + 1], [[b]] * 2, T, T)
    oracle.stage_forward(model, km, run_b, 0, sh.n_layers, tokens=tb)
    m.accept(run_b["positions"], [[b]] * 2, [0, 1])
    m.release(a)
    m.release(b)
    c = m.acquire()
    run_c = _run_from_meta(m, [T + 2, T + 3, T + 4], [[c]] * 3, T, T)
    assert run_c["slots"].tolist() == [T, T + 1, T + 4]               # A's freed cells are reused
    got = oracle.stage_forward(model, km.clone(), run_c, 0, sh.n_layers, tokens=tc)["logits"]
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-12)

    # compaction before C instead: dense prefix T + 2, same logits again
    m.release(c)
    assert m.compact(T, km.K, km.V) == (0, T + 2)
    km.kv_len = T + 2
    c = m.acquire()
    run_c2 = _run_from_meta(m, [T + 2, T + 3, T + 4], [[c]] * 3, T + 2, T + 2)
    got2 = oracle.stage_forward(model, km, run_c2, 0, sh.n_layers, tokens=tc)["logits"]
    assert np.allclose(got2, ref, rtol=1e-11, atol=1e-12)
