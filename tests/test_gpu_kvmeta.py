"""GPU parity for KV cell metadata and sequence partitions: every edit, the mask builder and
compaction through the C ABI against the CPU oracle, bit for bit (all of it is integer and
index work), and runs that share the cache through device-built slots and masks against the
decoder oracle."""
import numpy as np
import pytest
import torch

import synth
import oracle
from oracle import from_synth, OracleKVMeta
from synth import gpu_loader
import paper_2407_11798_amd as pi
from gpu_common import max_rel_rowwise

pytestmark = pytest.mark.gpu


def dev_i32(a):
    return torch.as_tensor(np.asarray(a, dtype=np.int32), device="cuda")


def dev_sets(seqs):
    """Sequence sets -> int32 tensor holding the uint32 bit sets."""
    return torch.as_tensor(np.asarray([pi.seq_bits(s) for s in seqs], dtype=np.uint32).view(np.int32), device="cuda")


class Pair:
    """The oracle's table and the device table, edited in step."""

    def __init__(self, n_cells, n_seq):
        self.n_cells, self.n_seq = n_cells, n_seq
        self.o = OracleKVMeta(n_cells, n_seq)
        self.g = pi.KVMeta(n_cells, n_seq)

    def check(self, what=""):
        pos, seq = self.g.read()
        opos, oseq = self.o.arrays()
        assert np.array_equal(pos, opos), "positions differ after " + what
        assert np.array_equal(seq, oseq), "sequence sets differ after " + what

    def acquire(self):
        a, b = self.o.acquire(), self.g.acquire()
        assert a == b
        return a

    def release(self, s):
        self.o.release(s)
        self.g.release(s)

    def fill(self, cell0, n, pos0, seqs):
        self.o.fill(cell0, n, pos0, seqs)
        self.g.fill(cell0, n, pos0, pi.seq_bits(seqs))

    def place(self, positions, seqs, window_base):
        n = len(positions)
        slots = torch.full((n,), -99, dtype=torch.int32, device="cuda")
        status = torch.full((1,), -99, dtype=torch.int32, device="cuda")
        self.g.place(n, dev_i32(positions), dev_sets(seqs), window_base, slots, status)
        st, oslots = self.o.place(positions, seqs, window_base)
        assert int(status.item()) == st
        assert slots.cpu().tolist() == (oslots if st == 0 else [-1] * n)
        return st, slots

    def seq_cp(self, src, dst, p0=0, p1=pi.PI_POS_MAX):
        self.o.seq_cp(src, dst, p0, p1)
        self.g.seq_cp(src, pi.seq_bits(dst), p0, p1)

    def seq_rm(self, seqs, p0=0, p1=pi.PI_POS_MAX):
        self.o.seq_rm(seqs, p0, p1)
        self.g.seq_rm(pi.seq_bits(seqs), p0, p1)

    def accept(self, positions, seqs, accepted):
        n = len(positions)
        acc = np.full(n, -1, dtype=np.int32)
        acc[:len(accepted)] = accepted
        self.o.accept(positions, seqs, list(accepted))
        self.g.accept(n, dev_i32(positions), dev_sets(seqs), dev_i32(acc), dev_i32([len(accepted), 7]))

    def build_mask(self, positions, seqs, prefix_len, window_base):
        n = len(positions)
        mask = torch.full((n,), -1, dtype=torch.int64, device="cuda")
        bad = torch.full((1,), -99, dtype=torch.int32, device="cuda")
        self.g.build_mask(n, dev_i32(positions), dev_sets(seqs), prefix_len, window_base, mask, bad)
        omask, obad = self.o.build_mask(positions, seqs, prefix_len, window_base)
        assert np.array_equal(mask.cpu().numpy().view(np.uint64), omask), "window words differ"
        assert int(bad.item()) == obad
        return mask, obad

    def compact(self, prefix_len, kv=None, K=None, V=None):
        res = torch.full((2,), -99, dtype=torch.int32, device="cuda")
        self.g.compact(kv, prefix_len, res)
        want = self.o.compact(prefix_len, K, V)
        assert tuple(res.cpu().tolist()) == want
        return want


# ---- the worked scenarios of the CPU pins, on the device -----------------------------------------

def test_double_buffer_scenario_on_the_device():
    p = Pair(16, 4)
    p.fill(0, 4, 0, [0, 1, 2, 3])
    a, b = p.acquire(), p.acquire()
    p.place([4, 5, 6], [[a]] * 3, 4)
    p.build_mask([4, 5, 6], [[a]] * 3, 4, 4)
    p.seq_cp(a, [b])
    p.place([7, 8], [[b]] * 2, 4)
    p.check("early sharing")
    mask, _ = p.build_mask([7, 8], [[b]] * 2, 4, 4)
    assert mask.cpu().tolist() == [0b1111, 0b11111]
    p.accept([4, 5, 6], [[a]] * 3, [0, 1])
    p.check("accept")
    p.release(a)
    p.release(b)
    p.check("release")
    pos, seq = p.g.read()
    assert pos.tolist() == [0, 1, 2, 3, 4, 5] + [-1] * 10 and seq.tolist() == [15] * 6 + [0] * 10
    assert [p.acquire() for _ in range(4)] == [3, 1, 2, None]


def test_refusals_reported_on_the_device():
    p = Pair(96, 3)
    p.fill(0, 8, 0, [0, 1, 2])
    s = p.acquire()
    st, _ = p.place(list(range(8, 24)), [[s]] * 16, 8)
    assert st == 0
    for k in range(3):
        p.place(list(range(24 + 15 * k, 39 + 15 * k)), [[s]] * 15, 8)   # 61 of 64 cells taken
    st, _ = p.place([70, 71, 72, 73], [[s]] * 4, 8)
    assert st == pi.PI_E_FULL
    p.check("full window")
    st, _ = p.place([70, -1], [[s], [s]], 8)
    assert st == pi.PI_E_ARG
    st, _ = p.place([70, 71], [[s], []], 8)
    assert st == pi.PI_E_ARG
    p.check("refused tokens")
    # what prefix + window cannot express is counted, not hidden
    p.fill(90, 1, 5, [s])
    p.seq_rm([s], 3, 4)
    _, bad = p.build_mask([69, 8], [[s], [s]], 8, 8)
    assert bad == 4
    _, bad = p.build_mask([8], [[0]], 8, 4)                                 # window overlaps the prefix
    assert bad == 0
    # release of a partition that is not held; compaction while a partition is in the window
    assert pi.lib().pi_kvmeta_seq_release(p.g.handle, 2, None) == pi.PI_E_ARG
    assert p.compact(8)[0] == pi.PI_E_BUSY
    p.check("refused compaction")


def test_degenerate_tables_and_windows():
    """No prefix at all, the largest batch, a table with a single partition, a window of one
    cell at the very end of the cache, compaction with nothing to move."""
    p = Pair(80, 2)                                   # sequence 0 and one partition
    s = p.acquire()
    assert s == 1 and p.acquire() is None
    st, _ = p.place(list(range(16)), [[s]] * 16, 0)   # empty prefix: positions 0..15 in cells 0..15
    assert st == 0
    mask, bad = p.build_mask(list(range(16)), [[s]] * 16, 0, 0)
    assert bad == 0 and mask.cpu().tolist() == [(2 << i) - 1 for i in range(16)]
    assert p.compact(0)[0] == pi.PI_E_BUSY
    p.accept(list(range(16)), [[s]] * 16, list(range(16)))
    p.release(s)
    assert p.compact(0) == (0, 16)
    assert p.compact(16) == (0, 16)                   # nothing in the window: nothing moves
    p.check("empty prefix")
    s = p.acquire()
    st, _ = p.place([16], [[s]], 79)                  # the window is the cache's last cell
    assert st == 0
    st, _ = p.place([17], [[s]], 79)
    assert st == pi.PI_E_FULL
    mask, bad = p.build_mask([16], [[s]], 16, 79)
    assert bad == 0 and mask.cpu().tolist() == [1]
    p.check("last cell")
    # calls that edit nothing are accepted and change nothing
    p.g.fill(0, 0, 0, 3)
    p.g.seq_cp(0, 0)
    p.g.seq_rm(0)
    p.g.seq_cp(1, 1, 5, 5)
    p.check("no-ops")


# ---- random edit sequences --------------------------------------------------------------------------

@pytest.mark.parametrize("n_cells,n_seq,seed", [(70, 4, 0), (200, 32, 1), (1152, 8, 2), (2112, 32, 3), (40000, 16, 4)])
def test_random_edit_sequences_match_the_oracle(n_cells, n_seq, seed):
    """Sizes: a window that runs past the last cell (70), the cache sizes of the 7B workload
    with 8 runs in flight (1024 + window, rounded) and of the 70B workload (2048 + 64), and a
    table larger than one pass of the mask builder's grid.  Runs come and go as in the method:
    each takes partitions of its own (one, or one per tree branch), may be given another
    run's entries, is accepted up to some token if it starts at the accepted end, and gives
    its partitions back; compaction is tried now and then."""
    rng = np.random.default_rng(100 + seed)
    p = Pair(n_cells, n_seq)
    T = int(rng.integers(4, n_cells // 2)) if n_cells < 300 else n_cells - 64 - int(rng.integers(0, 30))
    p.fill(0, T, 0, range(n_seq))
    P = T              # next position to be accepted (T counts dense cells, P positions)
    runs = []          # (positions, seqs, ids) of the runs in flight
    n_ops = 200 if n_cells < 5000 else 70
    # place, copy, remove, end a run, accept, mask, compact
    menu = [1] * 6 + [2] * 2 + [3] + [4] * 2 + [5] * 4 + [6] * 3 + [7] * 2

    def end_run(k):
        for s in runs.pop(k)[2]:
            p.release(s)

    for step in range(n_ops):
        op = menu[int(rng.integers(len(menu)))]
        wb = max(0, min(n_cells - 1, T + int(rng.integers(-3, 12))))
        if op == 1:
            n = int(rng.integers(1, 17))
            parent = synth.random_tree(seed, step, n) if rng.integers(2) else np.arange(-1, n - 1)
            ids = [p.acquire() for _ in range(synth.n_leaves(parent))]
            if None in ids:                                                # not enough partitions: give them back
                for s in ids:
                    if s is not None:
                        p.release(s)
                continue
            seqs = synth.tree_sequences(parent, ids)
            p0 = P + (int(rng.integers(0, 6)) if rng.integers(3) == 0 else 0)
            positions = synth.tree_run(parent, p0, p0)["positions"].tolist()
            st, _ = p.place(positions, seqs, wb)
            if st == 0:
                runs.append((positions, seqs, ids))
            else:
                for s in ids:
                    p.release(s)
        elif op == 2 and len(runs) >= 2:
            i, j = rng.choice(len(runs), 2, replace=False)
            if rng.integers(4):                                            # early sharing: what lies before run j's start
                p.seq_cp(runs[i][2][0], runs[j][2], 0, min(runs[j][0]))
            else:
                p.seq_cp(runs[i][2][0], runs[j][2], P + int(rng.integers(0, 3)), P + int(rng.integers(3, 20)))
        elif op == 3 and runs:
            p.seq_rm(runs[int(rng.integers(len(runs)))][2][:1], P + int(rng.integers(1, 10)))
        elif op == 4 and runs:
            end_run(int(rng.integers(len(runs))))
        elif op == 5 and runs:
            k = int(rng.integers(len(runs)))
            positions, seqs, ids = runs[k]
            if min(positions) == P:
                # an accepted path: walk down a branch from a token at the accepted end
                order = np.argsort(positions, kind="stable")
                a = int(rng.integers(0, min(4, len(positions)) + 1))
                path = [int(order[0])]
                for i in order[1:]:
                    if len(path) >= a:
                        break
                    if positions[i] == positions[path[-1]] + 1 and set(seqs[i]) <= set(seqs[path[-1]]):
                        path.append(int(i))
                p.accept(positions, seqs, path[:a])
                if path[:a]:
                    P = positions[path[:a][-1]] + 1
            end_run(k)
        elif op == 6:
            n = int(rng.integers(1, 17))
            seqs = [[int(rng.integers(0, n_seq))] + ([int(rng.integers(0, n_seq))] if rng.integers(2) else []) for _ in range(n)]
            positions = [P + int(rng.integers(-2, 20)) for _ in range(n)]
            prefix = max(0, min(n_cells, T + int(rng.integers(-2, 3))))
            p.build_mask(positions, seqs, prefix, wb)
        elif op == 7:
            if rng.integers(2):                                            # give compaction a chance: end every run
                while runs:
                    end_run(0)
            st, dense = p.compact(T)
            if st == 0:
                T = dense
        p.check("step %d (op %d)" % (step, op))
    while runs:
        end_run(0)
    st, dense = p.compact(T)
    p.check("final compaction")
    pos, seq = p.g.read()
    if st == 0:      # (a copy into a rival run can leave two accepted entries at one position: then it is refused)
        assert all(pos[c] >= 0 and seq[c] & 1 for c in range(dense))      # a dense canonical prefix ...
        assert not (pos[dense:min(n_cells, T + 64)] >= 0).any()            # ... and a free window behind it


# ---- compaction moves the cache data -----------------------------------------------------------------

@pytest.mark.parametrize("shape_name", ["tiny", "tiny_bf16", "tiny_gqa"])
def test_compaction_moves_every_layer_of_the_cache(shape_name):
    sh = synth.SHAPES[shape_name]
    n_cells, T = 96, 10
    gm = gpu_loader.load_model(sh, 0, 0.0)
    gkv = pi.KVCache(gm, n_cells)
    okv = oracle.OracleKV(sh, n_cells)
    for l in range(sh.n_layers):
        k, v = synth.kv_prefill_host(sh, 11, l, n_cells)               # every cell holds distinct data
        okv.set_cells(l, 0, k, v)
        gkv.set_cells(l, 0, k, v)
    gkv.set_len(T)
    p = Pair(n_cells, 6)
    p.fill(0, T, 0, range(6))
    scattered = [(T + 40, T + 2), (T + 3, T + 1), (T + 63, T + 4), (T + 17, T), (T + 18, T + 3)]
    for cell, pos in scattered:
        p.fill(cell, 1, pos, range(6))
    s = p.acquire()
    p.place([T + 5], [[s]], T)
    before = gkv.raw().copy()
    assert p.compact(T, gkv, okv.K, okv.V)[0] == pi.PI_E_BUSY
    assert np.array_equal(gkv.raw(), before) and len(gkv) == T
    p.release(s)
    st, dense = p.compact(T, gkv, okv.K, okv.V)
    assert (st, dense) == (0, T + 5) and len(gkv) == T + 5
    p.check("compaction")
    for l in range(sh.n_layers):
        k, v = gkv.get_cells(l, 0, n_cells)
        assert np.array_equal(k.astype(np.float64), okv.K[l]) and np.array_equal(v.astype(np.float64), okv.V[l])
    pos, _ = p.g.read()
    assert pos[:T + 5].tolist() == list(range(T + 5))                  # cell index == position again
    gm.free()


# ---- runs that share the cache, end to end ---------------------------------------------------------------

TOL = {"f32": ("abs", 1e-4), "bf16": ("rel", 2e-2)}


def _close(gpu, ref, dtype):
    kind, tol = TOL[dtype]
    err = float(np.max(np.abs(gpu - ref))) if kind == "abs" else max_rel_rowwise(gpu, ref)
    assert err <= tol, "logit error %g > %g" % (err, tol)


def _device_run(p, gm, gkv, om, okv, tokens, positions, seqs, prefix_len, window_base, parent=None):
    """Place and mask on both sides, run the forward on both with each side's own slots and
    masks, compare logits.  Returns (device Run, oracle run dict, gpu logits, oracle logits)."""
    sh = gm.shape
    n = len(positions)
    st, slots = p.place(positions, seqs, window_base)
    assert st == 0
    mask, bad = p.build_mask(positions, seqs, prefix_len, window_base)
    assert bad == 0
    orun = {"positions": np.asarray(positions, dtype=np.int32), "slots": slots.cpu().numpy(),
            "mask": mask.cpu().numpy().view(np.uint64), "prefix_len": prefix_len, "window_base": window_base}
    ref = oracle.stage_forward(om, okv, orun, 0, sh.n_layers, tokens=tokens)["logits"]
    run = pi.Run(tokens, positions, np.zeros(n, dtype=np.int32), np.zeros(n, dtype=np.uint64), prefix_len, window_base,
                 parent=parent)
    run.slots, run.mask = slots, mask                     # the device results, never copied to the host
    logits = torch.full((n, sh.vocab), float("nan"), device="cuda")
    status = torch.full((2,), -99, dtype=torch.int32, device="cuda")
    pi.stage_forward(gm, gkv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
    lg = logits.cpu().numpy()
    _close(lg, ref, sh.dtype)
    return run, orun, logits, ref


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_bf16", "tiny_gqa"])
def test_chained_rival_and_tree_runs_share_the_cache(shape_name):
    """A (4 tokens) speculates; B continues A before A is verified; R is a rival of A at the
    same positions; a tree run D hangs under the prefix.  Acceptance is decided on the device
    (verify -> accept), partitions are released, holes are reused, and a last run C sees the
    accepted entries where they lie.  Logits of every run, the tables and the final dense
    prefix agree with the oracle."""
    sh = synth.SHAPES[shape_name]
    n_cells, T = 128, 24
    om = from_synth.model_from_seed(sh, 0, 0.1)
    okv = from_synth.kv_synthetic(sh, 3, n_cells, T)
    gm = gpu_loader.load_model(sh, 0, 0.1)
    gkv = pi.KVCache(gm, n_cells)
    gpu_loader.prefill_kv_synthetic(gkv, sh, 3, T)
    p = Pair(n_cells, 12)
    p.fill(0, T, 0, range(12))
    toks = synth.tokens_host(sh, 5, 8, synth.T_DRAFT)
    a, b, r = p.acquire(), p.acquire(), p.acquire()

    pos_a = [T, T + 1, T + 2, T + 3]
    run_a, _, lg_a, ref_a = _device_run(p, gm, gkv, om, okv, toks[:4], pos_a, [[a]] * 4, T, T)
    p.seq_cp(a, [b])
    pos_b = [T + 4, T + 5, T + 6, T + 7]
    _device_run(p, gm, gkv, om, okv, toks[4:], pos_b, [[b]] * 4, T, T)
    # B's logits equal the tail of one 8-token causal batch (the oracle side of this is pinned on the CPU)
    rival_toks = synth.tokens_host(sh, 6, 4, synth.T_DRAFT)
    _device_run(p, gm, gkv, om, okv, rival_toks, pos_a, [[r]] * 4, T, T)

    parent = synth.random_tree(2, 9, 9)
    ids = [p.acquire() for _ in range(synth.n_leaves(parent))]
    assert None not in ids
    seqs_d = synth.tree_sequences(parent, ids)
    trun = synth.tree_run(parent, T, T)
    tree_toks = synth.sibling_distinct_tokens(sh, 4, 1, parent)
    run_d, orun_d, _, _ = _device_run(p, gm, gkv, om, okv, tree_toks, trun["positions"].tolist(), seqs_d, T, T,
                                      parent=parent)
    # the device mask of the tree equals the ancestor mask, moved to the cells the tokens got
    slots_d = orun_d["slots"]
    for i in range(9):
        want, j = 0, i
        while j >= 0:
            want |= 1 << int(slots_d[j] - T)
            j = int(parent[j])
        assert int(orun_d["mask"][i]) == want
    p.check("four runs in flight")

    # A is verified on the device.  Only the bookkeeping is under test here, so the draft is
    # rewritten after the forward such that exactly two tokens are accepted.
    draft = np.array(toks[:4], dtype=np.int32)
    root_expected = int(draft[0])
    draft[1] = int(np.argmax(ref_a[0]))
    draft[2] = (int(np.argmax(ref_a[1])) + 1) % sh.vocab
    planted = np.asarray(ref_a, dtype=np.float32).copy()   # verification is separate from the forward here
    acc = torch.full((4,), -7, dtype=torch.int32, device="cuda")
    res = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    pi.verify_greedy(dev_i32(draft), None, 4, torch.as_tensor(planted, device="cuda"), sh.vocab, root_expected, acc, res)
    a_ref, acc_ref, _ = oracle.verify_greedy(draft, None, planted, root_expected)
    assert a_ref == 2
    p.g.accept(4, dev_i32(pos_a), dev_sets([[a]] * 4), acc, res)          # device outputs straight in
    p.o.accept(pos_a, [[a]] * 4, acc_ref)
    p.check("accept from device results")
    for s in [a, b, r] + ids:
        p.release(s)
    p.check("all partitions released")
    pos, seq = p.g.read()
    assert pos[:T + 2].tolist() == list(range(T + 2)) and not (pos[T + 2:] >= 0).any()

    # C continues after the two accepted tokens; its cells reuse the holes
    c = p.acquire()
    toks_c = synth.tokens_host(sh, 8, 3, synth.T_DRAFT)
    okv.kv_len = T
    _device_run(p, gm, gkv, om, okv, toks_c, [T + 2, T + 3, T + 4], [[c]] * 3, T, T)
    p.release(c)
    st, dense = p.compact(T, gkv, okv.K, okv.V)
    assert (st, dense) == (0, T + 2) and len(gkv) == T + 2
    gm.free()
