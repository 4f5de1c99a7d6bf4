"""GPU parity of whole verification runs on the small configurations: trees, stage slices,
batch-vs-sequential equivalence, cancellation, and misuse of live cells."""
import ctypes

import numpy as np
import pytest
import torch

import synth
import oracle
from oracle import from_synth
from synth import gpu_loader
import paper_2407_11798_amd as pi
from gpu_common import forward, verify, max_rel_rowwise, TieBudget

pytestmark = pytest.mark.gpu


def _tol_ok(gpu, ref, dtype):
    if dtype == "f32":
        return float(np.max(np.abs(gpu - ref))) <= 1e-4
    return max_rel_rowwise(gpu, ref) <= 2e-2


def _setup(shape_name, n_prefill, n_cells, gain_sigma=0.1, seed=0):
    sh = synth.SHAPES[shape_name]
    om = from_synth.model_from_seed(sh, seed, gain_sigma)
    okv = from_synth.kv_synthetic(sh, seed, n_cells, n_prefill)
    gm = gpu_loader.load_model(sh, seed, gain_sigma)
    gkv = pi.KVCache(gm, n_cells)
    gpu_loader.prefill_kv_synthetic(gkv, sh, seed, n_prefill)
    return sh, om, okv, gm, gkv


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_bf16", "tiny_gqa"])
def test_token_trees_match_oracle_and_verify(shape_name):
    """Random trees (branching <= 3, depth <= 4) at several sizes incl. the largest batch; runs
    are placed at different offsets inside the 64-cell window."""
    sh, om, okv, gm, gkv = _setup(shape_name, 40, 112)
    ties = TieBudget(1)
    for trial, (n, offset) in enumerate([(1, 0), (4, 0), (4, 12), (7, 3), (16, 0), (16, 48), (13, 17)]):
        parent = synth.random_tree(1, trial, n)
        toks = synth.sibling_distinct_tokens(sh, 1, trial, parent)
        rd = synth.tree_run(parent, 40, 40, offset=offset)
        ref = oracle.stage_forward(om, okv.clone(), rd, 0, sh.n_layers, tokens=toks)["logits"]
        st, done, lg, _, grun = forward(gm, gkv, rd, toks)
        assert (st, done) == (pi.PI_OK, sh.n_layers)
        assert _tol_ok(lg, ref, sh.dtype)
        root_expected = int(toks[0])
        a, acc, bonus = oracle.verify_greedy(toks, parent, ref.astype(np.float32), root_expected)
        gacc, gres = verify(grun, toks, lg, sh.vocab, root_expected)
        if ties.decisive([oracle.top2_gap(ref[i]) for i in acc]):
            assert gres.cpu().tolist() == [a, bonus]
        pi.kv_rollback(gkv, grun.slots, n)               # discard: keep the prefix for the next trial
        assert len(gkv) == 40
    gm.free()


def test_tree_siblings_are_invisible_bit_for_bit():
    """Changing a token that is not an ancestor of node i leaves logits[i] bit-identical."""
    sh, om, okv, gm, gkv = _setup("tiny_gqa", 24, 96)
    parent = np.array([-1, 0, 0, 1, -1, 4], dtype=np.int32)
    rd = synth.tree_run(parent, 24, 24)
    toks = np.array([5, 6, 7, 8, 9, 10], dtype=np.int32)
    _, _, base, _, grun = forward(gm, gkv, rd, toks)
    pi.kv_rollback(gkv, grun.slots, 6)
    t2 = toks.copy()
    t2[2], t2[4], t2[5] = 300, 301, 302                   # not ancestors of nodes 0, 1, 3
    _, _, pert, _, grun = forward(gm, gkv, rd, t2)
    for i in (0, 1, 3):
        assert np.array_equal(base[i], pert[i])
    assert not np.array_equal(base[2], pert[2])
    gm.free()


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_gqa"])
def test_stage_slices_equal_whole_stack(shape_name):
    sh, om, okv, gm, gkv = _setup(shape_name, 16, 96)
    rd = synth.linear_run(5, 16)
    toks = synth.tokens_host(sh, 3, 5, synth.T_DRAFT)
    ref = oracle.stage_forward(om, okv.clone(), rd, 0, sh.n_layers, tokens=toks)
    _, _, whole, _, grun = forward(gm, gkv, rd, toks)
    pi.kv_rollback(gkv, grun.slots, 5)
    st, done, lg, hid, grun = forward(gm, gkv, rd, toks, 0, 1)
    assert (st, done) == (pi.PI_OK, 1) and lg is None
    href = oracle.stage_forward(om, okv.clone(), rd, 0, 1, tokens=toks)["hidden"]
    assert np.max(np.abs(hid - href)) <= (1e-4 if sh.dtype == "f32" else 2e-2 * np.max(np.abs(href)))
    st, done, lg, _, grun = forward(gm, gkv, rd, None, 1, sh.n_layers, hidden_in=hid)
    assert (st, done) == (pi.PI_OK, sh.n_layers)
    assert np.array_equal(lg, whole)                      # same arithmetic, same order: identical bits
    assert _tol_ok(lg, ref["logits"], sh.dtype)
    gm.free()


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_bf16"])
def test_batch_equals_sequential_steps_on_gpu(shape_name):
    """Verifying n tokens in one masked batch equals n single-token steps (logits within the
    tolerance, committed K/V cells bit-equal because the projection order does not depend on n)."""
    sh, om, okv, gm, gkv = _setup(shape_name, 20, 96)
    toks = synth.tokens_host(sh, 5, 6, synth.T_DRAFT)
    rd = synth.linear_run(6, 20)
    _, _, batch, _, grun = forward(gm, gkv, rd, toks)
    acc = torch.arange(6, dtype=torch.int32, device="cuda")
    res = torch.tensor([6, 0], dtype=torch.int32, device="cuda")
    pi.kv_rollback(gkv, grun.slots, 6, acc, res)
    raw_batch = gkv.raw().copy()
    gkv2 = pi.KVCache(gm, 96)
    gpu_loader.prefill_kv_synthetic(gkv2, sh, 0, 20)
    for i in range(6):
        r1 = synth.linear_run(1, 20 + i)
        _, _, li, _, g1 = forward(gm, gkv2, r1, toks[i:i + 1])
        tol = 1e-5 if sh.dtype == "f32" else 2e-3 * np.max(np.abs(batch[i]))
        assert np.max(np.abs(li[0] - batch[i])) <= tol
        pi.kv_rollback(gkv2, g1.slots, 1, acc[:1], torch.tensor([1, 0], dtype=torch.int32, device="cuda"))
    assert len(gkv) == len(gkv2) == 26
    assert np.array_equal(raw_batch, gkv2.raw())
    gm.free()


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_gqa"])
def test_cancel_at_every_layer_boundary(shape_name):
    """Deterministic cancellation: the stack is issued as [0, l) then [l, L) with the flag stored
    in-stream between the two calls, so the run must stop before layer l; after the discard the
    whole cache image is bit-identical to never having run, and a later run is unaffected."""
    sh, om, okv, gm, gkv = _setup(shape_name, 16, 96)
    rd = synth.linear_run(4, 16)
    toks = synth.tokens_host(sh, 7, 4, synth.T_DRAFT)
    snapshot = gkv.raw().copy()
    _, _, ref_logits, _, grun = forward(gm, gkv, rd, toks)
    pi.kv_rollback(gkv, grun.slots, 4)
    assert np.array_equal(gkv.raw(), snapshot)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    for stop in range(sh.n_layers + 0):
        flag.zero_()
        run = gpu_loader.make_run(rd, toks)
        hidden = torch.zeros((4, sh.d_model), device="cuda")
        logits = torch.full((4, sh.vocab), 7.0, device="cuda")
        status = torch.full((2,), -9, dtype=torch.int32, device="cuda")
        if stop > 0:
            pi.stage_forward(gm, gkv, run, 0, stop, hidden_out=hidden, cancel_flag=flag, run_status=status)
        flag.fill_(1)                                     # in-stream store between the two stage calls
        pi.stage_forward(gm, gkv, run, stop, sh.n_layers, hidden_in=hidden if stop > 0 else None,
                         logits_out=logits, cancel_flag=flag, run_status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_CANCELLED, stop]
        assert torch.all(logits == 7.0)                   # outputs untouched
        o2 = okv.clone()
        out = oracle.stage_forward(om, o2, rd, 0, sh.n_layers, tokens=toks, cancel_before_layer=stop)
        assert out["layers_done"] == stop
        for l in range(sh.n_layers):                      # K/V written exactly for the layers that ran
            k, _ = gkv.get_cells(l, 16, 4)
            assert bool(k.any()) == (l < stop)
        pi.kv_rollback(gkv, run.slots, 4)
        assert len(gkv) == 16 and np.array_equal(gkv.raw(), snapshot)
    _, _, again, _, grun = forward(gm, gkv, rd, toks)
    assert np.array_equal(again, ref_logits)
    gm.free()


def test_cancel_mid_run_from_the_host():
    """A mapped host word set by the host while the kernel runs: the run either finishes or stops
    at a layer boundary; either way the reported layers_done is consistent with the cache."""
    sh, om, okv, gm, gkv = _setup("tiny_gqa", 16, 96)
    rd = synth.linear_run(4, 16)
    toks = synth.tokens_host(sh, 7, 4, synth.T_DRAFT)
    snapshot = gkv.raw().copy()
    flag_host = torch.zeros(1, dtype=torch.int32, pin_memory=True)
    hip = ctypes.CDLL("libamdhip64.so")
    dev_ptr = ctypes.c_void_p()
    assert hip.hipHostGetDevicePointer(ctypes.byref(dev_ptr), ctypes.c_void_p(flag_host.data_ptr()), 0) == 0
    for when in ("before", "during"):
        flag_host[0] = 1 if when == "before" else 0
        run = gpu_loader.make_run(rd, toks)
        logits = torch.zeros((4, sh.vocab), device="cuda")
        status = torch.full((2,), -9, dtype=torch.int32, device="cuda")
        pi.stage_forward(gm, gkv, run, 0, sh.n_layers, logits_out=logits, run_status=status,
                         cancel_flag_ptr=dev_ptr.value)
        flag_host[0] = 1
        torch.cuda.synchronize()
        st, done = status.cpu().tolist()
        assert (st == pi.PI_CANCELLED and 0 <= done < sh.n_layers) or (st == pi.PI_OK and done == sh.n_layers)
        if when == "before":
            assert (st, done) == (pi.PI_CANCELLED, 0)
        for l in range(sh.n_layers):
            k, _ = gkv.get_cells(l, 16, 4)
            assert bool(k.any()) == (l < done)
        pi.kv_rollback(gkv, run.slots, 4)
        assert np.array_equal(gkv.raw(), snapshot)
    gm.free()


def test_write_into_live_cell_is_refused():
    sh, om, okv, gm, gkv = _setup("tiny", 16, 96)
    snapshot = gkv.raw().copy()
    bad = synth.linear_run(3, 16, window_base=15)          # first slot is the last canonical cell
    run = gpu_loader.make_run(bad, np.array([1, 2, 3], dtype=np.int32))
    logits = torch.zeros((3, sh.vocab), device="cuda")
    status = torch.full((2,), -9, dtype=torch.int32, device="cuda")
    pi.stage_forward(gm, gkv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [pi.PI_E_SLOT_LIVE, 0]
    assert np.array_equal(gkv.raw(), snapshot)
    gm.free()


def test_barrier_numbers_wrap_around():
    """The grid barrier compares barrier numbers modulo 2^16: enough launches on one model to pass
    that point several times give the same bits as the first."""
    sh, om, okv, gm, gkv = _setup("tiny", 16, 96)
    rd = synth.linear_run(3, 16)
    toks = synth.tokens_host(sh, 5, 3, synth.T_DRAFT)
    run = gpu_loader.make_run(rd, toks)
    logits = torch.zeros((3, sh.vocab), device="cuda")
    status = torch.full((2,), -9, dtype=torch.int32, device="cuda")
    per_launch = 5 * sh.n_layers + 4
    launches = 2 * 65536 // per_launch + 50
    first = None
    for it in range(launches):
        pi.stage_forward(gm, gkv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
        pi.kv_rollback(gkv, run.slots, 3)
        if it == 0:
            torch.cuda.synchronize()
            first = logits.clone()
        if it % 2000 == 1999:
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
            assert torch.equal(logits, first)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
    assert torch.equal(logits, first)
    gm.free()


def test_plan_override_grows_the_cross_slice_buffer():
    """Asking for more column slices than the built-in plan needs more cross-slice tiles than were
    allocated at load: the override grows the buffer (it used to be written past its end), and the
    results stay within tolerance of the oracle for every split."""
    sh, om, okv, gm, gkv = _setup("tiny_bf16", 16, 96)
    rd = synth.linear_run(6, 16)
    toks = synth.tokens_host(sh, 9, 6, synth.T_DRAFT)
    ref = oracle.stage_forward(om, okv.clone(), rd, 0, sh.n_layers, tokens=toks)["logits"]
    for plan in [(1, 1, 1, 1, 1), (2, 2, 2, 2, 2), (1, 2, 1, 2, 1), (0, 0, 0, 0, 0)]:
        for phase, sk in enumerate(plan):
            gm.set_plan(phase, sk)
        st, done, lg, _, grun = forward(gm, gkv, rd, toks)
        assert (st, done) == (pi.PI_OK, sh.n_layers), plan
        assert _tol_ok(lg, ref, sh.dtype), plan
        pi.kv_rollback(gkv, grun.slots, 6)
    # attention units per 100 workgroups: few large units (all drawn by the first workgroups to arrive),
    # the built-in choice, several units per workgroup
    for share in (3, 0, 400):
        gm.set_plan(8, share)
        st, done, lg, _, grun = forward(gm, gkv, rd, toks)
        assert (st, done) == (pi.PI_OK, sh.n_layers), share
        assert _tol_ok(lg, ref, sh.dtype), share
        pi.kv_rollback(gkv, grun.slots, 6)
    gm.set_plan(8, 0)
    # a split that leaves a slice fewer tiles than the smallest ring is refused, not launched
    gm.set_plan(0, 8)
    with pytest.raises(pi.PiError) as err:
        forward(gm, gkv, rd, toks)
    assert err.value.status == pi.PI_E_SHAPE
    gm.set_plan(0, 0)
    st, done, lg, _, grun = forward(gm, gkv, rd, toks)
    assert (st, done) == (pi.PI_OK, sh.n_layers) and _tol_ok(lg, ref, sh.dtype)
    gm.free()
