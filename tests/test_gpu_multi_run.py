"""GPU parity of several speculative runs sharing one weight pass (pi_stage_forward_multi): the
runs of a micro-batch are the trees of a forest under the shared prefix, so by tree isolation
(pinned for the oracle on the CPU) the oracle's logits of the whole forest are the logits of each
run evaluated alone; each run has its own cancel word and status."""
import numpy as np
import pytest
import torch

import synth
import oracle
from oracle import from_synth
from synth import gpu_loader
import paper_2407_11798_amd as pi
from gpu_common import max_rel_rowwise

pytestmark = pytest.mark.gpu

# four runs: a chain of 3, a 4-node tree, a single token, a 2-chain  (10 tokens)
PARENT = np.array([-1, 0, 1, -1, 3, 3, 4, -1, -1, 8], dtype=np.int32)
GROUP = [0, 0, 0, 1, 1, 1, 1, 2, 3, 3]


def _tol_ok(gpu, ref, dtype):
    if dtype == "f32":
        return float(np.max(np.abs(gpu - ref))) <= 1e-4
    return max_rel_rowwise(gpu, ref) <= 2e-2


def _setup(shape_name, n_prefill=24, n_cells=96, seed=0, gain_sigma=0.1):
    sh = synth.SHAPES[shape_name]
    om = from_synth.model_from_seed(sh, seed, gain_sigma)
    okv = from_synth.kv_synthetic(sh, seed, n_cells, n_prefill)
    gm = gpu_loader.load_model(sh, seed, gain_sigma)
    gkv = pi.KVCache(gm, n_cells)
    gpu_loader.prefill_kv_synthetic(gkv, sh, seed, n_prefill)
    return sh, om, okv, gm, gkv


def _cells_of(group):
    return [i for i, g in enumerate(GROUP) if g == group]


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_bf16", "tiny_gqa"])
def test_runs_sharing_a_pass_match_the_oracle(shape_name):
    sh, om, okv, gm, gkv = _setup(shape_name)
    n = len(PARENT)
    rd = synth.tree_run(PARENT, 24, 24, offset=5)
    toks = synth.tokens_host(sh, 11, n, synth.T_DRAFT)
    o2 = okv.clone()
    ref = oracle.stage_forward(om, o2, rd, 0, sh.n_layers, tokens=toks)["logits"]
    run = gpu_loader.make_run(rd, toks)
    logits = torch.full((n, sh.vocab), float("nan"), device="cuda")
    status = torch.full((2,), -9, dtype=torch.int32, device="cuda")
    gstat = torch.full((4, 2), -9, dtype=torch.int32, device="cuda")
    flags = torch.zeros(4, dtype=torch.int32, device="cuda")
    pi.stage_forward_multi(gm, gkv, run, GROUP, 0, sh.n_layers, logits_out=logits, cancel_flags=flags,
                           group_status=gstat, run_status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
    assert gstat.cpu().tolist() == [[pi.PI_OK, sh.n_layers]] * 4
    assert _tol_ok(logits.cpu().numpy(), ref, sh.dtype)
    # identical bits to the same micro-batch issued as one run
    pi.kv_rollback(gkv, run.slots, n)
    logits1 = torch.empty_like(logits)
    pi.stage_forward(gm, gkv, run, 0, sh.n_layers, logits_out=logits1, run_status=status)
    torch.cuda.synchronize()
    assert torch.equal(logits, logits1)
    gm.free()


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_gqa"])
def test_one_run_is_cancelled_and_the_others_finish(shape_name):
    """Deterministic cancellation of runs 1 and 3 before layer `stop` (flags stored in-stream
    between two stage calls): their cells hold K/V of the layers below `stop` only, their status
    says so, and the logits of runs 0 and 2 are those of the undisturbed pass."""
    sh, om, okv, gm, gkv = _setup(shape_name)
    n = len(PARENT)
    rd = synth.tree_run(PARENT, 24, 24, offset=5)
    toks = synth.tokens_host(sh, 11, n, synth.T_DRAFT)
    snapshot = gkv.raw().copy()
    o2 = okv.clone()
    ref = oracle.stage_forward(om, o2, rd, 0, sh.n_layers, tokens=toks)["logits"]
    first_cell = int(rd["slots"][0])
    for stop in range(1, sh.n_layers):
        run = gpu_loader.make_run(rd, toks)
        hidden = torch.zeros((n, sh.d_model), device="cuda")
        logits = torch.full((n, sh.vocab), float("nan"), device="cuda")
        status = torch.full((2,), -9, dtype=torch.int32, device="cuda")
        gstat = torch.full((4, 2), -9, dtype=torch.int32, device="cuda")
        flags = torch.zeros(4, dtype=torch.int32, device="cuda")
        pi.stage_forward_multi(gm, gkv, run, GROUP, 0, stop, hidden_out=hidden, cancel_flags=flags,
                               group_status=gstat, run_status=status)
        flags[1] = 1
        flags[3] = 1
        pi.stage_forward_multi(gm, gkv, run, GROUP, stop, sh.n_layers, hidden_in=hidden, logits_out=logits,
                               cancel_flags=flags, group_status=gstat, run_status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
        assert gstat.cpu().tolist() == [[pi.PI_OK, sh.n_layers], [pi.PI_CANCELLED, stop],
                                        [pi.PI_OK, sh.n_layers], [pi.PI_CANCELLED, stop]]
        lg = logits.cpu().numpy()
        alive = _cells_of(0) + _cells_of(2)
        assert _tol_ok(lg[alive], ref[alive], sh.dtype)
        for l in range(sh.n_layers):
            k, v = gkv.get_cells(l, first_cell, n)
            for g in range(4):
                written = l < stop or g in (0, 2)
                for i in _cells_of(g):
                    assert bool(k[i].any()) == written and bool(v[i].any()) == written
                    if written:                      # the cells that were written hold the oracle's K/V
                        ok = o2.K[l, first_cell + i]
                        assert np.max(np.abs(k[i] - ok)) <= (1e-4 if sh.dtype == "f32" else 2e-2 * np.max(np.abs(ok)))
        pi.kv_rollback(gkv, run.slots, n)
        assert np.array_equal(gkv.raw(), snapshot)
    gm.free()


def test_every_run_cancelled_stops_the_pass():
    sh, om, okv, gm, gkv = _setup("tiny")
    n = len(PARENT)
    rd = synth.tree_run(PARENT, 24, 24, offset=5)
    toks = synth.tokens_host(sh, 11, n, synth.T_DRAFT)
    run = gpu_loader.make_run(rd, toks)
    logits = torch.full((n, sh.vocab), 7.0, device="cuda")
    status = torch.full((2,), -9, dtype=torch.int32, device="cuda")
    gstat = torch.full((4, 2), -9, dtype=torch.int32, device="cuda")
    flags = torch.ones(4, dtype=torch.int32, device="cuda")
    pi.stage_forward_multi(gm, gkv, run, GROUP, 0, sh.n_layers, logits_out=logits, cancel_flags=flags,
                           group_status=gstat, run_status=status)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [pi.PI_CANCELLED, 0]
    assert gstat.cpu().tolist() == [[pi.PI_CANCELLED, 0]] * 4
    assert torch.all(logits == 7.0)
    # arguments that do not describe runs are refused on the host
    with pytest.raises(pi.PiError):
        pi.stage_forward_multi(gm, gkv, run, [0] * (n - 1) + [2], 0, sh.n_layers, logits_out=logits)  # run 1 empty
    gm.free()
