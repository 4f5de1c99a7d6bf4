"""GPU parity on the tiny configurations: HIP path vs the CPU oracle, element by element."""
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

TOL = {"f32": ("abs", 1e-4), "bf16": ("rel", 2e-2)}


def check_logits(gpu, ref, dtype):
    kind, tol = TOL[dtype]
    if kind == "abs":
        err = float(np.max(np.abs(gpu - ref)))
    else:
        err = max_rel_rowwise(gpu, ref)
    assert err <= tol, "logit error %g > %g" % (err, tol)
    return err


def test_device_fill_equals_host_fill():
    # block-scaled 4-bit matrices: codes and scales, a ragged last block per row
    rows, cols = 37, 688
    nc, ns = synth.fp4b_sizes(rows, cols)
    t = torch.empty(nc + ns, dtype=torch.uint8, device="cuda")
    sid = synth.stream_id(synth.T_WG, 3)
    assert synth.hip_lib().synth_fill_normal_fp4b_device(t.data_ptr(), t.data_ptr() + nc, rows, cols, 5, sid, 0.02,
                                                         torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert np.array_equal(t.cpu().numpy(), synth.normal_fp4b_host(rows, cols, 5, sid, 0.02))
    for dtype in ("f32", "bf16", "fp8", "fp4"):
        n = 1_000_003 if dtype != "fp4" else 1_000_004        # two 4-bit values per byte
        sid = synth.stream_id(synth.T_WD, 7)
        sigma = 0.02 * {"fp8": 2048, "fp4": 64}.get(dtype, 1)  # quantised weights are stored scaled up
        host = synth.normal_host(n, 3, sid, sigma, dtype)
        dev = gpu_loader.device_normal(n, 3, sid, sigma, dtype).cpu().numpy()
        if dtype == "bf16":
            dev = dev.view(np.uint16)
        assert np.array_equal(host, dev)


def _true_prefill(sh, seed, gain_sigma, n_prefill, n_cells):
    """Prefill both sides by running the prompt tokens through each path's own forward."""
    om = from_synth.model_from_seed(sh, seed, gain_sigma)
    okv = oracle.OracleKV(sh, n_cells)
    gm = gpu_loader.load_model(sh, seed, gain_sigma)
    gkv = pi.KVCache(gm, n_cells)
    toks = synth.tokens_host(sh, seed, n_prefill)
    last_o = last_g = None
    for b0 in range(0, n_prefill, 16):
        nb = min(16, n_prefill - b0)
        run = synth.linear_run(nb, b0)
        last_o = oracle.stage_forward(om, okv, run, 0, sh.n_layers, tokens=toks[b0:b0 + nb])["logits"]
        oracle.kv_rollback(okv, run["slots"], list(range(nb)))
        st, done, last_g, _, grun = forward(gm, gkv, run, toks[b0:b0 + nb])
        assert (st, done) == (pi.PI_OK, sh.n_layers)
        acc = torch.arange(nb, dtype=torch.int32, device="cuda")
        res = torch.tensor([nb, 0], dtype=torch.int32, device="cuda")
        pi.kv_rollback(gkv, grun.slots, nb, acc, res)
        torch.cuda.synchronize()
        check_logits(last_g, last_o, sh.dtype)
    assert len(gkv) == okv.kv_len == n_prefill
    return om, okv, gm, gkv, last_o, last_g


@pytest.mark.parametrize("shape_name,gain_sigma", [("tiny", 0.0), ("tiny", 0.1), ("tiny_bf16", 0.1), ("tiny_gqa", 0.1),
                                                   ("tiny_w8", 0.1), ("tiny_gqa_w8", 0.1), ("tiny_w4", 0.1),
                                                   ("tiny_gqa_w4", 0.1), ("tiny_w4b", 0.1), ("tiny_gqa_w4b", 0.1)])
def test_planted_draft_verify_and_rollback(shape_name, gain_sigma):
    """Tiny configuration: 64 prefilled positions, 4 draft tokens planted to agree with the
    oracle's argmax for the first 2; accepted count, bonus token and kv_len must match."""
    sh = synth.SHAPES[shape_name]
    om, okv, gm, gkv, pre_o, pre_g = _true_prefill(sh, 0, gain_sigma, 64, 128)
    # cache contents agree (prefill itself is a parity test)
    for l in range(sh.n_layers):
        k, v = gkv.get_cells(l, 0, 64)
        # fp32 cache: arithmetic error only; bf16 cache: at most one rounding step of a value of this size
        tol = 5e-5 if sh.dtype == "f32" else 2.0 ** -7 * max(np.abs(okv.K[l, :64]).max(), np.abs(okv.V[l, :64]).max())
        assert np.max(np.abs(k - okv.K[l, :64])) <= tol
        assert np.max(np.abs(v - okv.V[l, :64])) <= tol
    root_expected = int(np.argmax(pre_o[-1]))
    d = np.zeros(4, dtype=np.int32)
    d[0] = root_expected
    l0 = oracle.stage_forward(om, okv.clone(), synth.linear_run(1, 64), 0, sh.n_layers, tokens=d[:1])["logits"]
    d[1] = int(np.argmax(l0[0]))
    l1 = oracle.stage_forward(om, okv.clone(), synth.linear_run(2, 64), 0, sh.n_layers, tokens=d[:2])["logits"]
    d[2] = (int(np.argmax(l1[1])) + 1) % sh.vocab
    d[3] = int(synth.tokens_host(sh, 0, 1, synth.T_DRAFT)[0])
    run = synth.linear_run(4, 64)
    ref = oracle.stage_forward(om, okv, run, 0, sh.n_layers, tokens=d)["logits"]
    st, done, lg, _, grun = forward(gm, gkv, run, d)
    assert (st, done) == (pi.PI_OK, sh.n_layers)
    check_logits(lg, ref, sh.dtype)
    a_ref, acc_ref, bonus_ref = oracle.verify_greedy(d, run["parent"], ref.astype(np.float32), root_expected)
    assert a_ref == 2
    acc, res = verify(grun, d, lg, sh.vocab, root_expected)
    gaps = [oracle.top2_gap(ref[i]) for i in range(4)]
    # the planted rows are decisive in every configuration here (smallest gap 5e-3): no exemption
    assert TieBudget(0).decisive(gaps[:2])
    assert res.cpu().tolist() == [a_ref, bonus_ref]
    assert acc.cpu().tolist()[:a_ref] == acc_ref and acc.cpu().tolist()[a_ref:] == [-1, -1]
    pi.kv_rollback(gkv, grun.slots, 4, acc, res)
    oracle.kv_rollback(okv, run["slots"], acc_ref)
    assert len(gkv) == okv.kv_len == 66
    for l in range(sh.n_layers):
        k, v = gkv.get_cells(l, 64, 64)
        assert not k[2:].any() and not v[2:].any()          # rejected cells are free again
        # the committed cells: arithmetic error only (fp32 cache) or one rounding step (bf16 cache)
        tol = 5e-5 if sh.dtype == "f32" else 2.0 ** -7 * max(np.abs(okv.K[l, 64:66]).max(), np.abs(okv.V[l, 64:66]).max())
        assert np.max(np.abs(k[:2] - okv.K[l, 64:66])) <= tol
        assert np.max(np.abs(v[:2] - okv.V[l, 64:66])) <= tol
    gm.free()
