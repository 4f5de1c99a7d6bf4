"""Full-size parity: the Llama-7B-shaped bf16 configuration in the launch shape bench.py times,
compared with values the CPU oracle stored under tests/golden/ (written by make_golden.py, which
calls only oracle/).  Sampled logits per row, the row argmax and the accepted counts are checked."""
import json
import os

import numpy as np
import pytest
import torch

import synth
from synth import gpu_loader
import paper_2407_11798_amd as pi
from gpu_common import TieBudget

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _load(name):
    path = os.path.join(GOLDEN, name + ".json")
    assert os.path.exists(path), "stored oracle values %s missing (written by tests/golden/make_golden.py)" % name
    with open(path) as f:
        return json.load(f)


def _load_full(name):
    """Per-row records (JSON) and whole float32 logits rows, hidden states and cells (.npz)."""
    meta = _load(name)
    path = os.path.join(GOLDEN, name + ".npz")
    assert os.path.exists(path), "stored oracle arrays %s missing (written by tests/golden/make_golden.py)" % name
    return meta, np.load(path, allow_pickle=False)


@pytest.fixture(scope="module")
def llama7b():
    sh = synth.SHAPES["llama7b"]
    m = gpu_loader.load_model(sh, 0)
    yield sh, m
    m.free()


def _check_rows(gpu_logits, rows, cols, dtype_tol=2e-2):
    worst = 0.0
    ties = TieBudget(max(1, len(rows) // 8))   # rows whose argmax is not compared: counted and capped
    for i, rec in enumerate(rows):
        got = gpu_logits[i]
        ref = np.asarray(rec["sample"])
        err = np.max(np.abs(got[cols] - ref)) / rec["maxabs"]
        worst = max(worst, err)
        assert err <= dtype_tol, "row %d: sampled logit error %g of the row's max |logit|" % (i, err)
        assert abs(float(np.max(np.abs(got))) - rec["maxabs"]) <= dtype_tol * rec["maxabs"]
        if ties.decisive([rec["gap"]]):
            assert int(np.argmax(got)) == rec["argmax"], "row %d argmax" % i
    return worst


def _check_full_rows(gpu_logits, ref_rows, recs, dtype_tol=2e-2):
    """Every column of every row against the stored oracle row."""
    ties = TieBudget(max(1, len(recs) // 8))
    ref = np.asarray(ref_rows, dtype=np.float64)
    got = np.asarray(gpu_logits, dtype=np.float64)
    assert got.shape == ref.shape
    err = np.max(np.abs(got - ref), axis=-1) / np.max(np.abs(ref), axis=-1)
    assert err.max() <= dtype_tol, "logit error %g of the row's max |logit| (row %d)" % (err.max(), int(err.argmax()))
    for i, rec in enumerate(recs):
        assert abs(float(np.max(np.abs(ref[i]))) - rec["maxabs"]) <= 1e-6 * rec["maxabs"]   # the two files belong together
        if ties.decisive([rec["gap"]]):
            assert int(np.argmax(got[i])) == rec["argmax"], "row %d argmax" % i
    return float(err.max())


def _cells_close(got, ref):
    """bf16 cache cells: at most one rounding step of a value of this size."""
    return np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) <= 2.0 ** -7 * np.max(np.abs(ref))


def test_llama7b_linear_runs_match_oracle(llama7b):
    sh, m = llama7b
    g = _load("llama7b_linear")
    T = g["prefix"]
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
    cols = np.asarray(g["cols"])
    for n_str, rec in g["runs"].items():
        n = int(n_str)
        toks = np.asarray(rec["tokens"], dtype=np.int32)
        assert np.array_equal(toks, synth.tokens_host(sh, g["seed"], n, synth.T_DRAFT, salt=n))
        run = gpu_loader.make_run(synth.linear_run(n, T), toks)
        logits = torch.zeros((n, sh.vocab), device="cuda")
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
        worst = _check_rows(logits.cpu().numpy(), rec["rows"], cols)
        print("n=%d worst sampled logit error / row max: %.2e" % (n, worst))
        pi.kv_rollback(kv, run.slots, n)
    torch.cuda.synchronize()
    assert len(kv) == T


def test_llama7b_every_logit_column_matches_oracle(llama7b):
    """Linear runs of 1 and 8 tokens: all 32000 columns of every row against stored oracle rows,
    and the run's own K/V cells in the first and the last layer."""
    sh, m = llama7b
    g, arr = _load_full("llama7b_full")
    T = g["prefix"]
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
    for n_str, rec in g["runs"].items():
        n = int(n_str)
        toks = np.asarray(rec["tokens"], dtype=np.int32)
        assert np.array_equal(toks, synth.tokens_host(sh, g["seed"], n, synth.T_DRAFT, salt=n))
        run = gpu_loader.make_run(synth.linear_run(n, T), toks)
        logits = torch.zeros((n, sh.vocab), device="cuda")
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
        worst = _check_full_rows(logits.cpu().numpy(), arr["logits_n%d" % n], rec["rows"])
        print("n=%d worst logit error / row max over all columns: %.2e" % (n, worst))
        for l in (0, sh.n_layers - 1):
            k, v = kv.get_cells(l, T, n)
            assert _cells_close(k, arr["k_n%d_layer%d" % (n, l)]) and _cells_close(v, arr["v_n%d_layer%d" % (n, l)])
        pi.kv_rollback(kv, run.slots, n)
    torch.cuda.synchronize()
    assert len(kv) == T


@pytest.mark.parametrize("shape_name", ["llama7b_w8", "llama7b_w4", "llama7b_w4b"])
def test_llama7b_with_quantised_weights_matches_oracle(shape_name):
    """The same shape with FP8 E4M3 (one byte per weight) or FP4 E2M1 (half a byte) weight
    matrices: sampled logits against the oracle evaluated on the dequantised weights."""
    sh = synth.SHAPES[shape_name]
    g = _load(shape_name + "_linear")
    m = gpu_loader.load_model(sh, g["seed"])
    layer_bytes, lm_bytes = m.weight_bytes()
    if sh.weight_format == "fp8":
        assert layer_bytes == sh.layer_params and lm_bytes == sh.vocab * sh.d_model  # one byte per weight
    else:   # half a byte per weight; the down projection's 86 tiles of 128 columns are padded to 88
        pad = sh.d_model * (88 * 128 - sh.ffn) // 2
        codes, lm_codes = sh.layer_params // 2 + pad, sh.vocab * sh.d_model // 2
        if sh.weight_format == "fp4b":   # and one scale byte per 32 columns: a sixteenth on top
            assert layer_bytes == codes + codes // 16 and lm_bytes == lm_codes + lm_codes // 16
        else:
            assert layer_bytes == codes and lm_bytes == lm_codes
    T = g["prefix"]
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
    cols = np.asarray(g["cols"])
    for n_str, rec in g["runs"].items():
        n = int(n_str)
        toks = np.asarray(rec["tokens"], dtype=np.int32)
        run = gpu_loader.make_run(synth.linear_run(n, T), toks)
        logits = torch.zeros((n, sh.vocab), device="cuda")
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
        worst = _check_rows(logits.cpu().numpy(), rec["rows"], cols)
        print("%s n=%d worst sampled logit error / row max: %.2e" % (shape_name, n, worst))
        pi.kv_rollback(kv, run.slots, n)
    m.free()


def test_llama7b_concurrent_runs_with_cancellation(llama7b):
    """Eight 4-token tree runs over a shared 1024-cell prefix; half are cancelled before a seeded
    layer (stack issued as two stage calls with the flag stored in between).  Survivors must match
    the oracle's logits, accepted counts and bonus tokens; the best run is committed, the others
    rolled back, and cancelled runs leave no trace in the cache."""
    sh, m = llama7b
    g = _load("llama7b_runs")
    T, n = g["prefix"], 4
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
    cols = np.asarray(g["cols"])
    snapshot = kv.raw().copy()
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    results = []
    for r, rec in enumerate(g["runs"]):
        parent = np.asarray(rec["parent"], dtype=np.int32)
        toks = np.asarray(rec["tokens"], dtype=np.int32)
        rd = synth.tree_run(parent, T, T, offset=n * r)
        run = gpu_loader.make_run(rd, toks)
        logits = torch.zeros((n, sh.vocab), device="cuda")
        hidden = torch.zeros((n, sh.d_model), device="cuda")
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        stop = g["cancel_before_layer"][r]
        flag.zero_()
        if stop < 0:
            pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=logits, cancel_flag=flag, run_status=status)
        else:
            if stop > 0:
                pi.stage_forward(m, kv, run, 0, stop, hidden_out=hidden, cancel_flag=flag, run_status=status)
            flag.fill_(1)
            pi.stage_forward(m, kv, run, stop, sh.n_layers, hidden_in=hidden if stop > 0 else None,
                             logits_out=logits, cancel_flag=flag, run_status=status)
        torch.cuda.synchronize()
        if stop >= 0:
            assert status.cpu().tolist() == [pi.PI_CANCELLED, stop]
            pi.kv_rollback(kv, run.slots, n)
            results.append((r, -1, None, run))
            continue
        assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
        _check_rows(logits.cpu().numpy(), rec["rows"], cols)
        acc = torch.zeros(n, dtype=torch.int32, device="cuda")
        res = torch.zeros(2, dtype=torch.int32, device="cuda")
        pi.verify_greedy(run.tokens, run.parent, n, logits, sh.vocab, g["root_expected"], acc, res)
        torch.cuda.synchronize()
        if all(rec["rows"][i]["gap"] >= 1e-3 for i in rec["accepted_nodes"]):
            assert res.cpu().tolist() == [rec["accepted"], rec["bonus"]]
            assert acc.cpu().tolist()[:rec["accepted"]] == rec["accepted_nodes"]
        results.append((r, int(res[0].item()), (acc, res), run))
    # commit the best surviving run (ties: lowest run index), discard the others
    best = max((x for x in results if x[1] >= 0), key=lambda x: (x[1], -x[0]))
    for r, a, ar, run in results:
        if a >= 0 and r != best[0]:
            pi.kv_rollback(kv, run.slots, n)
    pi.kv_rollback(kv, best[3].slots, n, best[2][0], best[2][1])
    torch.cuda.synchronize()
    assert len(kv) == T + best[1]
    after = kv.raw()
    # everything except the committed cells equals the pre-run image
    es = 2
    img = after.copy().reshape(2, sh.n_layers, sh.n_kv_heads, T + 64, sh.head_dim * es)
    ref = snapshot.reshape(img.shape)
    assert np.array_equal(np.delete(img, np.s_[T:T + best[1]], axis=3), np.delete(ref, np.s_[T:T + best[1]], axis=3))
    assert best[1] == 0 or img[:, :, :, T:T + best[1]].any()


def test_llama7b_four_runs_per_weight_pass_match_oracle(llama7b):
    """The same eight tree runs, four per weight pass (pi_stage_forward_multi, 16 tokens): runs the
    schedule cancels stop before their layer (their words are stored in-stream between two stage
    calls per distinct stop layer), the others' sampled logits equal the oracle's values for that
    run evaluated alone, and every run reports its own status."""
    sh, m = llama7b
    g = _load("llama7b_runs")
    T, n = g["prefix"], 4
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
    cols = np.asarray(g["cols"])
    snapshot = kv.raw().copy()
    for q in range(2):
        recs = g["runs"][4 * q:4 * q + 4]
        stops = [g["cancel_before_layer"][4 * q + j] for j in range(4)]
        parent = np.concatenate([np.where(np.asarray(r["parent"]) >= 0, np.asarray(r["parent"]) + n * j, -1)
                                 for j, r in enumerate(recs)]).astype(np.int32)
        toks = np.concatenate([np.asarray(r["tokens"]) for r in recs]).astype(np.int32)
        rd = synth.tree_run(parent, T, T, offset=4 * n * q)
        run = gpu_loader.make_run(rd, toks)
        groups = [j for j in range(4) for _ in range(n)]
        logits = torch.zeros((4 * n, sh.vocab), device="cuda")
        hid = [torch.zeros((4 * n, sh.d_model), device="cuda") for _ in range(2)]
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        gstat = torch.full((4, 2), -9, dtype=torch.int32, device="cuda")
        flags = torch.zeros(4, dtype=torch.int32, device="cuda")
        cuts = sorted({s for s in stops if s > 0})          # stage boundaries at which words are raised
        for j, s in enumerate(stops):
            if s == 0:
                flags[j] = 1
        begin, hin = 0, None
        for k, cut in enumerate(cuts + [sh.n_layers]):
            last = cut == sh.n_layers
            pi.stage_forward_multi(m, kv, run, groups, begin, cut, hidden_in=hin,
                                   hidden_out=None if last else hid[k % 2], logits_out=logits if last else None,
                                   cancel_flags=flags, group_status=gstat, run_status=status)
            for j, s in enumerate(stops):
                if s == cut:
                    flags[j] = 1                             # in-stream store between two stage calls
            begin, hin = cut, hid[k % 2]
        torch.cuda.synchronize()
        if all(s >= 0 for s in stops):                       # every run of the pass cancelled: the pass itself stops
            assert status.cpu().tolist() == [pi.PI_CANCELLED, max(stops)]
        else:
            assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
        want = [[pi.PI_CANCELLED, s] if s >= 0 else [pi.PI_OK, sh.n_layers] for s in stops]
        assert gstat.cpu().tolist() == want
        lg = logits.cpu().numpy()
        for j, rec in enumerate(recs):
            if stops[j] < 0:
                _check_rows(lg[n * j:n * j + n], rec["rows"], cols)
        pi.kv_rollback(kv, run.slots, 4 * n)
        torch.cuda.synchronize()
        assert np.array_equal(kv.raw(), snapshot)


def test_llama7b_runs_described_by_cell_metadata(llama7b):
    """The same eight tree runs, described on the device: every run takes one partition per
    branch, its cells and window words come from the metadata kernels (they must equal the
    workload's own descriptors bit for bit), the forward reads them where they lie, the best
    run is accepted from the device's verification result, all partitions are given back, and
    compaction leaves a dense canonical prefix that holds the accepted path's entries."""
    from test_gpu_kvmeta import Pair, dev_i32, dev_sets
    sh, m = llama7b
    g = _load("llama7b_runs")
    T, n = g["prefix"], 4
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
    cols = np.asarray(g["cols"])
    p = Pair(T + 64, 32)
    p.fill(0, T, 0, range(32))
    survivors = []
    all_ids = []
    for r, rec in enumerate(g["runs"]):
        parent = np.asarray(rec["parent"], dtype=np.int32)
        toks = np.asarray(rec["tokens"], dtype=np.int32)
        rd = synth.tree_run(parent, T, T, offset=n * r)
        ids = [p.acquire() for _ in range(synth.n_leaves(parent))]
        assert None not in ids
        all_ids += ids
        seqs = synth.tree_sequences(parent, ids)
        positions = rd["positions"].tolist()
        st, slots = p.place(positions, seqs, T)
        mask, bad = p.build_mask(positions, seqs, T, T)
        assert st == 0 and bad == 0
        assert np.array_equal(slots.cpu().numpy(), rd["slots"])
        assert np.array_equal(mask.cpu().numpy().view(np.uint64), rd["mask"])
        if g["cancel_before_layer"][r] >= 0:
            continue                                       # a cancelled run: its cells stay unwritten
        run = gpu_loader.make_run(rd, toks)
        run.slots, run.mask = slots, mask
        logits = torch.zeros((n, sh.vocab), device="cuda")
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
        acc = torch.zeros(n, dtype=torch.int32, device="cuda")
        res = torch.zeros(2, dtype=torch.int32, device="cuda")
        pi.verify_greedy(run.tokens, run.parent, n, logits, sh.vocab, g["root_expected"], acc, res)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
        _check_rows(logits.cpu().numpy(), rec["rows"], cols)
        survivors.append((r, int(res[0].item()), acc, res, positions, seqs, slots.cpu().numpy()))
    p.check("eight runs placed")
    best = max(survivors, key=lambda x: (x[1], -x[0]))
    r, a, acc, res, positions, seqs, slots = best
    p.g.accept(n, dev_i32(positions), dev_sets(seqs), acc, res)          # device results straight in
    path = acc.cpu().tolist()[:a]
    p.o.accept(positions, seqs, path)
    for s in all_ids:
        p.release(s)
    p.check("accepted and released")
    before = kv.raw().copy().reshape(2, sh.n_layers, sh.n_kv_heads, T + 64, sh.head_dim * 2)
    st, dense = p.compact(T, kv)
    assert (st, dense) == (0, T + a) and len(kv) == T + a
    p.check("compaction")
    after = kv.raw().reshape(before.shape)
    src = [int(slots[i]) for i in path]                                   # path order == position order
    want = before.copy()
    want[:, :, :, T:T + a] = before[:, :, :, src]
    assert np.array_equal(after, want)
    assert a == 0 or after[:, :, :, T:T + a].any()
    pos, seq = p.g.read()
    assert pos[:T + a].tolist() == list(range(T + a)) and not (pos[T + a:] >= 0).any()


def test_llama7b_continuous_speculation_equals_plain_decoding(llama7b):
    """At full size there is no oracle sequence to compare with, but the method's own claim
    (Section "Model Accuracy") holds at any size: whatever the draft quality and however the
    runs are queued, cancelled and packed into passes, the tokens are those of decoding one
    token per forward.  Compared up to the first step whose top-2 logit gap is too small for
    the batch size not to matter."""
    from paper_2407_11798_amd.pipeline import ContinuousSpeculation
    sh, m = llama7b
    T, n_gen = 512, 24
    kv = pi.KVCache(m, T + 64 + 64)
    first = int(synth.tokens_host(sh, 0, 1, synth.T_MISC, salt=77)[0])
    gpu_loader.prefill_kv_synthetic(kv, sh, 0, T)
    lg = torch.empty((1, sh.vocab), device="cuda")
    acc = torch.zeros(1, dtype=torch.int32, device="cuda")
    res = torch.zeros(2, dtype=torch.int32, device="cuda")
    G, safe, t = [], n_gen, first
    for i in range(n_gen):
        run = gpu_loader.make_run(synth.linear_run(1, T + i), np.array([t], dtype=np.int32))
        pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=lg)
        pi.verify_greedy(run.tokens, None, 1, lg, sh.vocab, t, acc, res)
        pi.kv_rollback(kv, run.slots, 1, acc, res)
        torch.cuda.synchronize()
        top = torch.topk(lg[0], 2).values
        if float(top[0] - top[1]) < 1e-3 * float(lg[0].abs().max()) and safe == n_gen:
            safe = i
        t = int(res[1].item())
        G.append(t)
    assert safe >= 12
    for alpha, depth, rpp in ((0.7, 3, 1), (0.7, 2, 4)):
        gpu_loader.prefill_kv_synthetic(kv, sh, 0, T)
        u = synth.uniform_int_host(2 * (n_gen + 64), 5, synth.stream_id(synth.T_MISC, 10 * rpp), 1 << 20)

        def draft(pos, u=u):
            i = pos - (T + 1)
            g = G[i] if i < len(G) else 0
            return (g if u[2 * i] < alpha * (1 << 20) else (g + 3) % sh.vocab), float(u[2 * i + 1]) / (1 << 20)

        cs = ContinuousSpeculation(m, kv, T, first, draft, depth=depth, micro_batch=4, base_cutoff=0.0, recovery=0.05,
                                   decay=0.05, runs_per_pass=rpp)
        out = cs.generate(n_gen)
        st = dict(cs.stats)
        cs.close()
        assert out[:safe] == G[:safe], (alpha, depth, rpp)
        assert st["tokens_accepted_from_drafts"] > 0 and st["discarded"] > 0
        if rpp == 1:
            assert st["cancelled"] > 0 and st["layers_skipped"] > 0      # at this size the signal arrives in time
    kv.free()


def test_tinyllama_decode_steps_match_oracle():
    """TinyLlama-shaped draft model (grouped-query attention, 4 KV heads x 64): single-token decode
    steps at short and long prefixes, the generator side's workload."""
    sh = synth.SHAPES["tinyllama"]
    g = _load("tinyllama_decode")
    m = gpu_loader.load_model(sh, g["seed"])
    cols = np.asarray(g["cols"])
    try:
        for T_str, rec in g["runs"].items():
            T = int(T_str)
            kv = pi.KVCache(m, T + 64)
            gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
            toks = np.asarray(rec["tokens"], dtype=np.int32)
            assert np.array_equal(toks, synth.tokens_host(sh, g["seed"], 1, synth.T_DRAFT, salt=T))
            run = gpu_loader.make_run(synth.linear_run(1, T), toks)
            logits = torch.zeros((1, sh.vocab), device="cuda")
            status = torch.zeros(2, dtype=torch.int32, device="cuda")
            pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
            worst = _check_rows(logits.cpu().numpy(), rec["rows"], cols)
            print("T=%d worst sampled logit error / row max: %.2e" % (T, worst))
            kv.free()
    finally:
        m.free()


@pytest.mark.parametrize("shape_name", ["llama70b", "llama70b_w8", "llama70b_w4", "llama70b_w4b"])
def test_llama70b_shaped_layer_matches_oracle(shape_name):
    """One decoder layer plus the LM head of the Llama-70B shape (d 8192, 64 query / 8 KV heads,
    FFN 28672) over 2048 prefix cells, batches of 1 and 16 tokens: the widest matrices, the most
    column slices and the largest grouped-query fan-out the kernels meet; with bf16, 8-bit and
    4-bit weight matrices."""
    import dataclasses
    g = _load(shape_name + "_layer")
    sh = dataclasses.replace(synth.SHAPES[shape_name], n_layers=g["n_layers"], name=shape_name + "_l1")
    m = gpu_loader.load_model(sh, g["seed"])
    T = g["prefix"]
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
    cols = np.asarray(g["cols"])
    try:
        for n_str, rec in g["runs"].items():
            n = int(n_str)
            toks = np.asarray(rec["tokens"], dtype=np.int32)
            assert np.array_equal(toks, synth.tokens_host(sh, g["seed"], n, synth.T_DRAFT, salt=n))
            run = gpu_loader.make_run(synth.linear_run(n, T), toks)
            logits = torch.zeros((n, sh.vocab), device="cuda")
            status = torch.zeros(2, dtype=torch.int32, device="cuda")
            pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
            worst = _check_rows(logits.cpu().numpy(), rec["rows"], cols)
            print("n=%d worst sampled logit error / row max: %.2e" % (n, worst))
            pi.kv_rollback(kv, run.slots, n)
    finally:
        kv.free()
        m.free()


def test_llama70b_full_depth_matches_oracle():
    """The whole 80-layer Llama-70B-shaped stack (138 GB of bf16 weights), 2048 prefix cells,
    batches of 1 and 16 tokens: every logits column against stored oracle rows; the first 20
    layers as a pipeline stage of their own (hidden state after layer 20 against the oracle's,
    then layers 20..80 from it, bit-equal to the unsplit stack); the run's own K/V cells in
    layers 0, 19 and 79."""
    sh = synth.SHAPES["llama70b"]
    g, arr = _load_full("llama70b_full")
    free, _ = torch.cuda.mem_get_info()
    assert free > 150e9, "the 70B-shaped model needs 140 GB of device memory, %.0f GB free" % (free / 1e9)
    m = gpu_loader.load_model(sh, g["seed"])
    T = g["prefix"]
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, g["seed"], T)
    try:
        for n_str, rec in g["runs"].items():
            n = int(n_str)
            toks = np.asarray(rec["tokens"], dtype=np.int32)
            assert np.array_equal(toks, synth.tokens_host(sh, g["seed"], n, synth.T_DRAFT, salt=n))
            run = gpu_loader.make_run(synth.linear_run(n, T), toks)
            whole = torch.zeros((n, sh.vocab), device="cuda")
            status = torch.zeros(2, dtype=torch.int32, device="cuda")
            pi.stage_forward(m, kv, run, 0, sh.n_layers, logits_out=whole, run_status=status)
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
            worst = _check_full_rows(whole.cpu().numpy(), arr["logits_n%d" % n], rec["rows"])
            print("70B n=%d worst logit error / row max over all columns: %.2e" % (n, worst), flush=True)
            for l in (0, 19, 79):
                k, v = kv.get_cells(l, T, n)
                assert _cells_close(k, arr["k_n%d_layer%d" % (n, l)]) and _cells_close(v, arr["v_n%d_layer%d" % (n, l)]), l
            pi.kv_rollback(kv, run.slots, n)
            # one pipeline stage's share: layers [0, 20), then the rest from its output
            hidden = torch.zeros((n, sh.d_model), device="cuda")
            split = torch.zeros((n, sh.vocab), device="cuda")
            pi.stage_forward(m, kv, run, 0, 20, hidden_out=hidden, run_status=status)
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [pi.PI_OK, 20]
            href = arr["hidden_n%d_after20" % n].astype(np.float64)
            herr = np.max(np.abs(hidden.cpu().numpy() - href), axis=-1) / np.max(np.abs(href), axis=-1)
            assert herr.max() <= 2e-2, "hidden state after 20 layers: %g of the row's max" % herr.max()
            pi.stage_forward(m, kv, run, 20, sh.n_layers, hidden_in=hidden, logits_out=split, run_status=status)
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [pi.PI_OK, sh.n_layers]
            assert torch.equal(whole, split)
            pi.kv_rollback(kv, run.slots, n)
        torch.cuda.synchronize()
        assert len(kv) == T
        # Early Inference Cancellation on a 20-layer stage of this shape: the signal is raised from
        # another compute unit in the middle of a layer and the stage stops at that layer's end
        _cancel_raised_on_the_device(m, kv, sh, T, 8, 20, (0, 7, 18))
    finally:
        kv.free()
        m.free()


def _cancel_raised_on_the_device(m, kv, sh, T, n, layer_end, layers):
    """A workgroup in the middle of the grid stores the run's cancel word when it enters the gate/up
    phase of `layer` (pi_debug_raise_cancel): the run must stop at the boundary that ends this very
    layer -- no further layer starts after the signal -- and the stop must come within one layer's
    time of the store on the device's own clock."""
    cap = 5 * sh.n_layers + 8
    toks = synth.tokens_host(sh, 0, n, synth.T_DRAFT, salt=n)
    run = gpu_loader.make_run(synth.linear_run(n, T), toks)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    last = layer_end == sh.n_layers
    logits = torch.full((n, sh.vocab), 7.0, device="cuda") if last else None
    hidden = torch.full((n, sh.d_model), 7.0, device="cuda") if not last else None
    snapshot_len = len(kv)
    m.set_plan(5, 1)
    try:
        for layer in layers:
            flag.zero_()
            m.raise_cancel(layer, 3)
            pi.stage_forward(m, kv, run, 0, layer_end, hidden_out=hidden, logits_out=logits, cancel_flag=flag,
                             run_status=status)
            pi.kv_rollback(kv, run.slots, n)
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [pi.PI_CANCELLED, layer + 1], (layer, status.cpu().tolist())
            out = logits if last else hidden
            assert float(out.min()) == 7.0 and float(out.max()) == 7.0          # outputs untouched
            tr = m.read_trace(cap).astype(np.int64)
            t_store, t_stop = int(tr[cap - 1]), int(tr[3 + 2 * layer])
            t_prev = int(tr[3 + 2 * (layer - 1)]) if layer > 0 else int(tr[1])
            assert t_prev < t_store < t_stop                                     # raised inside the layer it stopped
            assert t_stop - t_store <= t_stop - t_prev                           # within one layer's time
            print("cancel raised in layer %d: stop %.1f us after the signal (the layer took %.1f us)"
                  % (layer, (t_stop - t_store) / 100.0, (t_stop - t_prev) / 100.0), flush=True)
    finally:
        m.raise_cancel(-1, 3)
        m.set_plan(5, 0)
    assert len(kv) == snapshot_len


def test_llama7b_cancel_raised_on_the_device_stops_at_the_end_of_the_layer(llama7b):
    sh, m = llama7b
    T = 512
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, 0, T)
    snapshot = kv.raw().copy()
    _cancel_raised_on_the_device(m, kv, sh, T, 8, sh.n_layers, (0, 1, 13, 30))
    assert np.array_equal(kv.raw(), snapshot)                                    # as if the runs had never started
    kv.free()


def test_llama70b_shaped_stage_slice_properties():
    """A 4-layer model of the 70B shape run as two 2-layer pipeline stages must equal the single
    4-layer stage bit for bit, and a 4-token batch must agree with four sequential single-token
    runs within the bf16 tolerance (no oracle at this size: properties that hold at any size)."""
    import dataclasses
    sh = dataclasses.replace(synth.SHAPES["llama70b"], n_layers=4, name="llama70b_l4")
    m = gpu_loader.load_model(sh, 0)
    T, n = 2048, 4
    kv = pi.KVCache(m, T + 64)
    gpu_loader.prefill_kv_synthetic(kv, sh, 0, T)
    toks = synth.tokens_host(sh, 0, n, synth.T_DRAFT, salt=n)
    try:
        run = gpu_loader.make_run(synth.linear_run(n, T), toks)
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        whole = torch.zeros((n, sh.vocab), device="cuda")
        pi.stage_forward(m, kv, run, 0, 4, logits_out=whole, run_status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_OK, 4]
        pi.kv_rollback(kv, run.slots, n)
        hidden = torch.zeros((n, sh.d_model), device="cuda")
        split = torch.zeros((n, sh.vocab), device="cuda")
        pi.stage_forward(m, kv, run, 0, 2, hidden_out=hidden, run_status=status)
        pi.stage_forward(m, kv, run, 2, 4, hidden_in=hidden, logits_out=split, run_status=status)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_OK, 4]
        assert torch.equal(whole, split)
        pi.kv_rollback(kv, run.slots, n)
        # sequential single-token steps, each committed before the next
        seq = []
        for i in range(n):
            r1 = gpu_loader.make_run(synth.linear_run(1, T + i), toks[i:i + 1])
            lg = torch.zeros((1, sh.vocab), device="cuda")
            pi.stage_forward(m, kv, r1, 0, 4, logits_out=lg, run_status=status)
            acc = torch.zeros(1, dtype=torch.int32, device="cuda")
            res = torch.tensor([1, 0], dtype=torch.int32, device="cuda")
            pi.kv_rollback(kv, r1.slots, 1, acc, res)
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [pi.PI_OK, 4]
            seq.append(lg.cpu().numpy()[0])
        seq = np.stack(seq)
        w = whole.cpu().numpy()
        err = np.max(np.abs(w - seq), axis=1) / np.max(np.abs(seq), axis=1)
        assert err.max() <= 2e-2, "batch vs sequential: %s" % err
        assert len(kv) == T + n
    finally:
        kv.free()
        m.free()
