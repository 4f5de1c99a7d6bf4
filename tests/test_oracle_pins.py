"""Pins that tie the CPU oracle to things other than itself: closed forms, invariants the
paper states, special cases that reduce to library routines, and planted answers."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
import oracle
from oracle import from_synth

RNG = np.random.default_rng(1234)


# ---- RMSNorm -------------------------------------------------------------------------------

def test_rmsnorm_unit_rms_closed_form_and_scale_invariance():
    x = RNG.normal(size=(5, 256)) * 3.7
    eps = 1e-5
    y = oracle.rmsnorm(x, np.ones(256), eps)
    ms = np.mean(x * x, axis=-1)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0 / np.sqrt(1.0 + eps / ms), rtol=1e-13)
    y2 = oracle.rmsnorm(1e4 * x, np.ones(256), 0.0)
    assert np.allclose(y2, oracle.rmsnorm(x, np.ones(256), 0.0), rtol=1e-12)
    # the gain is applied elementwise after normalisation
    g = RNG.normal(size=256)
    assert np.allclose(oracle.rmsnorm(x, g, eps), y * g, rtol=1e-13)


def test_rmsnorm_matches_library_routine():
    x = RNG.normal(size=(3, 64))
    g = RNG.normal(size=64)
    ref = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(oracle.rmsnorm(x, g, 1e-5), ref, rtol=1e-12, atol=1e-14)


# ---- RoPE ----------------------------------------------------------------------------------

def test_rope_known_angles_and_pairing():
    # hd = 4, base 10000: pair 0 rotates by pos * 1, pair 1 by pos * 10000^(-1/2) = pos * 0.01
    x = np.zeros((1, 1, 4))
    x[0, 0] = [1.0, 0.0, 0.0, 2.0]
    y = oracle.rope(x, np.array([3]), 10000.0)
    assert np.allclose(y[0, 0], [np.cos(3.0), np.sin(3.0), -2 * np.sin(0.03), 2 * np.cos(0.03)], atol=1e-15)


def test_rope_norm_preserved_relative_and_identity():
    q = RNG.normal(size=(4, 3, 64))
    k = RNG.normal(size=(4, 3, 64))
    pos = np.array([0, 5, 17, 600])
    rq = oracle.rope(q, pos, 10000.0)
    assert np.allclose(rq[0], q[0], atol=0)                       # position 0 is the identity
    assert np.allclose(np.linalg.norm(rq, axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    pn = rq.reshape(4, 3, 32, 2)
    assert np.allclose(np.linalg.norm(pn, axis=-1), np.linalg.norm(q.reshape(4, 3, 32, 2), axis=-1), rtol=1e-12)
    # scores depend on the position difference only
    a = np.einsum("nhd,nhd->nh", oracle.rope(q, pos, 1e4), oracle.rope(k, pos + 3, 1e4))
    b = np.einsum("nhd,nhd->nh", oracle.rope(q, pos + 100, 1e4), oracle.rope(k, pos + 103, 1e4))
    assert np.allclose(a, b, rtol=1e-9, atol=1e-10)


# ---- linear / SwiGLU -----------------------------------------------------------------------

def test_linear_orientation_and_identities():
    x = RNG.normal(size=(3, 8))
    assert np.allclose(oracle.linear(x, np.eye(8)), x)
    w = np.zeros((5, 8))
    w[2, 6] = 1.0                               # output 2 reads input 6 (W is [out, in])
    y = oracle.linear(x, w)
    assert np.allclose(y[:, 2], x[:, 6]) and np.count_nonzero(y) == 3
    wr = RNG.normal(size=(5, 8))
    assert np.allclose(oracle.linear(x, wr), F.linear(torch.from_numpy(x), torch.from_numpy(wr)).numpy())


def test_silu_known_values():
    assert oracle.silu(np.array([0.0]))[0] == 0.0
    assert abs(oracle.silu(np.array([1.0]))[0] - 1.0 / (1.0 + np.exp(-1.0))) < 1e-16
    assert abs(oracle.silu(np.array([40.0]))[0] - 40.0) < 1e-12
    assert abs(oracle.silu(np.array([-40.0]))[0]) < 1e-12
    z = RNG.normal(size=100)
    assert np.allclose(oracle.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-13)


# ---- attention -----------------------------------------------------------------------------

def test_attention_special_cases():
    hd, cells = 8, 12
    K = RNG.normal(size=(cells, 2, hd))
    V = RNG.normal(size=(cells, 2, hd))
    q = RNG.normal(size=(2, 4, hd))             # 4 query heads over 2 kv heads (groups of 2)
    # single visible cell: output is that cell's V, from kv head h // 2
    o = oracle.attention(q, K, V, prefix_len=0, window_base=5, mask=np.array([1, 2], dtype=np.uint64))
    for h in range(4):
        assert np.allclose(o[0, h], V[5, h // 2]) and np.allclose(o[1, h], V[6, h // 2])
    # all keys zero: uniform weights -> mean of the visible V rows
    o = oracle.attention(q, np.zeros_like(K), V, prefix_len=4, window_base=8, mask=np.array([1, 3], dtype=np.uint64))
    assert np.allclose(o[0, 3], V[[0, 1, 2, 3, 8], 1].mean(axis=0))
    assert np.allclose(o[1, 0], V[[0, 1, 2, 3, 8, 9], 0].mean(axis=0))
    # two cells: closed-form softmax weights with the 1/sqrt(hd) scale
    s = (K[[0, 1], 0] @ q[0, 0]) / np.sqrt(hd)
    w1 = 1.0 / (1.0 + np.exp(s[0] - s[1]))
    o = oracle.attention(q[:1], K, V, prefix_len=2, window_base=2, mask=np.array([0], dtype=np.uint64))
    assert np.allclose(o[0, 0], (1 - w1) * V[0, 0] + w1 * V[1, 0], rtol=1e-12)
    # a masked cell has no influence at all
    K2, V2 = K.copy(), V.copy()
    K2[9] += 100.0
    V2[9] -= 50.0
    m = np.array([0b0101, 0b0001], dtype=np.uint64)   # window cells 8 and 10 / 8 only
    assert np.array_equal(oracle.attention(q, K, V, 3, 8, m), oracle.attention(q, K2, V2, 3, 8, m))


def test_attention_matches_library_routine():
    n, hq, hkv, hd, cells = 5, 6, 2, 16, 40
    K = RNG.normal(size=(cells, hkv, hd))
    V = RNG.normal(size=(cells, hkv, hd))
    q = RNG.normal(size=(n, hq, hd))
    prefix, base = 23, 30
    mask = np.array([0b00001, 0b00011, 0b00101, 0b01101, 0b10001], dtype=np.uint64)
    o = oracle.attention(q, K, V, prefix, base, mask)
    allow = np.zeros((n, cells), dtype=bool)
    for i in range(n):
        allow[i, oracle.visible_cells(prefix, base, mask[i])] = True
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]                    # [1,Hq,n,hd]
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)[None]
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(allow)[None, None])
    assert np.allclose(o, ref[0].permute(1, 0, 2).numpy(), rtol=1e-11, atol=1e-13)


# ---- whole-run invariants ------------------------------------------------------------------

def _tiny(seed=0, gain_sigma=0.1, shape="tiny"):
    sh = synth.SHAPES[shape]
    return sh, from_synth.model_from_seed(sh, seed, gain_sigma)


def _prefill(sh, model, seed, n_prefill, n_cells):
    """True prefill: run n_prefill seeded tokens as one causal batch and commit them all."""
    kv = oracle.OracleKV(sh, n_cells)
    toks = synth.tokens_host(sh, seed, n_prefill)
    run = synth.linear_run(n_prefill, 0) if n_prefill <= 64 else None
    if run is None:
        raise ValueError
    out = oracle.stage_forward(model, kv, run, 0, sh.n_layers, tokens=toks)
    oracle.kv_rollback(kv, run["slots"], list(range(n_prefill)))
    return kv, toks, out["logits"]


def test_batch_equals_sequential_steps():
    """The paper's correctness claim: verifying n tokens in one masked batch gives what n
    single-token steps would (Section "Model Accuracy")."""
    sh, model = _tiny()
    kv, _, _ = _prefill(sh, model, 0, 16, 64)
    draft = synth.tokens_host(sh, 1, 5, synth.T_DRAFT)
    kb = kv.clone()
    run = synth.linear_run(5, 16)
    batch = oracle.stage_forward(model, kb, run, 0, sh.n_layers, tokens=draft)["logits"]
    ks = kv.clone()
    for i in range(5):
        r1 = synth.linear_run(1, 16 + i)
        li = oracle.stage_forward(model, ks, r1, 0, sh.n_layers, tokens=draft[i:i + 1])["logits"]
        oracle.kv_rollback(ks, r1["slots"], [0])
        assert np.max(np.abs(li[0] - batch[i])) < 1e-12
    oracle.kv_rollback(kb, run["slots"], list(range(5)))
    assert kb.kv_len == ks.kv_len == 21
    assert np.array_equal(kb.K, ks.K) and np.array_equal(kb.V, ks.V)


def test_stage_split_equals_whole():
    sh, model = _tiny(shape="tiny_gqa")
    kv, _, _ = _prefill(sh, model, 0, 8, 32)
    draft = synth.tokens_host(sh, 2, 3, synth.T_DRAFT)
    run = synth.linear_run(3, 8)
    whole = oracle.stage_forward(model, kv.clone(), run, 0, sh.n_layers, tokens=draft)["logits"]
    k2 = kv.clone()
    a = oracle.stage_forward(model, k2, run, 0, 1, tokens=draft)
    assert a["logits"] is None and a["layers_done"] == 1
    b = oracle.stage_forward(model, k2, run, 1, sh.n_layers, hidden_in=a["hidden"])
    assert np.array_equal(whole, b["logits"])


def test_tree_isolation_and_chain_equivalence():
    sh, model = _tiny()
    kv, _, _ = _prefill(sh, model, 0, 12, 64)
    parent = np.array([-1, 0, 0, 1, -1], dtype=np.int32)       # two roots, a fork under node 0
    toks = np.array([5, 6, 7, 8, 9], dtype=np.int32)
    run = synth.tree_run(parent, 12, 12)
    base = oracle.stage_forward(model, kv.clone(), run, 0, sh.n_layers, tokens=toks)["logits"]
    t2 = toks.copy()
    t2[2] = 500                                                 # sibling of node 1, not an ancestor of 1 or 3
    t2[4] = 321
    pert = oracle.stage_forward(model, kv.clone(), run, 0, sh.n_layers, tokens=t2)["logits"]
    for i in (0, 1, 3):
        assert np.array_equal(base[i], pert[i])
    assert not np.array_equal(base[2], pert[2])
    # the branch 0 -> 1 -> 3 equals a linear run of those three tokens
    lin = oracle.stage_forward(model, kv.clone(), synth.linear_run(3, 12), 0, sh.n_layers, tokens=toks[[0, 1, 3]])["logits"]
    assert np.max(np.abs(lin - base[[0, 1, 3]])) < 1e-12


def test_slot_in_live_cell_is_rejected():
    sh, model = _tiny()
    kv, _, _ = _prefill(sh, model, 0, 4, 16)
    run = synth.linear_run(2, 4, window_base=3)
    with pytest.raises(ValueError):
        oracle.stage_forward(model, kv, run, 0, sh.n_layers, tokens=np.array([1, 2]))


# ---- verification --------------------------------------------------------------------------

def _onehot_logits(n, vocab, winners):
    lg = RNG.normal(size=(n, vocab))
    for i, w in enumerate(winners):
        lg[i, w] = 50.0
    return lg


def test_verify_planted_prefix_lengths():
    n, vocab = 4, 64
    target_next = [11, 22, 33, 44]                  # target's choice after node i
    root_expected = 7
    for k in range(n + 1):
        draft = np.array([root_expected] + target_next[:n - 1], dtype=np.int32)  # fully agreeing chain
        if k < n:
            draft[k] = (draft[k] + 1) % vocab       # first disagreement at node k
        a, acc, bonus = oracle.verify_greedy(draft, None, _onehot_logits(n, vocab, target_next), root_expected)
        assert a == k and acc == list(range(k))
        assert bonus == (root_expected if k == 0 else target_next[k - 1])


def test_verify_tree_walk_and_ties():
    vocab = 32
    parent = np.array([-1, -1, 0, 0, 2, 1], dtype=np.int32)
    draft = np.array([3, 4, 9, 8, 5, 6], dtype=np.int32)
    lg = _onehot_logits(6, vocab, [8, 6, 5, 1, 2, 0])
    # root expects 3 -> node 0; node 0 says 8 -> node 3 (not node 2); node 3 says 1 -> no child
    a, acc, bonus = oracle.verify_greedy(draft, parent, lg, 3)
    assert (a, acc, bonus) == (2, [0, 3], 1)
    # root expects 4 -> node 1 -> says 6 -> node 5 -> leaf: bonus is the leaf's argmax
    a, acc, bonus = oracle.verify_greedy(draft, parent, lg, 4)
    assert (a, acc, bonus) == (2, [1, 5], 0)
    # ties: lowest token id wins; duplicate siblings: lowest node index wins
    lg2 = np.zeros((2, vocab))
    lg2[0, [4, 9]] = 1.0
    a, acc, bonus = oracle.verify_greedy(np.array([2, 2]), np.array([-1, -1]), lg2, 2)
    assert (a, acc, bonus) == (1, [0], 4)


def test_chained_verification_counts_only_behind_a_fully_accepted_run():
    vocab = 32
    lg = _onehot_logits(3, vocab, [8, 6, 5])            # the target's choice after node i
    draft = np.array([3, 8, 6], dtype=np.int32)         # right if the root is expected to be 3
    # the earlier run accepted all 4 of its tokens and predicts 3 next: this run counts in full
    assert oracle.verify_greedy_chained(draft, None, lg, 99, prev_result=(4, 3), prev_n=4) == (3, [0, 1, 2], 5)
    # ... predicts 7 next: the root is wrong, the target's own token stands
    assert oracle.verify_greedy_chained(draft, None, lg, 99, prev_result=(4, 7), prev_n=4) == (0, [], 7)
    # the earlier run was cut short at 2 of 4: whatever this run says, it built on a wrong token
    assert oracle.verify_greedy_chained(draft, None, lg, 3, prev_result=(2, 3), prev_n=4) == (0, [], -1)
    # a cancelled forward has no logits to speak of
    assert oracle.verify_greedy_chained(draft, None, lg, 3, run_ok=False) == (0, [], -1)
    # no earlier run: the plain rule
    assert oracle.verify_greedy_chained(draft, None, lg, 3) == oracle.verify_greedy(draft, None, lg, 3) == (3, [0, 1, 2], 5)
    # splitting a chain into two runs gives the same tokens as verifying it whole
    whole = oracle.verify_greedy(np.array([3, 8, 6, 5, 1]), None, _onehot_logits(5, vocab, [8, 6, 5, 1, 2]), 3)
    first = oracle.verify_greedy(np.array([3, 8, 6]), None, _onehot_logits(3, vocab, [8, 6, 5]), 3)
    second = oracle.verify_greedy_chained(np.array([5, 1]), None, _onehot_logits(2, vocab, [1, 2]), 0,
                                          prev_result=(first[0], first[2]), prev_n=3)
    assert whole == (5, [0, 1, 2, 3, 4], 2) and first[0] + second[0] == 5 and second[2] == whole[2]


def test_planted_draft_end_to_end_and_rollback_equals_sequential_decode():
    """Tiny configuration: 64 prefilled positions, 4 draft tokens planted to agree with the
    target for the first 2.  Accepted = 2, bonus = target's choice after node 1, and the
    committed cells equal those of decoding the 2 accepted tokens one by one."""
    sh, model = _tiny(gain_sigma=0.0)
    kv, _, pre_logits = _prefill(sh, model, 0, 64, 128)
    root_expected = int(np.argmax(pre_logits[63]))
    d = np.zeros(4, dtype=np.int32)
    d[0] = root_expected
    l0 = oracle.stage_forward(model, kv.clone(), synth.linear_run(1, 64), 0, sh.n_layers, tokens=d[:1])["logits"]
    d[1] = int(np.argmax(l0[0]))
    l1 = oracle.stage_forward(model, kv.clone(), synth.linear_run(2, 64), 0, sh.n_layers, tokens=d[:2])["logits"]
    d[2] = (int(np.argmax(l1[1])) + 1) % sh.vocab
    d[3] = int(synth.tokens_host(sh, 0, 1, synth.T_DRAFT)[0])
    run = synth.linear_run(4, 64)
    kb = kv.clone()
    lg = oracle.stage_forward(model, kb, run, 0, sh.n_layers, tokens=d)["logits"]
    a, acc, bonus = oracle.verify_greedy(d, run["parent"], lg.astype(np.float32), root_expected)
    assert (a, acc) == (2, [0, 1]) and bonus == int(np.argmax(l1[1]))
    oracle.kv_rollback(kb, run["slots"], acc)
    assert kb.kv_len == 66
    ks = kv.clone()
    for i in range(2):
        r1 = synth.linear_run(1, 64 + i)
        oracle.stage_forward(model, ks, r1, 0, sh.n_layers, tokens=d[i:i + 1])
        oracle.kv_rollback(ks, r1["slots"], [0])
    assert np.array_equal(kb.K, ks.K) and np.array_equal(kb.V, ks.V)
    assert not kb.K[:, 66:].any() and not kb.V[:, 66:].any()     # rejected cells are free again


def test_rollback_moves_tree_path_to_canonical_cells():
    sh, model = _tiny(shape="tiny_gqa")
    kv, _, _ = _prefill(sh, model, 0, 8, 40)
    parent = np.array([-1, -1, 1, 1, 3], dtype=np.int32)
    toks = np.array([1, 2, 3, 4, 5], dtype=np.int32)
    run = synth.tree_run(parent, 8, 8)
    kb = kv.clone()
    oracle.stage_forward(model, kb, run, 0, sh.n_layers, tokens=toks)
    path = [1, 3, 4]
    expectK = kb.K[:, [9, 11, 12]].copy()
    oracle.kv_rollback(kb, run["slots"], path)
    assert kb.kv_len == 11 and np.array_equal(kb.K[:, 8:11], expectK) and not kb.K[:, 11:].any()
    # and they equal the cells of a linear decode of the path's tokens
    ks = kv.clone()
    lin = synth.linear_run(3, 8)
    oracle.stage_forward(model, ks, lin, 0, sh.n_layers, tokens=toks[path])
    assert np.max(np.abs(ks.K[:, 8:11] - kb.K[:, 8:11])) == 0.0


# ---- cancellation --------------------------------------------------------------------------

def test_cancel_leaves_cache_as_if_never_run():
    sh, model = _tiny(shape="tiny_gqa")
    kv, _, _ = _prefill(sh, model, 0, 8, 32)
    run = synth.linear_run(3, 8)
    toks = np.array([7, 8, 9], dtype=np.int32)
    ref = oracle.stage_forward(model, kv.clone(), run, 0, sh.n_layers, tokens=toks)["logits"]
    for stop in range(sh.n_layers):
        kc = kv.clone()
        out = oracle.stage_forward(model, kc, run, 0, sh.n_layers, tokens=toks, cancel_before_layer=stop)
        assert out["status"] == oracle.PI_CANCELLED and out["layers_done"] == stop and out["logits"] is None
        assert (not kc.K[stop:, 8:].any()) and (stop == 0 or kc.K[:stop, 8:11].any())
        oracle.kv_rollback(kc, run["slots"], [])
        assert kc.kv_len == 8 and np.array_equal(kc.K, kv.K) and np.array_equal(kc.V, kv.V)
        again = oracle.stage_forward(model, kc, run, 0, sh.n_layers, tokens=toks)["logits"]
        assert np.array_equal(again, ref)


def test_storage_rounding_of_cache():
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 0.1])
    assert oracle.round_to_storage(x, "bf16").tolist() == [1.0, 1.015625, 0.10009765625]
    assert oracle.round_to_storage(x, "f32")[2] == float(np.float32(0.1))
