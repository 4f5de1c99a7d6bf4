"""Pins for the ORDER in which the oracle's stage_forward composes its operators, and for the
top-2 gap that exempts rows from argmax comparison.

The single operators are pinned in test_oracle_pins.py.  Here the whole layer is rebuilt from
library routines only (torch's rms_norm, linear, scaled_dot_product_attention, silu; the rotary
embedding as a complex multiplication) in the Llama-2 arrangement that Section "Background and
Motivation" refers to, and compared with the oracle; and special weight settings with known
answers check each place where an operator could sit wrongly: SiLU on the gate (not the up)
branch, both residual additions, pre- (not post-) normalisation, rotation of queries and keys but
not of values.  Every test here fails for at least one such mistake planted in the oracle (the
last test plants them)."""
import dataclasses

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
import oracle
from oracle import from_synth

RNG = np.random.default_rng(4321)
NAMES_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "wg", "wu", "wd")
NAMES_GLOBAL = ("embed", "final_norm", "lm_head")


def _random_model(shape_name, seed=0, overrides=None):
    """An oracle model with N(0, 0.05) matrices and gains 1 + N(0, 0.2) in float64; `overrides`
    maps a tensor name to a function of (layer, tensor) -> tensor."""
    sh = dataclasses.replace(synth.SHAPES[shape_name], dtype="f32")
    rng = np.random.default_rng(seed)
    dims = {"embed": (sh.vocab, sh.d_model), "lm_head": (sh.vocab, sh.d_model), "final_norm": (sh.d_model,),
            "attn_norm": (sh.d_model,), "ffn_norm": (sh.d_model,),
            "wq": (sh.n_q_heads * sh.head_dim, sh.d_model), "wk": (sh.n_kv_heads * sh.head_dim, sh.d_model),
            "wv": (sh.n_kv_heads * sh.head_dim, sh.d_model), "wo": (sh.d_model, sh.n_q_heads * sh.head_dim),
            "wg": (sh.ffn, sh.d_model), "wu": (sh.ffn, sh.d_model), "wd": (sh.d_model, sh.ffn)}
    store = {}
    for name in NAMES_GLOBAL:
        store[(name, 0)] = None
    for l in range(sh.n_layers):
        for name in NAMES_LAYER:
            store[(name, l)] = None
    for key in sorted(store):
        name, l = key
        t = 1.0 + 0.2 * rng.normal(size=dims[name]) if name.endswith("norm") else 0.05 * rng.normal(size=dims[name])
        if overrides and name in overrides:
            t = overrides[name](l, t)
        store[key] = t
    return sh, oracle.OracleModel(sh, lambda name, layer=0: store[(name, layer if name in NAMES_LAYER else 0)]), store


def _run_and_cache(sh, n_prefix, parent, seed=0):
    rng = np.random.default_rng(100 + seed)
    kv = oracle.OracleKV(sh, n_prefix + 64, dtype="f32")
    for l in range(sh.n_layers):
        kv.set_cells(l, 0, rng.normal(size=(n_prefix, sh.n_kv_heads, sh.head_dim)).astype(np.float32),
                     rng.normal(size=(n_prefix, sh.n_kv_heads, sh.head_dim)).astype(np.float32))
    kv.kv_len = n_prefix
    run = synth.tree_run(np.asarray(parent, dtype=np.int32), n_prefix, n_prefix)
    toks = rng.integers(0, sh.vocab, size=len(parent))
    return kv, run, toks


def _library_forward(sh, store, kv, run, toks):
    """The same stack from library routines, float64.  K/V of a layer = prefix cells followed by
    the run's own cells (rounded to the float32 cache type like the oracle's); the boolean
    attention mask is the ancestor-or-self relation written out from the run's parent array."""
    t64 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    n = len(toks)
    T = run["prefix_len"]
    hq, hkv, hd = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    pos = t64(run["positions"])
    theta = sh.rope_base ** (-2.0 * torch.arange(hd // 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(n, hd // 2, dtype=torch.float64), pos[:, None] * theta[None, :])  # e^{i pos theta}

    def rotary(x):  # x [n, heads, hd]: adjacent pairs as complex numbers
        xc = torch.view_as_complex(x.reshape(n, -1, hd // 2, 2).contiguous())
        return torch.view_as_real(xc * rot[:, None, :]).reshape(n, -1, hd)

    parent = run["parent"]
    allowed = torch.zeros(n, T + n, dtype=torch.bool)
    allowed[:, :T] = True
    for i in range(n):
        u = i
        while u >= 0:
            allowed[i, T + u] = True
            u = int(parent[u])
    x = t64(store[("embed", 0)])[torch.as_tensor(np.asarray(toks))]
    for l in range(sh.n_layers):
        h = F.rms_norm(x, (sh.d_model,), t64(store[("attn_norm", l)]), eps=sh.rms_eps)
        q = rotary(F.linear(h, t64(store[("wq", l)])).reshape(n, hq, hd))
        k = rotary(F.linear(h, t64(store[("wk", l)])).reshape(n, hkv, hd))
        v = F.linear(h, t64(store[("wv", l)])).reshape(n, hkv, hd)
        k = k.to(torch.float32).to(torch.float64)  # the cache stores float32
        v = v.to(torch.float32).to(torch.float64)
        K = torch.cat([t64(kv.K[l, :T]), k], dim=0)  # [T+n, hkv, hd]
        V = torch.cat([t64(kv.V[l, :T]), v], dim=0)
        g = hq // hkv
        Kh = K.permute(1, 0, 2).repeat_interleave(g, dim=0)  # [hq, T+n, hd]
        Vh = V.permute(1, 0, 2).repeat_interleave(g, dim=0)
        o = F.scaled_dot_product_attention(q.permute(1, 0, 2), Kh, Vh, attn_mask=allowed[None])  # [hq, n, hd]
        x = x + F.linear(o.permute(1, 0, 2).reshape(n, hq * hd), t64(store[("wo", l)]))
        h = F.rms_norm(x, (sh.d_model,), t64(store[("ffn_norm", l)]), eps=sh.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, t64(store[("wg", l)]))) * F.linear(h, t64(store[("wu", l)])), t64(store[("wd", l)]))
    return F.linear(F.rms_norm(x, (sh.d_model,), t64(store[("final_norm", 0)]), eps=sh.rms_eps), t64(store[("lm_head", 0)])).numpy()


CASES = [("tiny", 12, [-1, 0, 1, 2]), ("tiny_gqa", 9, [-1, 0, 0, 1, 1]), ("tiny_gqa", 0, [-1, 0, 1])]


def _oracle_logits(sh, model, kv, run, toks):
    return oracle.stage_forward(model, kv.clone(), run, 0, sh.n_layers, tokens=toks)["logits"]


@pytest.mark.parametrize("shape_name,n_prefix,parent", CASES)
def test_stack_equals_the_same_stack_built_from_library_routines(shape_name, n_prefix, parent):
    sh, model, store = _random_model(shape_name)
    kv, run, toks = _run_and_cache(sh, n_prefix, parent)
    run = dict(run, parent=np.asarray(parent))
    got = _oracle_logits(sh, model, kv, run, toks)
    ref = _library_forward(sh, store, kv, run, toks)
    assert np.max(np.abs(got - ref)) <= 1e-10 * max(1.0, np.max(np.abs(ref)))


def _zero(l, t):
    return np.zeros_like(t)


def test_all_matrices_zero_gives_lm_head_of_normalised_embedding():
    sh, model, store = _random_model("tiny", overrides={k: _zero for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")})
    kv, run, toks = _run_and_cache(sh, 7, [-1, 0, 1])
    got = _oracle_logits(sh, model, kv, run, toks)
    x = store[("embed", 0)][toks]
    h = x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + sh.rms_eps) * store[("final_norm", 0)]
    assert np.allclose(got, h @ store[("lm_head", 0)].T, rtol=1e-12, atol=1e-14)


def test_zero_gate_or_zero_down_matrix_switches_the_mlp_off_and_zero_up_does_too():
    kvargs = ("tiny", 7, [-1, 0, 1])
    for name in ("wg", "wu", "wd"):
        sh, model, store = _random_model("tiny", overrides={name: _zero})
        sh2, model2, _ = _random_model("tiny", overrides={"wg": _zero, "wu": _zero, "wd": _zero})
        kv, run, toks = _run_and_cache(sh, kvargs[1], kvargs[2])
        assert np.allclose(_oracle_logits(sh, model, kv, run, toks), _oracle_logits(sh2, model2, kv, run, toks),
                           rtol=1e-12, atol=1e-14), name


def test_silu_sits_on_the_gate_branch():
    """One layer, attention off.  With h = the normalised input: gate = -40 h_0 and up = 1 h_1 on
    one FFN feature, the down matrix writing that feature to the output.  silu(-40 h_0) u differs
    from (-40 h_0) silu(u) by orders of magnitude when h_0 > 0, so the branch is unambiguous."""
    def gate(l, t):
        t = np.zeros_like(t); t[0, 0] = -40.0; return t

    def up(l, t):
        t = np.zeros_like(t); t[0, 1] = 1.0; return t

    def down(l, t):
        t = np.zeros_like(t); t[2, 0] = 1.0; return t

    ones = lambda l, t: np.ones_like(t)
    sh, model, store = _random_model("tiny", overrides={"wo": _zero, "wg": gate, "wu": up, "wd": down,
                                                        "ffn_norm": ones, "attn_norm": ones})
    sh = dataclasses.replace(sh, n_layers=1)
    model.shape = sh
    kv, run, toks = _run_and_cache(sh, 3, [-1])
    out = oracle.stage_forward(model, kv.clone(), run, 0, 1, tokens=toks)
    # n_layers == 1: the stage ends at the LM head; read the residual stream through a second call
    sh2 = dataclasses.replace(sh, n_layers=2)
    model.shape = sh2
    kv2 = oracle.OracleKV(sh2, 3 + 64, dtype="f32")
    kv2.kv_len = 3
    x1 = oracle.stage_forward(model, kv2, run, 0, 1, tokens=toks)["hidden"][0]
    x0 = store[("embed", 0)][toks][0]
    h = x0 / np.sqrt(np.mean(x0 * x0) + sh.rms_eps)
    z = -40.0 * h[0]
    want = x0.copy()
    want[2] += z / (1.0 + np.exp(-z)) * h[1]
    assert np.allclose(x1, want, rtol=1e-12, atol=1e-15)
    assert out["logits"] is not None


def test_zero_output_projection_switches_attention_off_but_keys_and_values_are_still_cached():
    sh, model, store = _random_model("tiny_gqa", overrides={"wo": _zero})
    sh2, model2, _ = _random_model("tiny_gqa", overrides={"wo": _zero, "wq": _zero})
    kv, run, toks = _run_and_cache(sh, 5, [-1, 0, 1])
    a, b = kv.clone(), kv.clone()
    la = oracle.stage_forward(model, a, run, 0, sh.n_layers, tokens=toks)["logits"]
    lb = oracle.stage_forward(model2, b, run, 0, sh.n_layers, tokens=toks)["logits"]
    assert np.allclose(la, lb, rtol=1e-12, atol=1e-14)
    assert np.any(a.K[0, run["slots"]] != 0.0) and np.array_equal(a.K, b.K) and np.array_equal(a.V, b.V)


def test_values_are_not_rotated_and_keys_are():
    """Empty prefix and Wk = 0: every score is 0, attention is the plain mean of the visible
    values, so moving the whole run to other positions must leave the logits unchanged -- unless
    the rotary embedding also touched V.  With Wk restored the cached keys do depend on position."""
    sh, model, store = _random_model("tiny_gqa", overrides={"wk": _zero})
    kv, run, toks = _run_and_cache(sh, 0, [-1, 0, 1, 1])
    base = _oracle_logits(sh, model, kv, run, toks)
    moved = dict(run, positions=np.asarray(run["positions"]) + 37)
    assert np.allclose(_oracle_logits(sh, model, kv, moved, toks), base, rtol=1e-12, atol=1e-14)
    sh, model, store = _random_model("tiny_gqa")
    a, b = kv.clone(), kv.clone()
    oracle.stage_forward(model, a, run, 0, 1, tokens=toks)
    oracle.stage_forward(model, b, moved, 0, 1, tokens=toks)
    assert np.array_equal(a.V[0], b.V[0]) and not np.allclose(a.K[0, run["slots"]], b.K[0, run["slots"]])


def test_normalisation_comes_before_each_block_and_the_residual_carries_the_unnormalised_stream():
    """Scaling one token's embedding row by c > 0 leaves what both blocks ADD unchanged (they see
    the normalised stream; eps = 0 here), so the residual stream after a layer is c x0 + (x1 - x0)
    -- not c x1 (post-normalisation would renormalise the sum) and not x1 (dropped residual)."""
    sh, model, store = _random_model("tiny")
    sh = dataclasses.replace(sh, rms_eps=0.0)
    model.shape = sh
    kv, run, toks = _run_and_cache(sh, 6, [-1])
    x1 = oracle.stage_forward(model, kv.clone(), run, 0, 1, tokens=toks)["hidden"][0]
    x0 = store[("embed", 0)][toks][0].copy()
    store[("embed", 0)][toks[0]] *= 3.0
    y1 = oracle.stage_forward(model, kv.clone(), run, 0, 1, tokens=toks)["hidden"][0]
    # the attention block adds d1 (same for both); the MLP sees x0 + d1 resp. 3 x0 + d1, which differ
    # after normalisation, so only the attention part is compared: switch the MLP off
    sh_, model_, store_ = _random_model("tiny", overrides={"wd": _zero})
    sh_ = dataclasses.replace(sh_, rms_eps=0.0)
    model_.shape = sh_
    a0 = store_[("embed", 0)][toks][0].copy()
    a1 = oracle.stage_forward(model_, kv.clone(), run, 0, 1, tokens=toks)["hidden"][0]
    store_[("embed", 0)][toks[0]] *= 3.0
    b1 = oracle.stage_forward(model_, kv.clone(), run, 0, 1, tokens=toks)["hidden"][0]
    assert np.allclose(b1 - 3.0 * a0, a1 - a0, rtol=1e-10, atol=1e-13)
    assert not np.allclose(y1, 3.0 * x1) and not np.allclose(y1, x1)


def test_one_hot_lm_head_reads_one_coordinate_of_the_normalised_stream():
    def head(l, t):
        t = np.zeros_like(t); t[5, 17] = 1.0; t[9, 3] = -2.0; return t
    sh, model, store = _random_model("tiny", overrides={"lm_head": head, "wo": _zero, "wd": _zero})
    kv, run, toks = _run_and_cache(sh, 4, [-1, 0])
    lg = _oracle_logits(sh, model, kv, run, toks)
    x = store[("embed", 0)][toks]
    h = x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + sh.rms_eps) * store[("final_norm", 0)]
    want = np.zeros_like(lg)
    want[:, 5] = h[:, 17]
    want[:, 9] = -2.0 * h[:, 3]
    assert np.allclose(lg, want, rtol=1e-12, atol=1e-15)


# ---- top-2 gap ---------------------------------------------------------------------------------

def test_top2_gap_on_hand_made_rows():
    assert oracle.top2_gap(np.array([0.5, 3.0, -1.0, 2.25])) == 0.75
    assert oracle.top2_gap(np.array([7.0, 7.0, 1.0])) == 0.0                 # a tie has no gap
    assert oracle.top2_gap(np.array([-5.0, -2.0, -9.0])) == 3.0              # all negative
    assert oracle.top2_gap(np.array([1.0, 2.0])) == 1.0                      # the shortest row
    row = RNG.normal(size=1000)
    s = np.sort(row)
    assert oracle.top2_gap(row) == s[-1] - s[-2]
    assert oracle.top2_gap(row[::-1].copy()) == s[-1] - s[-2]                # order of the row does not matter


# ---- the pins above do catch the mistakes they are there for --------------------------------------

def _mutants():
    """stage_forward variants with one plausible mistake each, as source edits of the oracle."""
    import inspect
    src = inspect.getsource(oracle.decoder.stage_forward)
    edits = {
        "silu on up": ("silu(linear(h, model.w(\"wg\", l))) * linear(h, model.w(\"wu\", l))",
                       "linear(h, model.w(\"wg\", l)) * silu(linear(h, model.w(\"wu\", l)))"),
        "attention residual dropped": ("x = x + linear(o.reshape(n, hq * hd), model.w(\"wo\", l))",
                                       "x = linear(o.reshape(n, hq * hd), model.w(\"wo\", l))"),
        "mlp residual dropped": ("x = x + linear(a, model.w(\"wd\", l))", "x = linear(a, model.w(\"wd\", l))"),
        "post-norm": ("x = x + linear(a, model.w(\"wd\", l))",
                      "x = rmsnorm(x + linear(a, model.w(\"wd\", l)), model.w(\"ffn_norm\", l), sh.rms_eps)"),
        "rope on v": ("k = rope(k, pos, sh.rope_base)", "k = rope(k, pos, sh.rope_base); v = rope(v, pos, sh.rope_base)"),
        "no rope on k": ("k = rope(k, pos, sh.rope_base)", "k = k"),
        "ffn norm skipped": ("h = rmsnorm(x, model.w(\"ffn_norm\", l), sh.rms_eps)", "h = x"),
        "final norm skipped": ("linear(rmsnorm(x, model.w(\"final_norm\"), sh.rms_eps), model.w(\"lm_head\"))",
                               "linear(x, model.w(\"lm_head\"))"),
    }
    out = {}
    for name, (old, new) in edits.items():
        assert src.count(old) == 1, name
        ns = dict(vars(oracle.decoder))
        exec(compile(src.replace(old, new), "<mutant %s>" % name, "exec"), ns)
        out[name] = ns["stage_forward"]
    return out


THIS_MODULE_PINS = [
    test_all_matrices_zero_gives_lm_head_of_normalised_embedding,
    test_zero_gate_or_zero_down_matrix_switches_the_mlp_off_and_zero_up_does_too,
    test_silu_sits_on_the_gate_branch,
    test_zero_output_projection_switches_attention_off_but_keys_and_values_are_still_cached,
    test_values_are_not_rotated_and_keys_are,
    test_normalisation_comes_before_each_block_and_the_residual_carries_the_unnormalised_stream,
    test_one_hot_lm_head_reads_one_coordinate_of_the_normalised_stream,
]


@pytest.mark.parametrize("mistake", ["silu on up", "attention residual dropped", "mlp residual dropped", "post-norm",
                                     "rope on v", "no rope on k", "ffn norm skipped", "final norm skipped"])
def test_a_planted_mistake_in_the_oracle_turns_pins_red(mistake, monkeypatch):
    mutant = _mutants()[mistake]
    monkeypatch.setattr(oracle, "stage_forward", mutant)
    monkeypatch.setattr(oracle.decoder, "stage_forward", mutant)
    # the library-built stack catches every one of them ...
    with pytest.raises(AssertionError):
        for case in CASES:
            test_stack_equals_the_same_stack_built_from_library_routines(*case)
    # ... and so does at least one of the special-case pins, which use no library routine at all
    red = 0
    for pin in THIS_MODULE_PINS:
        try:
            pin()
        except AssertionError:
            red += 1
    assert red >= 1, "no special-case pin noticed: %s" % mistake
