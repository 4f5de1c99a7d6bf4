"""CPU oracle for the speculative-verification hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what one target-model verification run computes:
a Llama-style decoder stack evaluated on a micro-batch of speculated tokens over a KV
cache with a tree attention mask, greedy token verification, KV commit/rollback and
cancellation at a layer boundary.  Nothing here is tuned, blocked or fused, and nothing
is shared with the HIP library (no code, tables or helpers); only tests, the smoke check
and the benchmark's cpu_baseline leg may import it.

What the paper fixes (and where):
  * layers are evaluated in sequence, each an attention module plus an MLP, with K/V
    cached per token                      -- Section "Background and Motivation"
  * all tokens of a speculated tree go through the target model in one batch under a
    mask that keeps tree branches mutually invisible while preserving causality, giving
    one logit vector per tree token        -- Section "Speculative Inference / Verification"
  * a speculated token is accepted iff the target's own choice at that point equals it;
    the first mismatch ends verification with the target's token; a fully accepted
    branch yields a bonus token from its leaf  -- same section; greedy sampling per
    Section "Experiments"
  * speculative runs write K/V only into private cells; accepted entries are then
    copied to the canonical sequence and the rest removed
                                           -- Section "Pipelined KV Cache Multibuffering"
  * a cancelled run stops at a synchronisation point and leaves state consistent
                                           -- Section "Early Inference Cancellation"
The decoder formulas themselves are not printed in the paper (it refers to Llama 2); the
readings taken here are: pre-norm RMSNorm, no biases, rotary embedding on adjacent pairs
(2t, 2t+1) with angle pos * base^(-2t/hd), softmax scale 1/sqrt(hd), grouped-query
sharing hq -> hq // (Hq/Hkv), SwiGLU MLP, untied LM head after a final RMSNorm.

Precision: all arithmetic in fp64.  Storage contracts are part of the method and are
applied explicitly: weights arrive already rounded to their storage type; K/V are
rounded to the cache type (fp32 or bf16, round-to-nearest-even) when stored.
"""
from __future__ import annotations

import numpy as np

PI_OK = 0
PI_CANCELLED = 1


# ----------------------------------------------------------------------------- storage types

def _bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_f64(t: np.ndarray) -> np.ndarray:
    """Weights/KV arrive as float32 values or as uint16 bf16 bit patterns."""
    if t.dtype == np.uint16:
        return _bf16_bits_to_f64(t)
    return t.astype(np.float64)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 values -> the values a cache of type `dtype` would hold, returned as fp64."""
    f = x.astype(np.float32)  # RNE
    if dtype == "f32":
        return f.astype(np.float64)
    assert dtype == "bf16"
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16  # RNE to the upper 16 bits
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- operators

def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x[n,d] * gain / sqrt(mean_j x_j^2 + eps)."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * gain / np.sqrt(ms + eps)


def linear(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y[n,out] = x[n,in] . w[out,in]^T  (no bias)."""
    return x @ w.T


def rope(x: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotate each head's adjacent pairs (2t, 2t+1) by angle pos * base^(-2t/hd).
    x: [n, heads, hd]."""
    n, h, hd = x.shape
    t = np.arange(hd // 2, dtype=np.float64)
    theta = base ** (-2.0 * t / hd)
    ang = positions.astype(np.float64)[:, None] * theta[None, :]  # [n, hd/2]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x0, x1 = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = x0 * c - x1 * s
    out[..., 1::2] = x0 * s + x1 * c
    return out


def visible_cells(prefix_len: int, window_base: int, mask_word: int) -> np.ndarray:
    """Cells token i may attend to: the shared prefix plus the window cells in its mask."""
    win = [window_base + c for c in range(64) if (int(mask_word) >> c) & 1]
    return np.concatenate([np.arange(prefix_len, dtype=np.int64), np.asarray(win, dtype=np.int64)])


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, prefix_len: int, window_base: int,
              mask: np.ndarray) -> np.ndarray:
    """q: [n, Hq, hd]; K, V: [cells, Hkv, hd] (one layer).  Returns o: [n, Hq, hd]."""
    n, hq, hd = q.shape
    hkv = K.shape[1]
    g = hq // hkv
    o = np.zeros_like(q)
    for i in range(n):
        cells = visible_cells(prefix_len, window_base, mask[i])
        assert len(cells) > 0
        for h in range(hq):
            kh = K[cells, h // g, :]
            vh = V[cells, h // g, :]
            s = kh @ q[i, h, :] / np.sqrt(float(hd))
            p = np.exp(s - np.max(s))
            p = p / np.sum(p)
            o[i, h, :] = p @ vh
    return o


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


# ----------------------------------------------------------------------------- model + cache

class OracleModel:
    """shape: any object with n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
    rms_eps, rope_base, dtype.  `weights(name, layer)` returns the stored tensor (float32
    or uint16 bf16 bits) for name in embed, attn_norm, wq, wk, wv, wo, ffn_norm, wg, wu, wd,
    final_norm, lm_head; it is called when the tensor is needed, so very large models can be
    produced layer by layer."""

    def __init__(self, shape, weights):
        self.shape = shape
        self.weights = weights

    def w(self, name, layer=0):
        return to_f64(self.weights(name, layer))


class OracleKV:
    """K, V: [n_layers, n_cells, Hkv, hd] fp64 holding cache-type-rounded values; zero = free."""

    def __init__(self, shape, n_cells: int, dtype: str | None = None):
        self.dtype = dtype or shape.dtype
        dims = (shape.n_layers, n_cells, shape.n_kv_heads, shape.head_dim)
        self.K = np.zeros(dims, dtype=np.float64)
        self.V = np.zeros(dims, dtype=np.float64)
        self.kv_len = 0
        self.n_cells = n_cells

    def set_cells(self, layer: int, cell0: int, k: np.ndarray, v: np.ndarray):
        n = k.shape[0]
        self.K[layer, cell0:cell0 + n] = round_to_storage(to_f64(k), self.dtype)
        self.V[layer, cell0:cell0 + n] = round_to_storage(to_f64(v), self.dtype)

    def clone(self):
        c = OracleKV.__new__(OracleKV)
        c.dtype, c.kv_len, c.n_cells = self.dtype, self.kv_len, self.n_cells
        c.K, c.V = self.K.copy(), self.V.copy()
        return c


# ----------------------------------------------------------------------------- the run

def stage_forward(model: OracleModel, kv: OracleKV, run: dict, layer_begin: int, layer_end: int,
                  tokens: np.ndarray | None = None, hidden_in: np.ndarray | None = None,
                  cancel_before_layer: int | None = None) -> dict:
    """Evaluate layers [layer_begin, layer_end) of one verification run.

    run: dict with positions[n], slots[n], mask[n] (uint64), prefix_len, window_base.
    A cancel takes effect at a layer boundary: cancel_before_layer = l means the flag was
    seen before layer l started, so layers >= l do nothing (no K/V writes, no output).
    Returns status, layers_done (absolute index of the first layer not evaluated), and
    hidden [n,d] or logits [n,V] when the stage ran to its end.
    """
    sh = model.shape
    n = len(run["positions"])
    pos = np.asarray(run["positions"])
    slots = np.asarray(run["slots"])
    if np.any(slots < kv.kv_len):
        raise ValueError("speculative write into a live canonical cell")
    if layer_begin == 0:
        x = model.w("embed")[np.asarray(tokens), :]
    else:
        x = np.asarray(hidden_in, dtype=np.float64).copy()
    hq, hkv, hd = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    for l in range(layer_begin, layer_end):
        if cancel_before_layer is not None and cancel_before_layer <= l:
            return {"status": PI_CANCELLED, "layers_done": l, "hidden": None, "logits": None}
        h = rmsnorm(x, model.w("attn_norm", l), sh.rms_eps)
        q = linear(h, model.w("wq", l)).reshape(n, hq, hd)
        k = linear(h, model.w("wk", l)).reshape(n, hkv, hd)
        v = linear(h, model.w("wv", l)).reshape(n, hkv, hd)
        q = rope(q, pos, sh.rope_base)
        k = rope(k, pos, sh.rope_base)
        kv.K[l, slots] = round_to_storage(k, kv.dtype)   # every write of the layer lands
        kv.V[l, slots] = round_to_storage(v, kv.dtype)   # before any read of the layer
        o = attention(q, kv.K[l], kv.V[l], run["prefix_len"], run["window_base"], run["mask"])
        x = x + linear(o.reshape(n, hq * hd), model.w("wo", l))
        h = rmsnorm(x, model.w("ffn_norm", l), sh.rms_eps)
        a = silu(linear(h, model.w("wg", l))) * linear(h, model.w("wu", l))
        x = x + linear(a, model.w("wd", l))
    out = {"status": PI_OK, "layers_done": layer_end, "hidden": None, "logits": None}
    if layer_end == sh.n_layers:
        out["logits"] = linear(rmsnorm(x, model.w("final_norm"), sh.rms_eps), model.w("lm_head"))
    else:
        out["hidden"] = x
    return out


def verify_greedy(draft: np.ndarray, parent: np.ndarray | None, logits: np.ndarray,
                  root_expected: int):
    """Greedy token-tree verification.

    logits[i] is the target's distribution for the token that follows tree node i.
    Starting at the root (u = -1) with expected = the target's choice after the last
    accepted token, accept the lowest-index child of u whose draft token equals
    `expected`; then expected becomes argmax(logits[child]) (lowest id on ties).  Stop at
    the first node with no matching child.  Returns (count, accepted node list, bonus):
    bonus is the target's own next token after the accepted path.
    """
    n = len(draft)
    if parent is None:
        parent = np.arange(-1, n - 1)
    u, expected, acc = -1, int(root_expected), []
    while True:
        nxt = -1
        for c in range(n):
            if int(parent[c]) == u and int(draft[c]) == expected:
                nxt = c
                break
        if nxt < 0:
            break
        acc.append(nxt)
        u = nxt
        expected = int(np.argmax(logits[nxt]))
    return len(acc), acc, expected


def verify_greedy_chained(draft, parent, logits, root_expected, prev_result=None, prev_n=0, run_ok=True):
    """Verification of a run that builds on another run's speculation (Section "Continuous
    Speculation"): it counts only if the run it builds on accepted all prev_n of its tokens
    -- that run's bonus token is then what the root is checked against -- and only if its own
    forward ran to the end.  Otherwise nothing is accepted and there is no bonus token (-1).
    prev_result: (accepted count, bonus token) of the earlier run, or None for a run that
    starts at the accepted end (root_expected is used)."""
    n = len(draft)
    if prev_result is not None:
        if int(prev_result[0]) != int(prev_n):
            return 0, [], -1
        root_expected = int(prev_result[1])
    if not run_ok:
        return 0, [], -1
    return verify_greedy(draft, parent, logits, root_expected)


def kv_rollback(kv: OracleKV, slots: np.ndarray, accepted_nodes: list[int]) -> None:
    """Commit the accepted path to canonical cells kv_len .. kv_len+a-1 (path order), free
    (zero) every other cell the run wrote, and advance kv_len by a.  A cancelled or fully
    rejected run is the case a = 0."""
    slots = np.asarray(slots)
    a = len(accepted_nodes)
    src = [int(slots[i]) for i in accepted_nodes]
    keepK = kv.K[:, src].copy()
    keepV = kv.V[:, src].copy()
    kv.K[:, slots] = 0.0
    kv.V[:, slots] = 0.0
    kv.K[:, kv.kv_len:kv.kv_len + a] = keepK
    kv.V[:, kv.kv_len:kv.kv_len + a] = keepV
    kv.kv_len += a


def top2_gap(logits_row: np.ndarray) -> float:
    s = np.partition(logits_row, -2)[-2:]
    return float(s[1] - s[0])
