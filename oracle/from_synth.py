"""Glue (test infrastructure): feed the oracle with the seeded synthetic inputs."""
from __future__ import annotations

import numpy as np

import synth
from .decoder import OracleModel, OracleKV

_NAME_TO_KIND = {
    "embed": synth.T_EMBED, "attn_norm": synth.T_ATTN_NORM, "wq": synth.T_WQ, "wk": synth.T_WK,
    "wv": synth.T_WV, "wo": synth.T_WO, "ffn_norm": synth.T_FFN_NORM, "wg": synth.T_WG,
    "wu": synth.T_WU, "wd": synth.T_WD, "final_norm": synth.T_FINAL_NORM,
    "lm_head": synth.T_LM_HEAD,
}


def _e4m3_table() -> np.ndarray:
    """Value of every FP8 E4M3 byte (sign, 4 exponent bits with bias 7, 3 mantissa bits,
    subnormals at exponent 0, no infinities; 0x7f and 0xff are NaN)."""
    t = np.empty(256, dtype=np.float64)
    for b in range(256):
        sign = -1.0 if b & 0x80 else 1.0
        e, m = (b >> 3) & 0xF, b & 7
        if e == 15 and m == 7:
            t[b] = np.nan
        elif e == 0:
            t[b] = sign * (m / 8.0) * 2.0 ** -6
        else:
            t[b] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


E4M3 = _e4m3_table()


def dequantise_fp8(codes: np.ndarray, scale_exp2: int) -> np.ndarray:
    """8-bit weights as the model defines them: e4m3(byte) * 2^scale_exp2 (exact in float32)."""
    return (E4M3[codes] * 2.0 ** scale_exp2).astype(np.float32)


E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0] + [-0.0, -0.5, -1.0, -1.5, -2.0, -3.0, -4.0, -6.0])


def dequantise_fp4(packed: np.ndarray, scale_exp2: int) -> np.ndarray:
    """4-bit weights as the model defines them: packed[r][j] holds columns 2j (low nibble) and
    2j+1 (high nibble) of row r as FP4 E2M1 codes (sign, 2 exponent bits, 1 mantissa bit);
    weight = e2m1(code) * 2^scale_exp2."""
    rows, half = packed.shape
    out = np.empty((rows, 2 * half), dtype=np.float64)
    out[:, 0::2] = E2M1[packed & 0xF]
    out[:, 1::2] = E2M1[packed >> 4]
    return (out * 2.0 ** scale_exp2).astype(np.float32)


def dequantise_fp4_blocks(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """Block-scaled 4-bit weights as the model defines them: codes[r][j] holds columns 2j (low
    nibble) and 2j+1 (high nibble) of row r as FP4 E2M1 codes; scales[r][b] belongs to columns
    32b .. 32b+31 of row r; weight = e2m1(code) * 2^(scale - 127)."""
    rows, half = codes.shape
    out = np.empty((rows, 2 * half), dtype=np.float64)
    out[:, 0::2] = E2M1[codes & 0xF]
    out[:, 1::2] = E2M1[codes >> 4]
    per_col = np.repeat(scales.astype(np.int64), 32, axis=1)[:, :2 * half]
    return (out * np.exp2((per_col - 127).astype(np.float64))).astype(np.float32)


def dequantise(shape, kind: int, t: np.ndarray) -> np.ndarray:
    """A stored tensor of `shape` as the values the model defines (quantised matrices decoded)."""
    if t.dtype != np.uint8:
        return t
    if shape.weight_format == "fp4b":
        rows, cols = synth.tensor_shape(shape, kind)
        return dequantise_fp4_blocks(*synth.split_fp4b(t, rows, cols))
    return (dequantise_fp4 if shape.weight_format == "fp4" else dequantise_fp8)(t, shape.weight_scale_exp2)


def model_from_seed(shape: synth.ModelShape, seed: int, gain_sigma: float = 0.0,
                    cache: bool = True) -> OracleModel:
    """Weights are regenerated from the seed when asked for; `cache` keeps them (small models)."""
    store = {}

    def weights(name, layer):
        key = (name, layer)
        if key in store:
            return store[key]
        t = dequantise(shape, _NAME_TO_KIND[name], synth.weight_host(shape, seed, _NAME_TO_KIND[name], layer, gain_sigma))
        if cache:
            store[key] = t
        return t

    return OracleModel(shape, weights)


def kv_synthetic(shape: synth.ModelShape, seed: int, n_cells: int, n_prefill: int) -> OracleKV:
    kv = OracleKV(shape, n_cells)
    for l in range(shape.n_layers):
        k, v = synth.kv_prefill_host(shape, seed, l, n_prefill)
        kv.set_cells(l, 0, k, v)
    kv.kv_len = n_prefill
    return kv
