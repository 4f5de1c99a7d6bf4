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


def model_from_seed(shape: synth.ModelShape, seed: int, gain_sigma: float = 0.0,
                    cache: bool = True) -> OracleModel:
    """Weights are regenerated from the seed when asked for; `cache` keeps them (small models)."""
    store = {}

    def weights(name, layer):
        key = (name, layer)
        if key in store:
            return store[key]
        t = synth.weight_host(shape, seed, _NAME_TO_KIND[name], layer, gain_sigma)
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
