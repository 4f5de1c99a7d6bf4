"""Put seeded synthetic inputs on the GPU (device-side generation) and hand them to the
HIP library through its public binding.  Inputs only; no decoder arithmetic."""
from __future__ import annotations

import numpy as np
import torch

import synth
from paper_2407_11798_amd import binding as pi

_KIND_TO_PI = {
    synth.T_EMBED: pi.PI_T_EMBED, synth.T_ATTN_NORM: pi.PI_T_ATTN_NORM, synth.T_WQ: pi.PI_T_WQ,
    synth.T_WK: pi.PI_T_WK, synth.T_WV: pi.PI_T_WV, synth.T_WO: pi.PI_T_WO,
    synth.T_FFN_NORM: pi.PI_T_FFN_NORM, synth.T_WG: pi.PI_T_WG, synth.T_WU: pi.PI_T_WU,
    synth.T_WD: pi.PI_T_WD, synth.T_FINAL_NORM: pi.PI_T_FINAL_NORM, synth.T_LM_HEAD: pi.PI_T_LM_HEAD,
}


def device_normal(n: int, seed: int, sid: int, sigma: float, dtype: str) -> torch.Tensor:
    """Device tensor of n generator values: float32, int16 holding bf16 bit patterns, or uint8
    holding FP8 E4M3 bytes."""
    t = torch.empty(n // 2 if dtype == "fp4" else n, dtype={"f32": torch.float32, "bf16": torch.int16, "fp8": torch.uint8, "fp4": torch.uint8}[dtype],
                    device="cuda")
    synth.normal_device(t.data_ptr(), n, seed, sid, sigma, dtype, torch.cuda.current_stream().cuda_stream)
    return t


def load_model(shape: synth.ModelShape, seed: int, gain_sigma: float = 0.0, max_pos: int = 4096,
               from_host: bool = False) -> pi.Model:
    """Create a pi model and fill every tensor from the seeded generator (device fill by
    default; host fill + upload when from_host is set -- both give the same bits)."""
    m = pi.Model(shape, max_pos=max_pos)

    def put(kind, layer):
        if kind in synth.NORM_KINDS or from_host:
            t = synth.weight_host(shape, seed, kind, layer, gain_sigma)
            code = None
            if t.dtype == np.uint8:
                code = {"fp4": pi.PI_DTYPE_FP4_E2M1, "fp4b": pi.PI_DTYPE_FP4_E2M1_B32}.get(shape.weight_format, pi.PI_DTYPE_FP8_E4M3)
            m.set_tensor(_KIND_TO_PI[kind], layer, t, src_dtype=code)
            return
        rows, cols = synth.tensor_shape(shape, kind)
        if shape.weight_format == "fp4b" and kind != synth.T_EMBED:
            nc, ns = synth.fp4b_sizes(rows, cols)
            t = torch.empty(nc + ns, dtype=torch.uint8, device="cuda")    # codes, then scales: the layout the ABI takes
            rc = synth.hip_lib().synth_fill_normal_fp4b_device(t.data_ptr(), t.data_ptr() + nc, rows, cols, seed,
                                                               synth.stream_id(kind, layer), float(synth.WEIGHT_SIGMA),
                                                               torch.cuda.current_stream().cuda_stream)
            assert rc == 0
            torch.cuda.current_stream().synchronize()
            m.set_tensor(_KIND_TO_PI[kind], layer, t, src_dtype=pi.PI_DTYPE_FP4_E2M1_B32)
            return
        if shape.weight_format in ("fp8", "fp4") and kind != synth.T_EMBED:
            t = device_normal(rows * cols, seed, synth.stream_id(kind, layer),
                              synth.WEIGHT_SIGMA * 2.0 ** -shape.weight_scale_exp2, shape.weight_format)
            torch.cuda.current_stream().synchronize()
            m.set_tensor(_KIND_TO_PI[kind], layer, t,
                         src_dtype=pi.PI_DTYPE_FP4_E2M1 if shape.weight_format == "fp4" else pi.PI_DTYPE_FP8_E4M3)
            return
        t = device_normal(rows * cols, seed, synth.stream_id(kind, layer), synth.WEIGHT_SIGMA, shape.dtype)
        torch.cuda.current_stream().synchronize()
        if shape.dtype == "bf16":
            t = t.view(torch.bfloat16)
        m.set_tensor(_KIND_TO_PI[kind], layer, t)

    for kind in synth.GLOBAL_KINDS:
        put(kind, 0)
    for layer in range(shape.n_layers):
        for kind in synth.LAYER_KINDS:
            put(kind, layer)
    return m


def prefill_kv_synthetic(kv: pi.KVCache, shape: synth.ModelShape, seed: int, n_prefill: int) -> None:
    """Synthetic prefill: K, V ~ N(0,1) in the cache dtype for cells [0, n_prefill)."""
    n = n_prefill * shape.n_kv_heads * shape.head_dim
    for layer in range(shape.n_layers):
        k = device_normal(n, seed, synth.stream_id(synth.T_KV_K, layer), 1.0, shape.dtype)
        v = device_normal(n, seed, synth.stream_id(synth.T_KV_V, layer), 1.0, shape.dtype)
        torch.cuda.current_stream().synchronize()
        if shape.dtype == "bf16":
            k, v = k.view(torch.bfloat16), v.view(torch.bfloat16)
        kv.set_cells(layer, 0, k.view(n_prefill, shape.n_kv_heads, shape.head_dim),
                     v.view(n_prefill, shape.n_kv_heads, shape.head_dim))
    kv.set_len(n_prefill)


def make_run(run: dict, tokens) -> pi.Run:
    return pi.Run(tokens, run["positions"], run["slots"], run["mask"], run["prefix_len"],
                  run["window_base"], parent=run.get("parent"))
