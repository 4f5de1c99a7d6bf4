"""Seeded synthetic inputs shared by the oracle side and the HIP side.

This package only *makes inputs*: model shapes, seeded Gaussian tensors, token ids,
speculation trees, masks and cancel schedules.  None of the decoder's arithmetic lives
here.  The Gaussian generator (synth_core.h) is a counter-based Box-Muller written with
exactly-rounded operations only, so the host fill (gcc) and the device fill (hipcc)
produce bit-identical tensors for the same (seed, stream).

Workload shapes follow the models the paper evaluates (a Llama-2-70B-class target, 7B
and TinyLlama-class drafts; Section "Experiments", model table) and its speculative
micro-batch sizes of 1-4 tokens (Section "Continuous Speculation / Microbatching").
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, asdict

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_HOST_SO = os.path.join(_HERE, "libpisynth_host.so")
_HIP_SO = os.path.join(_HERE, "libpisynth_hip.so")

# ----------------------------------------------------------------------------- shapes


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: str = "bf16"  # storage type of weights and KV cache: "f32" or "bf16"
    # "fp8" / "fp4": the weight matrices (not the embedding table) are FP8 E4M3 bytes / FP4 E2M1
    # nibbles (two per byte) and the weight is code value * 2^weight_scale_exp2; "fp4b": FP4 E2M1
    # nibbles with one power-of-two scale per 32 columns of a row (weight = code value *
    # 2^(scale byte - 127)); everything else follows `dtype`
    weight_format: str = "native"
    weight_scale_exp2: int = 0

    def as_dict(self):
        return asdict(self)

    @property
    def layer_params(self) -> int:
        d, hq, hkv, hd, f = self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.ffn
        return d * hq * hd + 2 * d * hkv * hd + hq * hd * d + 3 * d * f

    @property
    def bytes_per_weight(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def bytes_per_matrix_weight(self) -> int:
        return {"fp8": 1, "fp4": 0.5, "fp4b": 0.53125}.get(self.weight_format, self.bytes_per_weight)


SHAPES = {
    "tiny": ModelShape("tiny", 2, 256, 4, 4, 64, 688, 1024, dtype="f32"),
    "tiny_bf16": ModelShape("tiny_bf16", 2, 256, 4, 4, 64, 688, 1024, dtype="bf16"),
    "tiny_gqa": ModelShape("tiny_gqa", 3, 256, 8, 2, 32, 352, 512, dtype="bf16"),
    "llama7b": ModelShape("llama7b", 32, 4096, 32, 32, 128, 11008, 32000),
    "tinyllama": ModelShape("tinyllama", 22, 2048, 32, 4, 64, 5632, 32000),
    "llama70b": ModelShape("llama70b", 80, 8192, 64, 8, 128, 28672, 32000),
    # the same shapes with 8-bit weight matrices; N(0, 0.02) times 2^11 sits well inside +-448
    "tiny_w8": ModelShape("tiny_w8", 2, 256, 4, 4, 64, 688, 1024, weight_format="fp8", weight_scale_exp2=-11),
    "tiny_gqa_w8": ModelShape("tiny_gqa_w8", 3, 256, 8, 2, 32, 352, 512, weight_format="fp8", weight_scale_exp2=-11),
    "llama7b_w8": ModelShape("llama7b_w8", 32, 4096, 32, 32, 128, 11008, 32000, weight_format="fp8",
                             weight_scale_exp2=-11),
    "llama70b_w8": ModelShape("llama70b_w8", 80, 8192, 64, 8, 128, 28672, 32000, weight_format="fp8",
                              weight_scale_exp2=-11),
    # 4-bit weight matrices; N(0, 0.02) times 2^6 has its standard deviation at 1.28 of a range of +-6
    "tiny_w4": ModelShape("tiny_w4", 2, 256, 4, 4, 64, 688, 1024, weight_format="fp4", weight_scale_exp2=-6),
    "tiny_gqa_w4": ModelShape("tiny_gqa_w4", 3, 256, 8, 2, 32, 352, 512, weight_format="fp4", weight_scale_exp2=-6),
    "llama7b_w4": ModelShape("llama7b_w4", 32, 4096, 32, 32, 128, 11008, 32000, weight_format="fp4",
                             weight_scale_exp2=-6),
    "llama70b_w4": ModelShape("llama70b_w4", 80, 8192, 64, 8, 128, 28672, 32000, weight_format="fp4",
                              weight_scale_exp2=-6),
    # 4-bit weight matrices with one power-of-two scale per 32 columns of a row (4.25 bits per weight)
    "tiny_w4b": ModelShape("tiny_w4b", 2, 256, 4, 4, 64, 688, 1024, weight_format="fp4b"),
    "tiny_gqa_w4b": ModelShape("tiny_gqa_w4b", 3, 256, 8, 2, 32, 352, 512, weight_format="fp4b"),
    "llama7b_w4b": ModelShape("llama7b_w4b", 32, 4096, 32, 32, 128, 11008, 32000, weight_format="fp4b"),
    "llama70b_w4b": ModelShape("llama70b_w4b", 80, 8192, 64, 8, 128, 28672, 32000, weight_format="fp4b"),
}

# Tensor kinds (also the upper part of the generator stream id).
T_EMBED, T_ATTN_NORM, T_WQ, T_WK, T_WV, T_WO, T_FFN_NORM, T_WG, T_WU, T_WD, T_FINAL_NORM, T_LM_HEAD = range(12)
T_KV_K, T_KV_V, T_TOKENS, T_DRAFT, T_TREE, T_CANCEL, T_MISC = range(12, 19)

WEIGHT_SIGMA = 0.02


def stream_id(kind: int, layer: int = 0) -> int:
    return (kind << 32) | (layer & 0xFFFFFFFF)


def tensor_shape(shape: ModelShape, kind: int):
    """Logical (rows, cols) of a weight tensor; matrices are [out_features, in_features]."""
    d, hq, hkv, hd, f, v = (shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                            shape.ffn, shape.vocab)
    return {
        T_EMBED: (v, d), T_ATTN_NORM: (d,), T_WQ: (hq * hd, d), T_WK: (hkv * hd, d),
        T_WV: (hkv * hd, d), T_WO: (d, hq * hd), T_FFN_NORM: (d,), T_WG: (f, d), T_WU: (f, d),
        T_WD: (d, f), T_FINAL_NORM: (d,), T_LM_HEAD: (v, d),
    }[kind]


LAYER_KINDS = (T_ATTN_NORM, T_WQ, T_WK, T_WV, T_WO, T_FFN_NORM, T_WG, T_WU, T_WD)
GLOBAL_KINDS = (T_EMBED, T_FINAL_NORM, T_LM_HEAD)
NORM_KINDS = (T_ATTN_NORM, T_FFN_NORM, T_FINAL_NORM)

# ----------------------------------------------------------------------------- build/load


def build(verbose: bool = False) -> None:
    """Compile the host fill (gcc) and the device fill (hipcc, gfx950)."""
    cmds = [
        ["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", _HOST_SO,
         os.path.join(_HERE, "synth_host.c"), "-lm"],
        ["hipcc", "--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", _HIP_SO,
         os.path.join(_HERE, "synth_device.hip")],
    ]
    for c in cmds:
        r = subprocess.run(c, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("synth build failed: %s\n%s" % (" ".join(c), r.stderr))
        if verbose:
            print("built", c[c.index("-o") + 1])


_host = None
_hip = None


def host_lib():
    global _host
    if _host is None:
        if not os.path.exists(_HOST_SO):
            build()
        _host = ctypes.CDLL(_HOST_SO)
        _host.synth_fill_normal_host.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64,
                                                 ctypes.c_uint64, ctypes.c_double, ctypes.c_int]
        _host.synth_fill_uniform_int_host.argtypes = [ctypes.c_void_p, ctypes.c_int64,
                                                      ctypes.c_uint64, ctypes.c_uint64,
                                                      ctypes.c_uint32]
        _host.synth_debug_pair_host.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                                ctypes.c_void_p]
        _host.synth_debug_e4m3_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        _host.synth_debug_e2m1_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64]
        _host.synth_fill_normal_fp4b_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                                      ctypes.c_uint64, ctypes.c_uint64, ctypes.c_double]
    return _host


def hip_lib():
    global _hip
    if _hip is None:
        if not os.path.exists(_HIP_SO):
            raise RuntimeError("synth device library missing: run __graft_entry__.build() first")
        import torch  # noqa: F401  (its HIP runtime first: the fills write into torch's device memory)
        _hip = ctypes.CDLL(_HIP_SO)
        _hip.synth_fill_normal_device.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64,
                                                  ctypes.c_uint64, ctypes.c_double, ctypes.c_int,
                                                  ctypes.c_void_p]
        _hip.synth_fill_uniform_int_device.argtypes = [ctypes.c_void_p, ctypes.c_int64,
                                                       ctypes.c_uint64, ctypes.c_uint64,
                                                       ctypes.c_uint32, ctypes.c_void_p]
        _hip.synth_fill_normal_fp4b_device.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                                       ctypes.c_uint64, ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p]
    return _hip


# ----------------------------------------------------------------------------- host fills


_CODE = {"f32": 0, "bf16": 1, "fp8": 2, "fp4": 3}
_NP = {"f32": np.float32, "bf16": np.uint16, "fp8": np.uint8, "fp4": np.uint8}


def normal_host(n: int, seed: int, sid: int, sigma: float, dtype: str) -> np.ndarray:
    """n values ~ N(0, sigma^2); dtype "f32" -> float32 array, "bf16" -> uint16 bit patterns,
    "fp8" -> FP8 E4M3 bytes, "fp4" -> n/2 bytes of two FP4 E2M1 nibbles each, element 2p in the
    low nibble (both round to nearest even, saturating)."""
    out = np.empty(n // 2 if dtype == "fp4" else n, dtype=_NP[dtype])
    rc = host_lib().synth_fill_normal_host(out.ctypes.data, n, seed, sid, float(sigma), _CODE[dtype])
    if rc != 0:
        raise RuntimeError("synth_fill_normal_host failed")
    return out


def fp4b_sizes(rows: int, cols: int):
    """Bytes of codes and of scales of a block-scaled 4-bit matrix [rows][cols]."""
    return rows * cols // 2, rows * ((cols + 31) // 32)


def normal_fp4b_host(rows: int, cols: int, seed: int, sid: int, sigma: float) -> np.ndarray:
    """A block-scaled 4-bit matrix ~ N(0, sigma^2) as ONE uint8 array: codes[rows][cols / 2] (two FP4
    E2M1 nibbles per byte, even column low) followed by scales[rows][ceil(cols / 32)] (weight = code
    value * 2^(scale - 127), one scale per 32 columns of a row, chosen so that the block's largest
    magnitude lands in [4, 8) before rounding)."""
    nc, ns = fp4b_sizes(rows, cols)
    out = np.empty(nc + ns, dtype=np.uint8)
    rc = host_lib().synth_fill_normal_fp4b_host(out.ctypes.data, out.ctypes.data + nc, rows, cols, seed, sid, float(sigma))
    if rc != 0:
        raise RuntimeError("synth_fill_normal_fp4b_host failed")
    return out


def split_fp4b(buf: np.ndarray, rows: int, cols: int):
    """(codes[rows][cols / 2], scales[rows][ceil(cols / 32)]) views of a block-scaled 4-bit matrix."""
    nc, ns = fp4b_sizes(rows, cols)
    return buf[:nc].reshape(rows, cols // 2), buf[nc:nc + ns].reshape(rows, (cols + 31) // 32)


def uniform_int_host(n: int, seed: int, sid: int, rng: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    rc = host_lib().synth_fill_uniform_int_host(out.ctypes.data, n, seed, sid, rng)
    if rc != 0:
        raise RuntimeError("synth_fill_uniform_int_host failed")
    return out


def f32_to_e4m3_host(x: np.ndarray) -> np.ndarray:
    """The generator's FP8 rounding applied to given floats (for pin tests)."""
    src = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(src.size, dtype=np.uint8)
    host_lib().synth_debug_e4m3_host(src.ctypes.data, out.ctypes.data, src.size)
    return out.reshape(src.shape)


def f32_to_e2m1_host(x: np.ndarray) -> np.ndarray:
    """The generator's FP4 rounding applied to given floats: one nibble per element (for pin tests)."""
    src = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(src.size, dtype=np.uint8)
    host_lib().synth_debug_e2m1_host(src.ctypes.data, out.ctypes.data, src.size)
    return out.reshape(src.shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def weight_host(shape: ModelShape, seed: int, kind: int, layer: int = 0,
                gain_sigma: float = 0.0) -> np.ndarray:
    """One weight tensor in its storage dtype (float32, uint16 bf16 bits, or -- the matrices of
    a shape with 8-bit weights -- FP8 E4M3 bytes of the value times 2^-weight_scale_exp2).

    Matrices ~ N(0, 0.02^2).  RMSNorm gains are exactly 1 (gain_sigma = 0, the default
    recipe) or 1 + N(0, gain_sigma^2) (used by tests so that a dropped gain is visible);
    gains are always float32.
    """
    dims = tensor_shape(shape, kind)
    n = int(np.prod(dims))
    if kind in NORM_KINDS:
        if gain_sigma == 0.0:
            return np.ones(dims, dtype=np.float32)
        return (1.0 + normal_host(n, seed, stream_id(kind, layer), gain_sigma, "f32")).astype(
            np.float32).reshape(dims)
    if shape.weight_format == "fp8" and kind != T_EMBED:
        return normal_host(n, seed, stream_id(kind, layer), WEIGHT_SIGMA * 2.0 ** -shape.weight_scale_exp2,
                           "fp8").reshape(dims)
    if shape.weight_format == "fp4b" and kind != T_EMBED:
        return normal_fp4b_host(dims[0], dims[1], seed, stream_id(kind, layer), WEIGHT_SIGMA)
    if shape.weight_format == "fp4" and kind != T_EMBED:
        return normal_host(n, seed, stream_id(kind, layer), WEIGHT_SIGMA * 2.0 ** -shape.weight_scale_exp2,
                           "fp4").reshape(dims[0], dims[1] // 2)
    return normal_host(n, seed, stream_id(kind, layer), WEIGHT_SIGMA, shape.dtype).reshape(dims)


def kv_prefill_host(shape: ModelShape, seed: int, layer: int, n_cells: int):
    """Synthetic K and V for cells [0, n_cells) of one layer: N(0,1) in the cache dtype,
    logical layout [n_cells, n_kv_heads, head_dim]."""
    n = n_cells * shape.n_kv_heads * shape.head_dim
    dims = (n_cells, shape.n_kv_heads, shape.head_dim)
    k = normal_host(n, seed, stream_id(T_KV_K, layer), 1.0, shape.dtype).reshape(dims)
    v = normal_host(n, seed, stream_id(T_KV_V, layer), 1.0, shape.dtype).reshape(dims)
    return k, v


def tokens_host(shape: ModelShape, seed: int, n: int, kind: int = T_TOKENS, salt: int = 0):
    return uniform_int_host(n, seed, stream_id(kind, salt), shape.vocab)


# ----------------------------------------------------------------------------- device fills


def normal_device(ptr: int, n: int, seed: int, sid: int, sigma: float, dtype: str,
                  stream: int = 0) -> None:
    rc = hip_lib().synth_fill_normal_device(ptr, n, seed, sid, float(sigma), _CODE[dtype], stream)
    if rc != 0:
        raise RuntimeError("synth_fill_normal_device failed (%d)" % rc)


# ----------------------------------------------------------------------------- structure


def linear_run(n: int, prefix_len: int, window_base: int | None = None, offset: int = 0):
    """A linear chain of n speculated tokens: parent[i] = i-1, position = prefix_len + i,
    slot = window_base + offset + i, mask_i = own slot and all earlier slots of the run."""
    if window_base is None:
        window_base = prefix_len
    parent = np.arange(-1, n - 1, dtype=np.int32)
    return tree_run(parent, prefix_len, window_base, offset)


def tree_run(parent: np.ndarray, prefix_len: int, window_base: int, offset: int = 0):
    """Positions, slots and window masks of a speculation tree given parent[] (parent < child,
    -1 = child of the last accepted token).  A node sees the shared prefix, its ancestors and
    itself; siblings and other branches stay invisible (tree attention mask)."""
    n = len(parent)
    depth = np.zeros(n, dtype=np.int32)
    mask = np.zeros(n, dtype=np.uint64)
    for i in range(n):
        p = int(parent[i])
        assert -1 <= p < i
        bit = np.uint64(1) << np.uint64(offset + i)
        if p >= 0:
            depth[i] = depth[p] + 1
            mask[i] = mask[p] | bit
        else:
            mask[i] = bit
    positions = (prefix_len + depth).astype(np.int32)
    slots = (window_base + offset + np.arange(n)).astype(np.int32)
    return {"parent": np.asarray(parent, dtype=np.int32), "positions": positions, "slots": slots,
            "mask": mask, "prefix_len": int(prefix_len), "window_base": int(window_base), "n": n}


def tree_sequences(parent: np.ndarray, ids):
    """One sequence identifier per branch: the k-th leaf (in node order) takes ids[k], and a
    node belongs to the sequences of all leaves below it.  Returns a list of sorted lists."""
    n = len(parent)
    is_leaf = [True] * n
    for i in range(n):
        if parent[i] >= 0:
            is_leaf[int(parent[i])] = False
    sets = [set() for _ in range(n)]
    k = 0
    for i in range(n):
        if is_leaf[i]:
            j = i
            while j >= 0:
                sets[j].add(int(ids[k]))
                j = int(parent[j])
            k += 1
    return [sorted(s) for s in sets]


def n_leaves(parent: np.ndarray) -> int:
    has_child = set(int(p) for p in parent if p >= 0)
    return len(parent) - len(has_child)


def random_tree(seed: int, salt: int, n: int, max_children: int = 3, max_depth: int = 4):
    """Seeded growth: node 0 is a root; node k attaches to a uniformly chosen earlier node
    that still has < max_children children and depth < max_depth-1 (depth counts the root
    as 1), or becomes another root if none qualifies."""
    r = uniform_int_host(4 * n + 4, seed, stream_id(T_TREE, salt), 1 << 30)
    parent = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int32)
    nchild = np.zeros(n, dtype=np.int32)
    for k in range(1, n):
        cand = [j for j in range(k) if nchild[j] < max_children and depth[j] + 1 < max_depth]
        if cand:
            p = cand[int(r[k]) % len(cand)]
            parent[k] = p
            depth[k] = depth[p] + 1
            nchild[p] += 1
    return parent


def sibling_distinct_tokens(shape: ModelShape, seed: int, salt: int, parent: np.ndarray):
    """Uniform-random draft tokens, redrawn so that siblings carry distinct tokens."""
    n = len(parent)
    pool = uniform_int_host(8 * n + 8, seed, stream_id(T_DRAFT, salt), shape.vocab)
    toks = np.zeros(n, dtype=np.int32)
    used = {}
    j = 0
    for i in range(n):
        seen = used.setdefault(int(parent[i]), set())
        while int(pool[j]) in seen:
            j += 1
        toks[i] = pool[j]
        seen.add(int(pool[j]))
        j += 1
    return toks


def cancel_schedule(seed: int, n_runs: int, n_layers: int, fraction: float = 0.5):
    """For each run: -1 (never cancelled) or the layer before which the cancel flag is set."""
    r = uniform_int_host(2 * n_runs, seed, stream_id(T_CANCEL, 0), 1 << 30)
    order = sorted(range(n_runs), key=lambda i: (int(r[i]), i))
    chosen = set(order[: int(round(fraction * n_runs))])
    return [int(r[n_runs + i]) % n_layers if i in chosen else -1 for i in range(n_runs)]
