"""ctypes binding of the C ABI in include/pipeinfer.h: argument marshalling only.

Every step of the hot path runs inside libpipeinfer_hip.so; this module converts Python
objects to pointers and sizes.  Device buffers are torch tensors (torch is used for device
memory and streams only).  There is no CPU fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_int32, c_int64, c_void_p, c_float, c_double, POINTER, byref

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# the library built in-tree, unless PIPEINFER_LIB names another build of it
LIB_PATH = os.environ.get("PIPEINFER_LIB") or os.path.join(_HERE, "libpipeinfer_hip.so")

PI_OK, PI_CANCELLED = 0, 1
PI_E_ARG, PI_E_SHAPE, PI_E_OOM, PI_E_SLOT_LIVE, PI_E_HIP, PI_E_STATE = -1, -2, -3, -4, -5, -6
PI_E_FULL, PI_E_BUSY = -7, -8
PI_MAX_BATCH, PI_WINDOW = 16, 64
PI_MAX_SEQ, PI_SEQ_CANONICAL, PI_POS_MAX = 32, 0, 0x7FFFFFFF
PI_RUN_SUPERFLUOUS, PI_RUN_INVALIDATED = 1, 2
PI_DTYPE_F32, PI_DTYPE_BF16, PI_DTYPE_FP8_E4M3, PI_DTYPE_FP4_E2M1, PI_DTYPE_FP4_E2M1_B32 = 0, 1, 2, 3, 4
PI_LOC_HOST, PI_LOC_DEVICE = 0, 1
(PI_T_EMBED, PI_T_ATTN_NORM, PI_T_WQ, PI_T_WK, PI_T_WV, PI_T_WO, PI_T_FFN_NORM, PI_T_WG, PI_T_WU,
 PI_T_WD, PI_T_FINAL_NORM, PI_T_LM_HEAD) = range(12)

EXPORTS = [
    "pi_model_load", "pi_model_set_tensor", "pi_model_free", "pi_model_weight_bytes", "pi_kv_alloc",
    "pi_kv_free", "pi_kv_set_cells", "pi_kv_get_cells", "pi_kv_set_len", "pi_kv_len", "pi_kv_raw",
    "pi_stage_forward", "pi_stage_forward_multi", "pi_verify_greedy", "pi_verify_greedy_noalloc", "pi_verify_greedy_chained", "pi_kv_rollback", "pi_strerror", "pi_debug_set_plan",
    "pi_debug_read_scratch", "pi_debug_read_trace", "pi_debug_wgtrace", "pi_debug_raise_cancel", "pi_debug_stream_probe",
    "pi_kvmeta_alloc", "pi_kvmeta_free", "pi_kvmeta_seq_acquire", "pi_kvmeta_seq_release", "pi_kvmeta_fill",
    "pi_kvmeta_place", "pi_kvmeta_seq_cp", "pi_kvmeta_seq_rm", "pi_kvmeta_accept", "pi_kvmeta_build_mask",
    "pi_kvmeta_compact", "pi_kvmeta_read",
    "pi_sched_create", "pi_sched_free", "pi_sched_begin_run", "pi_sched_accept_tokens", "pi_sched_complete_run",
    "pi_sched_want_speculation", "pi_sched_on_speculated", "pi_sched_on_speculation_stopped", "pi_sched_state",
    "pi_mapped_device_pointer",
    "pi_spec_create", "pi_spec_generate", "pi_spec_settle", "pi_spec_read_cells", "pi_spec_get_stats", "pi_spec_free",
]


class PiModelConfig(ctypes.Structure):
    _fields_ = [("n_layers", c_int32), ("d_model", c_int32), ("n_q_heads", c_int32),
                ("n_kv_heads", c_int32), ("head_dim", c_int32), ("ffn", c_int32), ("vocab", c_int32),
                ("rms_eps", c_float), ("rope_base", c_float), ("dtype", c_int32), ("max_pos", c_int32),
                ("weight_dtype", c_int32), ("weight_scale_exp2", c_int32)]


PI_DRAFT_FN = ctypes.CFUNCTYPE(c_int32, c_void_p, c_int32, POINTER(c_int32), POINTER(c_double))
PI_ALTERNATIVE_FN = ctypes.CFUNCTYPE(c_int32, c_void_p, c_int32, POINTER(c_int32))


class PiSpecConfig(ctypes.Structure):
    _fields_ = [("prefix_len", c_int32), ("first_token", c_int32), ("depth", c_int32), ("micro_batch", c_int32),
                ("runs_per_pass", c_int32), ("n_seq", c_int32), ("base_cutoff", c_double), ("recovery", c_double),
                ("decay", c_double), ("draft", PI_DRAFT_FN), ("alternative", PI_ALTERNATIVE_FN), ("ctx", c_void_p)]


SPEC_STATS = ["passes", "runs", "non_speculative", "speculative", "discarded", "cancelled", "layers_skipped",
              "tokens_speculated", "tokens_accepted_from_drafts", "compactions", "cutoff_stops", "tree_runs",
              "alternatives_accepted"]


class PiSpecStats(ctypes.Structure):
    _fields_ = [(name, c_int64) for name in SPEC_STATS]


class PiRunDesc(ctypes.Structure):
    _fields_ = [("n", c_int32), ("tokens", c_void_p), ("positions", c_void_p), ("slots", c_void_p),
                ("mask", c_void_p), ("prefix_len", c_int32), ("window_base", c_int32)]


class PiGroupDesc(ctypes.Structure):
    _fields_ = [("n_groups", c_int32), ("group_of_token", c_void_p), ("cancel_flags", c_void_p),
                ("group_status", c_void_p)]


class PiError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, strerror(status), status))


_lib = None


def lib():
    """Load the HIP library (fails loudly if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpipeinfer_hip.so is missing: run __graft_entry__.build() "
                               "(python -m paper_2407_11798_amd.build) first; there is no fallback path")
        # torch ships a HIP runtime of its own; it must be in the process first, so that this
        # library binds to the same one (device pointers and streams are shared with torch)
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        L.pi_model_load.argtypes = [POINTER(PiModelConfig), POINTER(c_void_p)]
        L.pi_model_set_tensor.argtypes = [c_void_p, c_int32, c_int32, c_void_p, c_int32, c_int32]
        L.pi_model_free.argtypes = [c_void_p]
        L.pi_model_weight_bytes.argtypes = [c_void_p, POINTER(c_int64), POINTER(c_int64)]
        L.pi_kv_alloc.argtypes = [c_void_p, c_int32, c_int32, POINTER(c_void_p)]
        L.pi_kv_free.argtypes = [c_void_p]
        L.pi_kv_set_cells.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_void_p, c_void_p, c_int32, c_int32]
        L.pi_kv_get_cells.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_void_p, c_void_p]
        L.pi_kv_set_len.argtypes = [c_void_p, c_int32]
        L.pi_kv_len.argtypes = [c_void_p, POINTER(c_int32)]
        L.pi_kv_raw.argtypes = [c_void_p, c_void_p, POINTER(c_int64)]
        L.pi_stage_forward_multi.argtypes = [c_void_p, c_void_p, POINTER(PiRunDesc), POINTER(PiGroupDesc), c_int32,
                                             c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
        L.pi_stage_forward.argtypes = [c_void_p, c_void_p, POINTER(PiRunDesc), c_int32, c_int32, c_void_p,
                                       c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
        L.pi_verify_greedy.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_int32, c_int32, c_void_p,
                                       c_void_p, c_void_p]
        L.pi_verify_greedy_noalloc.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_int32, c_int32, c_void_p,
                                               c_void_p, c_void_p]
        L.pi_verify_greedy_chained.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_int32, c_int32, c_void_p, c_int32,
                                               c_void_p, c_void_p, c_void_p, c_void_p]
        L.pi_kv_rollback.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p]
        L.pi_strerror.argtypes = [c_int32]
        L.pi_strerror.restype = ctypes.c_char_p
        L.pi_debug_set_plan.argtypes = [c_void_p, c_int32, c_int32]
        L.pi_debug_raise_cancel.argtypes = [c_void_p, c_int32, c_int32]
        L.pi_debug_stream_probe.argtypes = [c_int64, c_int32, POINTER(c_double)]
        L.pi_debug_read_trace.argtypes = [c_void_p, c_void_p, c_int32]
        L.pi_debug_read_scratch.argtypes = [c_void_p, c_int32, c_void_p, c_int64]
        c_uint32 = ctypes.c_uint32
        L.pi_debug_wgtrace.argtypes = [c_void_p, c_int32, c_void_p]
        L.pi_kvmeta_alloc.argtypes = [c_int32, c_int32, POINTER(c_void_p)]
        L.pi_kvmeta_free.argtypes = [c_void_p]
        L.pi_kvmeta_seq_acquire.argtypes = [c_void_p, POINTER(c_int32)]
        L.pi_kvmeta_seq_release.argtypes = [c_void_p, c_int32, c_void_p]
        L.pi_kvmeta_fill.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_uint32, c_void_p]
        L.pi_kvmeta_place.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_int32, c_void_p, c_void_p, c_void_p]
        L.pi_kvmeta_seq_cp.argtypes = [c_void_p, c_int32, c_uint32, c_int32, c_int32, c_void_p]
        L.pi_kvmeta_seq_rm.argtypes = [c_void_p, c_uint32, c_int32, c_int32, c_void_p]
        L.pi_kvmeta_accept.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
        L.pi_kvmeta_build_mask.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_int32, c_int32, c_void_p,
                                           c_void_p, c_void_p]
        L.pi_kvmeta_compact.argtypes = [c_void_p, c_void_p, c_int32, c_void_p, c_void_p]
        L.pi_kvmeta_read.argtypes = [c_void_p, c_void_p, c_void_p]
        L.pi_mapped_device_pointer.argtypes = [c_void_p, POINTER(c_void_p)]
        L.pi_sched_create.argtypes = [c_double, c_double, c_double, POINTER(c_void_p)]
        L.pi_sched_free.argtypes = [c_void_p]
        L.pi_sched_begin_run.argtypes = [c_void_p, c_int32, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                         c_int32, c_void_p, POINTER(c_int32)]
        L.pi_sched_accept_tokens.argtypes = [c_void_p, c_void_p, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_int32,
                                             POINTER(c_int32)]
        L.pi_sched_complete_run.argtypes = [c_void_p, c_int32, POINTER(c_int32)]
        L.pi_sched_want_speculation.argtypes = [c_void_p, c_double, POINTER(c_int32)]
        L.pi_sched_on_speculated.argtypes = [c_void_p]
        L.pi_sched_on_speculation_stopped.argtypes = [c_void_p, c_int32]
        L.pi_sched_state.argtypes = [c_void_p, POINTER(c_double), POINTER(c_int32), c_void_p, c_int32, POINTER(c_int32)]
        L.pi_spec_create.argtypes = [c_void_p, c_void_p, POINTER(PiSpecConfig), c_void_p, POINTER(c_void_p)]
        L.pi_spec_generate.argtypes = [c_void_p, c_int32, c_void_p]
        L.pi_spec_settle.argtypes = [c_void_p, POINTER(c_int32), POINTER(c_int32)]
        L.pi_spec_read_cells.argtypes = [c_void_p, c_void_p, c_void_p]
        L.pi_spec_get_stats.argtypes = [c_void_p, POINTER(PiSpecStats)]
        L.pi_spec_free.argtypes = [c_void_p]
        for name in EXPORTS:
            if name != "pi_strerror":
                getattr(L, name).restype = c_int32
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().pi_strerror(status).decode()


def _check(status, where):
    if status < 0:
        raise PiError(status, where)
    return status


def _ptr(t):
    """Device pointer of a torch tensor (or None)."""
    return None if t is None else c_void_p(t.data_ptr())


def _dtype_code(name: str) -> int:
    return {"f32": PI_DTYPE_F32, "bf16": PI_DTYPE_BF16}[name]


def _stream_handle(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return c_void_p(stream.cuda_stream)


class Model:
    """pi_model handle.  `shape` is any object with the decoder shape attributes."""

    def __init__(self, shape, max_pos: int = 4096):
        self.shape = shape
        self.max_pos = max_pos
        wf = getattr(shape, "weight_format", "native")
        fp8 = wf in ("fp8", "fp4")   # formats with one power-of-two scale per model
        cfg = PiModelConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                            shape.head_dim, shape.ffn, shape.vocab, shape.rms_eps, shape.rope_base,
                            _dtype_code(shape.dtype), max_pos,
                            {"fp8": PI_DTYPE_FP8_E4M3, "fp4": PI_DTYPE_FP4_E2M1, "fp4b": PI_DTYPE_FP4_E2M1_B32}.get(wf, _dtype_code(shape.dtype)),
                            getattr(shape, "weight_scale_exp2", 0) if fp8 else 0)
        h = c_void_p()
        _check(lib().pi_model_load(byref(cfg), byref(h)), "pi_model_load")
        self.handle = h

    def set_tensor(self, kind: int, layer: int, src, src_dtype=None):
        """src: numpy array (host; float32, uint16 bf16 bits or uint8 FP8 E4M3 bytes) or a torch
        device tensor (float32, bfloat16, int16/uint16 holding bf16 bits, or uint8 FP8 bytes)."""
        if isinstance(src, np.ndarray):
            src = np.ascontiguousarray(src)
            code = {np.dtype(np.float32): PI_DTYPE_F32, np.dtype(np.uint16): PI_DTYPE_BF16,
                    np.dtype(np.uint8): PI_DTYPE_FP8_E4M3}[src.dtype]
            code = code if src_dtype is None else src_dtype
            st = lib().pi_model_set_tensor(self.handle, kind, layer, c_void_p(src.ctypes.data), code, PI_LOC_HOST)
        else:
            import torch
            assert src.is_cuda and src.is_contiguous()
            code = (PI_DTYPE_F32 if src.dtype == torch.float32 else
                    PI_DTYPE_FP8_E4M3 if src.dtype == torch.uint8 else PI_DTYPE_BF16)
            code = code if src_dtype is None else src_dtype
            st = lib().pi_model_set_tensor(self.handle, kind, layer, _ptr(src), code, PI_LOC_DEVICE)
        _check(st, "pi_model_set_tensor")

    def weight_bytes(self):
        a, b = c_int64(), c_int64()
        _check(lib().pi_model_weight_bytes(self.handle, byref(a), byref(b)), "pi_model_weight_bytes")
        return a.value, b.value

    def set_plan(self, phase, s_k=0):
        _check(lib().pi_debug_set_plan(self.handle, phase, s_k), "pi_debug_set_plan")

    def raise_cancel(self, layer: int, phase: int = 3):
        _check(lib().pi_debug_raise_cancel(self.handle, layer, phase), "pi_debug_raise_cancel")

    def wgtrace(self, layer: int, read: bool = False, grid: int = 256):
        """Select the layer whose phases later runs record (-1: none); with read=True first return the
        last recording as [grid][5 phases][8] clock values."""
        buf = np.zeros(grid * 40, dtype=np.uint64) if read else None
        _check(lib().pi_debug_wgtrace(self.handle, layer, c_void_p(buf.ctypes.data) if read else None), "pi_debug_wgtrace")
        return None if buf is None else buf.reshape(grid, 5, 8)

    def read_trace(self, count: int):
        out = np.zeros(count, dtype=np.uint64)
        _check(lib().pi_debug_read_trace(self.handle, c_void_p(out.ctypes.data), count), "pi_debug_read_trace")
        return out

    def read_scratch(self, which: int, shape):
        out = np.empty(shape, dtype=np.float32)
        _check(lib().pi_debug_read_scratch(self.handle, which, c_void_p(out.ctypes.data), out.size),
               "pi_debug_read_scratch")
        return out

    def free(self):
        if self.handle:
            lib().pi_model_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class KVCache:
    def __init__(self, model: Model, n_cells: int, dtype: str | None = None):
        self.model = model
        self.dtype = dtype or model.shape.dtype
        self.n_cells = n_cells
        h = c_void_p()
        _check(lib().pi_kv_alloc(model.handle, n_cells, _dtype_code(self.dtype), byref(h)), "pi_kv_alloc")
        self.handle = h

    def set_cells(self, layer: int, cell_begin: int, k, v):
        if isinstance(k, np.ndarray):
            k, v = np.ascontiguousarray(k), np.ascontiguousarray(v)
            code = PI_DTYPE_F32 if k.dtype == np.float32 else PI_DTYPE_BF16
            st = lib().pi_kv_set_cells(self.handle, layer, cell_begin, k.shape[0], c_void_p(k.ctypes.data),
                                       c_void_p(v.ctypes.data), code, PI_LOC_HOST)
        else:
            import torch
            code = PI_DTYPE_F32 if k.dtype == torch.float32 else PI_DTYPE_BF16
            st = lib().pi_kv_set_cells(self.handle, layer, cell_begin, k.shape[0], _ptr(k), _ptr(v), code,
                                       PI_LOC_DEVICE)
        _check(st, "pi_kv_set_cells")

    def get_cells(self, layer: int, cell_begin: int, n: int):
        sh = self.model.shape
        k = np.empty((n, sh.n_kv_heads, sh.head_dim), dtype=np.float32)
        v = np.empty_like(k)
        _check(lib().pi_kv_get_cells(self.handle, layer, cell_begin, n, c_void_p(k.ctypes.data),
                                     c_void_p(v.ctypes.data)), "pi_kv_get_cells")
        return k, v

    def set_len(self, n: int):
        _check(lib().pi_kv_set_len(self.handle, n), "pi_kv_set_len")

    def __len__(self):
        out = c_int32()
        _check(lib().pi_kv_len(self.handle, byref(out)), "pi_kv_len")
        return out.value

    def raw(self) -> np.ndarray:
        nb = c_int64()
        _check(lib().pi_kv_raw(self.handle, None, byref(nb)), "pi_kv_raw")
        buf = np.empty(nb.value, dtype=np.uint8)
        _check(lib().pi_kv_raw(self.handle, c_void_p(buf.ctypes.data), byref(nb)), "pi_kv_raw")
        return buf

    def free(self):
        if self.handle:
            lib().pi_kv_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class Run:
    """Device-side copy of one run's batch description (tokens, positions, slots, mask)."""

    def __init__(self, tokens, positions, slots, mask, prefix_len: int, window_base: int, parent=None):
        import torch
        dev = "cuda"
        self.n = len(positions)
        self.tokens = None if tokens is None else torch.as_tensor(np.asarray(tokens, dtype=np.int32), device=dev)
        self.positions = torch.as_tensor(np.asarray(positions, dtype=np.int32), device=dev)
        self.slots = torch.as_tensor(np.asarray(slots, dtype=np.int32), device=dev)
        self.mask = torch.as_tensor(np.asarray(mask, dtype=np.uint64).view(np.int64), device=dev)
        self.parent = None if parent is None else torch.as_tensor(np.asarray(parent, dtype=np.int32), device=dev)
        self.prefix_len = int(prefix_len)
        self.window_base = int(window_base)

    @classmethod
    def from_device(cls, n: int, tokens, positions, slots, mask, prefix_len: int, window_base: int, parent=None):
        """A run whose arrays are already device tensors (int32 tokens/positions/slots/parent,
        int64 mask words), e.g. slots and masks produced by the cell-metadata kernels; the first
        n entries of each are used."""
        r = cls.__new__(cls)
        r.n, r.tokens, r.positions, r.slots, r.mask, r.parent = int(n), tokens, positions, slots, mask, parent
        r.prefix_len, r.window_base = int(prefix_len), int(window_base)
        return r

    def desc(self) -> PiRunDesc:
        return PiRunDesc(self.n, _ptr(self.tokens), _ptr(self.positions), _ptr(self.slots), _ptr(self.mask),
                         self.prefix_len, self.window_base)


def stage_forward(model: Model, kv: KVCache, run: Run, layer_begin: int, layer_end: int, hidden_in=None,
                  hidden_out=None, logits_out=None, cancel_flag=None, run_status=None, stream=None,
                  cancel_flag_ptr: int | None = None) -> int:
    """Enqueue pi_stage_forward.  cancel_flag: torch int32 device tensor (or pass a raw
    device-visible address with cancel_flag_ptr, e.g. mapped pinned host memory)."""
    d = run.desc()
    cf = c_void_p(cancel_flag_ptr) if cancel_flag_ptr is not None else _ptr(cancel_flag)
    st = lib().pi_stage_forward(model.handle, kv.handle, byref(d), layer_begin, layer_end, _ptr(hidden_in),
                                _ptr(hidden_out), _ptr(logits_out), cf, _ptr(run_status),
                                _stream_handle(stream))
    return _check(st, "pi_stage_forward")


def stage_forward_multi(model: Model, kv: KVCache, run: Run, group_of_token, layer_begin: int, layer_end: int,
                        hidden_in=None, hidden_out=None, logits_out=None, cancel_flags=None, group_status=None,
                        run_status=None, stream=None, cancel_flags_ptr: int | None = None) -> int:
    """Enqueue pi_stage_forward_multi: the run's tokens belong to several runs (group_of_token: one
    run index per token, host side); cancel_flags: torch int32 device tensor with one word per run
    (or a raw device-visible address), group_status: torch int32 device tensor [n_groups][2]."""
    d = run.desc()
    g = [int(v) for v in group_of_token]
    arr = (c_int32 * len(g))(*g)
    gd = PiGroupDesc()
    gd.n_groups = (max(g) + 1) if g else 0
    gd.group_of_token = ctypes.cast(arr, c_void_p)
    gd.cancel_flags = c_void_p(cancel_flags_ptr) if cancel_flags_ptr is not None else _ptr(cancel_flags)
    gd.group_status = _ptr(group_status)
    st = lib().pi_stage_forward_multi(model.handle, kv.handle, byref(d), byref(gd), layer_begin, layer_end,
                                      _ptr(hidden_in), _ptr(hidden_out), _ptr(logits_out), _ptr(run_status),
                                      _stream_handle(stream))
    return _check(st, "pi_stage_forward_multi")


def verify_greedy(draft, parent, n: int, logits, vocab: int, root_expected: int, accepted_nodes, result,
                  stream=None) -> int:
    st = lib().pi_verify_greedy(_ptr(draft), _ptr(parent), n, _ptr(logits), vocab, root_expected,
                                _ptr(accepted_nodes), _ptr(result), _stream_handle(stream))
    return _check(st, "pi_verify_greedy")


def verify_greedy_noalloc(draft, parent, n: int, logits, vocab: int, root_expected: int, accepted_nodes, result,
                          stream=None) -> int:
    """pi_verify_greedy for callers that cannot allocate (its scratch is a device array of the library)."""
    st = lib().pi_verify_greedy_noalloc(_ptr(draft), _ptr(parent), n, _ptr(logits), vocab, root_expected,
                                        _ptr(accepted_nodes), _ptr(result), _stream_handle(stream))
    return _check(st, "pi_verify_greedy_noalloc")


def verify_greedy_chained(draft, parent, n: int, logits, vocab: int, root_expected: int, prev_result, prev_n: int,
                          run_status, accepted_nodes, result, stream=None) -> int:
    st = lib().pi_verify_greedy_chained(_ptr(draft), _ptr(parent), n, _ptr(logits), vocab, root_expected,
                                        _ptr(prev_result), prev_n, _ptr(run_status), _ptr(accepted_nodes), _ptr(result),
                                        _stream_handle(stream))
    return _check(st, "pi_verify_greedy_chained")


def kv_rollback(kv: KVCache, slots, n: int, accepted_nodes=None, result=None, stream=None) -> int:
    st = lib().pi_kv_rollback(kv.handle, _ptr(slots), n, _ptr(accepted_nodes), _ptr(result),
                              _stream_handle(stream))
    return _check(st, "pi_kv_rollback")


def stream_probe(nbytes: int = 2 << 30, reps: int = 5) -> float:
    """GB/s a bare streaming read of the forward's launch shape reaches (pi_debug_stream_probe)."""
    g = c_double()
    _check(lib().pi_debug_stream_probe(nbytes, reps, byref(g)), "pi_debug_stream_probe")
    return g.value


def seq_bits(seqs) -> int:
    """Sequence identifiers -> the uint32 set the C ABI takes."""
    m = 0
    for q in seqs:
        m |= 1 << int(q)
    return m


class KVMeta:
    """pi_kvmeta handle: cell metadata (position, sequence set) on the device and the FIFO of
    free partition identifiers.  Device arguments are torch tensors: positions int32[n],
    tok_seq int32[n] holding the uint32 bit sets, slots int32[n], mask int64[n], status words
    int32."""

    def __init__(self, n_cells: int, n_seq: int):
        self.n_cells, self.n_seq = n_cells, n_seq
        h = c_void_p()
        _check(lib().pi_kvmeta_alloc(n_cells, n_seq, byref(h)), "pi_kvmeta_alloc")
        self.handle = h

    def acquire(self):
        """Partition identifier at the head of the queue, or None when all are in use."""
        out = c_int32()
        st = lib().pi_kvmeta_seq_acquire(self.handle, byref(out))
        if st == PI_E_FULL:
            return None
        _check(st, "pi_kvmeta_seq_acquire")
        return out.value

    def release(self, seq: int, stream=None):
        _check(lib().pi_kvmeta_seq_release(self.handle, seq, _stream_handle(stream)), "pi_kvmeta_seq_release")

    def fill(self, cell_begin: int, n: int, pos_begin: int, seq_mask: int, stream=None):
        _check(lib().pi_kvmeta_fill(self.handle, cell_begin, n, pos_begin, seq_mask, _stream_handle(stream)),
               "pi_kvmeta_fill")

    def place(self, n: int, positions, tok_seq, window_base: int, slots_out, status, stream=None):
        _check(lib().pi_kvmeta_place(self.handle, n, _ptr(positions), _ptr(tok_seq), window_base, _ptr(slots_out),
                                     _ptr(status), _stream_handle(stream)), "pi_kvmeta_place")

    def seq_cp(self, src: int, dst_mask: int, p0: int = 0, p1: int = PI_POS_MAX, stream=None):
        _check(lib().pi_kvmeta_seq_cp(self.handle, src, dst_mask, p0, p1, _stream_handle(stream)), "pi_kvmeta_seq_cp")

    def seq_rm(self, seq_mask: int, p0: int = 0, p1: int = PI_POS_MAX, stream=None):
        _check(lib().pi_kvmeta_seq_rm(self.handle, seq_mask, p0, p1, _stream_handle(stream)), "pi_kvmeta_seq_rm")

    def accept(self, n: int, positions, tok_seq, accepted_nodes, result, stream=None):
        _check(lib().pi_kvmeta_accept(self.handle, n, _ptr(positions), _ptr(tok_seq), _ptr(accepted_nodes),
                                      _ptr(result), _stream_handle(stream)), "pi_kvmeta_accept")

    def build_mask(self, n: int, positions, tok_seq, prefix_len: int, window_base: int, mask_out, n_unexpressed,
                   stream=None):
        _check(lib().pi_kvmeta_build_mask(self.handle, n, _ptr(positions), _ptr(tok_seq), prefix_len, window_base,
                                          _ptr(mask_out), _ptr(n_unexpressed), _stream_handle(stream)),
               "pi_kvmeta_build_mask")

    def compact(self, kv, prefix_len: int, result, stream=None):
        _check(lib().pi_kvmeta_compact(self.handle, None if kv is None else kv.handle, prefix_len, _ptr(result),
                                       _stream_handle(stream)), "pi_kvmeta_compact")

    def read(self):
        pos = np.empty(self.n_cells, dtype=np.int32)
        seq = np.empty(self.n_cells, dtype=np.uint32)
        _check(lib().pi_kvmeta_read(self.handle, c_void_p(pos.ctypes.data), c_void_p(seq.ctypes.data)),
               "pi_kvmeta_read")
        return pos, seq

    def free(self):
        if self.handle:
            lib().pi_kvmeta_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def mapped_device_pointer(pinned_tensor) -> int:
    """Device-visible address of a pinned (mapped) host tensor."""
    out = c_void_p()
    _check(lib().pi_mapped_device_pointer(c_void_p(pinned_tensor.data_ptr()), byref(out)), "pi_mapped_device_pointer")
    return out.value


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


class Scheduler:
    """pi_sched handle: the head node's run records, invalidation detection and reactive
    cutoff (host only).  cancel_word_ptr: host-visible address of a run's cancel word."""

    def __init__(self, base_cutoff: float, recovery: float, decay: float):
        h = c_void_p()
        _check(lib().pi_sched_create(base_cutoff, recovery, decay, byref(h)), "pi_sched_create")
        self.handle = h

    def begin_run(self, speculative, assumed, assumed_pos0, tokens, parent, positions, cancel_word_ptr=None) -> int:
        a, t, p, q = _i32(assumed), _i32(tokens), _i32(parent), _i32(positions)
        rid = c_int32()
        _check(lib().pi_sched_begin_run(self.handle, int(bool(speculative)), c_void_p(a.ctypes.data) if len(a) else None,
                                        len(a), assumed_pos0, c_void_p(t.ctypes.data), c_void_p(p.ctypes.data),
                                        c_void_p(q.ctypes.data), len(t),
                                        None if cancel_word_ptr is None else c_void_p(cancel_word_ptr), byref(rid)),
               "pi_sched_begin_run")
        return rid.value

    def accept_tokens(self, tokens, run_completed: bool = True, cap: int = 64):
        t = _i32(tokens)
        ids, reasons, sig = (np.zeros(cap, dtype=np.int32) for _ in range(3))
        found = c_int32()
        _check(lib().pi_sched_accept_tokens(self.handle, c_void_p(t.ctypes.data) if len(t) else None, len(t),
                                            int(bool(run_completed)), c_void_p(ids.ctypes.data),
                                            c_void_p(reasons.ctypes.data), c_void_p(sig.ctypes.data), cap, byref(found)),
               "pi_sched_accept_tokens")
        k = min(found.value, cap)
        return [(int(ids[i]), int(reasons[i]), bool(sig[i])) for i in range(k)]

    def complete_run(self, run_id: int) -> int:
        st = c_int32()
        _check(lib().pi_sched_complete_run(self.handle, run_id, byref(st)), "pi_sched_complete_run")
        return st.value

    def want_speculation(self, confidence: float) -> bool:
        yes = c_int32()
        _check(lib().pi_sched_want_speculation(self.handle, confidence, byref(yes)), "pi_sched_want_speculation")
        return bool(yes.value)

    def on_speculated(self):
        _check(lib().pi_sched_on_speculated(self.handle), "pi_sched_on_speculated")

    def on_speculation_stopped(self, logits_waiting: bool):
        _check(lib().pi_sched_on_speculation_stopped(self.handle, int(bool(logits_waiting))),
               "pi_sched_on_speculation_stopped")

    def state(self, cap: int = 64):
        cutoff, na, nr = ctypes.c_double(), c_int32(), c_int32()
        ids = np.zeros(cap, dtype=np.int32)
        _check(lib().pi_sched_state(self.handle, byref(cutoff), byref(na), c_void_p(ids.ctypes.data), cap, byref(nr)),
               "pi_sched_state")
        return cutoff.value, na.value, [int(v) for v in ids[:min(nr.value, cap)]]

    def free(self):
        if self.handle:
            lib().pi_sched_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass
