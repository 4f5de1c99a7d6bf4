"""The C-ABI library loads and exports every function the header declares (no compute calls:
these tests run without a GPU), the binding's list matches the header, and argument checks that
need no device reject bad calls with the documented status codes."""
import ctypes
import os
import re

import pytest

import paper_2407_11798_amd as pi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pipeinfer.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)  # comments mention function names too
    return sorted(set(re.findall(r"\b(pi_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_boundary_calls():
    names = declared_functions()
    for required in ("pi_model_load", "pi_kv_alloc", "pi_stage_forward", "pi_verify_greedy", "pi_kv_rollback"):
        assert required in names


def test_library_exports_every_declared_function():
    lib = pi.lib()
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, "declared in include/pipeinfer.h but not exported: %s" % missing


def test_binding_lists_every_declared_function():
    assert sorted(pi.binding.EXPORTS) == declared_functions()


def test_status_strings():
    lib = pi.lib()
    lib.pi_strerror.restype = ctypes.c_char_p
    lib.pi_strerror.argtypes = [ctypes.c_int32]
    seen = set()
    for code in (0, 1, -1, -2, -3, -4, -5, -6, -7, -8):
        s = lib.pi_strerror(code)
        assert s and s != b"unknown status"
        seen.add(s)
    assert len(seen) == 10
    assert lib.pi_strerror(12345) == b"unknown status"


def test_null_and_shape_arguments_are_refused_without_touching_a_device():
    lib = pi.lib()
    out = ctypes.c_void_p()
    assert lib.pi_model_load(None, ctypes.byref(out)) == pi.binding.PI_E_ARG
    cfg = pi.binding.PiModelConfig(n_layers=1, d_model=48, n_q_heads=2, n_kv_heads=2, head_dim=24, ffn=64,
                                   vocab=64, rms_eps=1e-5, rope_base=10000.0, dtype=0, max_pos=16)
    assert lib.pi_model_load(ctypes.byref(cfg), ctypes.byref(out)) == pi.binding.PI_E_SHAPE  # head_dim 24
    assert out.value is None
    # 8-bit weight matrices go with a bf16 model only, and the scale exponent is bounded
    ok = dict(n_layers=1, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=256, vocab=64, rms_eps=1e-5,
              rope_base=10000.0, max_pos=16)
    for bad in (dict(dtype=0, weight_dtype=2), dict(dtype=1, weight_dtype=2, weight_scale_exp2=40),
                dict(dtype=1, weight_dtype=5), dict(dtype=0, weight_dtype=3), dict(dtype=0, weight_dtype=1),
                dict(dtype=0, weight_dtype=4), dict(dtype=1, weight_dtype=4, weight_scale_exp2=-6)):   # block scales: bf16 model only, no model-wide scale
        cfg2 = pi.binding.PiModelConfig(**ok, **bad)
        assert lib.pi_model_load(ctypes.byref(cfg2), ctypes.byref(out)) == pi.binding.PI_E_SHAPE, bad
    assert lib.pi_stage_forward(None, None, None, 0, 1, None, None, None, None, None, None) == pi.binding.PI_E_ARG
    assert lib.pi_verify_greedy(None, None, 1, None, 16, 0, None, None, None) == pi.binding.PI_E_ARG
    assert lib.pi_kv_rollback(None, None, 1, None, None, None) == pi.binding.PI_E_ARG
    # several runs per pass: the description of the runs is checked before anything else
    run = pi.binding.PiRunDesc(n=4)
    gd = pi.binding.PiGroupDesc()
    assert lib.pi_stage_forward_multi(None, None, ctypes.byref(run), None, 0, 1, None, None, None, None, None) == pi.binding.PI_E_ARG
    grp = (ctypes.c_int32 * 4)(0, 0, 2, 2)                      # run 1 has no token
    gd.n_groups, gd.group_of_token = 3, ctypes.cast(grp, ctypes.c_void_p)
    assert lib.pi_stage_forward_multi(None, None, ctypes.byref(run), ctypes.byref(gd), 0, 1, None, None, None, None, None) == pi.binding.PI_E_ARG
    gd.n_groups = 17
    assert lib.pi_stage_forward_multi(None, None, ctypes.byref(run), ctypes.byref(gd), 0, 1, None, None, None, None, None) == pi.binding.PI_E_SHAPE
    grp2 = (ctypes.c_int32 * 4)(0, 1, 1, 0)
    gd.n_groups, gd.group_of_token = 2, ctypes.cast(grp2, ctypes.c_void_p)
    assert lib.pi_stage_forward_multi(None, None, ctypes.byref(run), ctypes.byref(gd), 0, 1, None, None, None, None, None) == pi.binding.PI_E_ARG  # no model


def test_cell_metadata_calls_refuse_bad_arguments_without_touching_a_device():
    lib = pi.lib()
    B = pi.binding
    out = ctypes.c_void_p()
    assert lib.pi_kvmeta_alloc(64, 4, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_alloc(0, 4, ctypes.byref(out)) == B.PI_E_SHAPE
    assert lib.pi_kvmeta_alloc(64, 1, ctypes.byref(out)) == B.PI_E_SHAPE       # no partition beside sequence 0
    assert lib.pi_kvmeta_alloc(64, 33, ctypes.byref(out)) == B.PI_E_SHAPE
    assert out.value is None
    seq = ctypes.c_int32()
    assert lib.pi_kvmeta_seq_acquire(None, ctypes.byref(seq)) == B.PI_E_ARG
    assert lib.pi_kvmeta_seq_release(None, 1, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_fill(None, 0, 1, 0, 1, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_place(None, 1, None, None, 0, None, None, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_seq_cp(None, 0, 1, 0, 1, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_seq_rm(None, 1, 0, 1, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_accept(None, 1, None, None, None, None, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_build_mask(None, 1, None, None, 0, 0, None, None, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_compact(None, None, 0, None, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_read(None, None, None) == B.PI_E_ARG
    assert lib.pi_kvmeta_free(None) == B.PI_E_ARG


def test_speculation_loop_calls_refuse_bad_arguments_without_touching_a_device():
    lib = pi.lib()
    B = pi.binding
    out = ctypes.c_void_p()
    cfg = B.PiSpecConfig(0, 1, 3, 4, 1, 32, 0.3, 0.05, 0.05, B.PI_DRAFT_FN(), B.PI_ALTERNATIVE_FN(), None)
    assert lib.pi_spec_create(None, None, ctypes.byref(cfg), None, ctypes.byref(out)) == B.PI_E_ARG
    assert lib.pi_spec_create(None, None, None, None, None) == B.PI_E_ARG
    assert out.value is None
    assert lib.pi_spec_generate(None, 1, None) == B.PI_E_ARG
    assert lib.pi_spec_settle(None, None, None) == B.PI_E_ARG
    assert lib.pi_spec_read_cells(None, None, None) == B.PI_E_ARG
    assert lib.pi_spec_get_stats(None, None) == B.PI_E_ARG
    assert lib.pi_spec_free(None) == B.PI_E_ARG
