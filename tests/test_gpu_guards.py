"""What the device does with run descriptions it cannot accept, and with forwards of two models
issued side by side: refusals instead of out-of-bounds accesses, rollbacks that leave live cells
alone, and one forward at a time on the device."""
import numpy as np
import pytest
import torch

import synth
from synth import gpu_loader
import paper_2407_11798_amd as pi
from gpu_common import forward

pytestmark = pytest.mark.gpu


def _setup(shape_name="tiny_gqa", T=24, n_cells=96, max_pos=4096):
    sh = synth.SHAPES[shape_name]
    gm = gpu_loader.load_model(sh, 0, 0.1, max_pos=max_pos)
    gkv = pi.KVCache(gm, n_cells)
    gpu_loader.prefill_kv_synthetic(gkv, sh, 0, T)
    return sh, gm, gkv


@pytest.mark.parametrize("bad_slots", [[3, 25, 26], [24, -1, 26], [24, 25, 96], [24, 25, 4000000]])
def test_refused_run_followed_by_rollback_leaves_the_cache_untouched(bad_slots):
    """A run with a slot in a live canonical cell, a slot of -1 (what a failed placement hands
    out) or a slot past the cache is refused by the forward; the rollback queued right behind it
    -- as in a back-to-back queue, with no host look at the status in between -- must neither
    zero a live cell nor touch memory outside the cache, whatever the result words say."""
    sh, gm, gkv = _setup()
    T = 24
    snapshot = gkv.raw().copy()
    rd = synth.linear_run(3, T)
    rd = dict(rd, slots=np.asarray(bad_slots, dtype=np.int32))
    toks = np.array([5, 6, 7], dtype=np.int32)
    run = gpu_loader.make_run(rd, toks)
    logits = torch.full((3, sh.vocab), 7.0, device="cuda")
    status = torch.full((2,), -99, dtype=torch.int32, device="cuda")
    acc = torch.tensor([0, 1, 2], dtype=torch.int32, device="cuda")
    for claimed in (0, 3, 99, -5):   # result words a confused caller might pass along
        res = torch.tensor([claimed, 0], dtype=torch.int32, device="cuda")
        pi.stage_forward(gm, gkv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
        pi.kv_rollback(gkv, run.slots, 3, acc, res)
        torch.cuda.synchronize()
        assert status.cpu().tolist() == [pi.PI_E_SLOT_LIVE, 0]
        assert float(logits.min()) == 7.0 and float(logits.max()) == 7.0     # nothing was evaluated
        # no live cell was zeroed and nothing outside the cache was touched: the image is unchanged
        # (whatever was "committed" came from free, all-zero cells of the cache)
        assert np.array_equal(gkv.raw(), snapshot)
        grown = len(gkv) - T
        assert grown == 0 if claimed <= 0 else 0 <= grown <= 3
        gkv.set_len(T)
    # a proper run still works afterwards
    st, done, lg, _, grun = forward(gm, gkv, synth.linear_run(3, T), toks)
    assert (st, done) == (pi.PI_OK, sh.n_layers) and np.all(np.isfinite(lg))
    gkv.free()
    gm.free()


def test_rollback_ignores_accepted_entries_that_are_not_tokens_of_the_run():
    sh, gm, gkv = _setup()
    T = 24
    toks = np.array([5, 6, 7, 8], dtype=np.int32)
    st, done, lg, _, grun = forward(gm, gkv, synth.linear_run(4, T), toks)
    assert (st, done) == (pi.PI_OK, sh.n_layers)
    k_run = [gkv.get_cells(l, T, 4)[0] for l in range(sh.n_layers)]
    acc = torch.tensor([0, 1, 17, 2], dtype=torch.int32, device="cuda")      # entry 2 names no token of the run
    res = torch.tensor([4, 0], dtype=torch.int32, device="cuda")
    pi.kv_rollback(gkv, grun.slots, 4, acc, res)
    torch.cuda.synchronize()
    assert len(gkv) == T + 2                                                  # the path is cut before it
    for l in range(sh.n_layers):
        k, _ = gkv.get_cells(l, T, 4)
        assert np.array_equal(k[:2], k_run[l][:2]) and not k[2:].any()
    gkv.free()
    gm.free()


@pytest.mark.parametrize("positions", [[24, 25, 64], [24, -1, 26], [2 ** 30, 25, 26]])
def test_position_outside_the_rotary_table_is_refused(positions):
    sh, gm, gkv = _setup(max_pos=64)
    T = 24
    snapshot = gkv.raw().copy()
    rd = dict(synth.linear_run(3, T), positions=np.asarray(positions, dtype=np.int32))
    run = gpu_loader.make_run(rd, np.array([5, 6, 7], dtype=np.int32))
    logits = torch.full((3, sh.vocab), 7.0, device="cuda")
    status = torch.full((2,), -99, dtype=torch.int32, device="cuda")
    pi.stage_forward(gm, gkv, run, 0, sh.n_layers, logits_out=logits, run_status=status)
    pi.kv_rollback(gkv, run.slots, 3)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [pi.PI_E_ARG, 0]
    assert float(logits.min()) == 7.0 and np.array_equal(gkv.raw(), snapshot)
    # the last position the table has is fine
    rd = dict(synth.linear_run(3, T), positions=np.asarray([61, 62, 63], dtype=np.int32))
    st, done, lg, _, grun = forward(gm, gkv, rd, np.array([5, 6, 7], dtype=np.int32))
    assert (st, done) == (pi.PI_OK, sh.n_layers) and np.all(np.isfinite(lg))
    gkv.free()
    gm.free()


def test_forwards_of_two_models_on_two_streams_both_complete():
    """The paper's target and draft pipelines run side by side; on one GPU a forward is a
    persistent kernel that needs every compute unit, so the library orders forwards on the device.
    Two models, two streams, several forwards each, enqueued alternately with no host waits: every
    one completes with PI_OK and gives the logits it gives alone."""
    sh_a, sh_b = synth.SHAPES["tiny_gqa"], synth.SHAPES["tiny_bf16"]
    ma, mb = gpu_loader.load_model(sh_a, 0, 0.1), gpu_loader.load_model(sh_b, 1, 0.1)
    ka, kb = pi.KVCache(ma, 96), pi.KVCache(mb, 96)
    gpu_loader.prefill_kv_synthetic(ka, sh_a, 0, 24)
    gpu_loader.prefill_kv_synthetic(kb, sh_b, 1, 24)
    toks = np.array([5, 6, 7, 8], dtype=np.int32)
    ref = {}
    for name, m, kv, sh in (("a", ma, ka, sh_a), ("b", mb, kb, sh_b)):
        st, done, lg, _, grun = forward(m, kv, synth.linear_run(4, 24), toks)
        assert (st, done) == (pi.PI_OK, sh.n_layers)
        pi.kv_rollback(kv, grun.slots, 4)
        ref[name] = lg
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    run_a, run_b = gpu_loader.make_run(synth.linear_run(4, 24), toks), gpu_loader.make_run(synth.linear_run(4, 24), toks)
    reps = 6
    out_a = [torch.zeros((4, sh_a.vocab), device="cuda") for _ in range(reps)]
    out_b = [torch.zeros((4, sh_b.vocab), device="cuda") for _ in range(reps)]
    st_a = torch.full((reps, 2), -99, dtype=torch.int32, device="cuda")
    st_b = torch.full((reps, 2), -99, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    for r in range(reps):
        pi.stage_forward(ma, ka, run_a, 0, sh_a.n_layers, logits_out=out_a[r], run_status=st_a[r], stream=s1)
        pi.kv_rollback(ka, run_a.slots, 4, stream=s1)
        pi.stage_forward(mb, kb, run_b, 0, sh_b.n_layers, logits_out=out_b[r], run_status=st_b[r], stream=s2)
        pi.kv_rollback(kb, run_b.slots, 4, stream=s2)
    torch.cuda.synchronize()
    assert st_a.cpu().tolist() == [[pi.PI_OK, sh_a.n_layers]] * reps
    assert st_b.cpu().tolist() == [[pi.PI_OK, sh_b.n_layers]] * reps
    for r in range(reps):
        assert np.array_equal(out_a[r].cpu().numpy(), ref["a"]) and np.array_equal(out_b[r].cpu().numpy(), ref["b"])
    for h in (ka, kb, ma, mb):
        h.free()
