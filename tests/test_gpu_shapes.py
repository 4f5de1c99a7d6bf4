"""GPU parity on shapes chosen for their ragged edges: feature counts that are not multiples of
the 16-row / 32-column weight tiles' natural sizes, every supported head size, grouped-query
ratios 1, 3 and 8, an empty prefix, prefixes that end one cell before / after a 32-cell
boundary, one token and the largest micro-batch, runs at the far end of the window."""
import numpy as np
import pytest
import torch

import synth
import oracle
from oracle import from_synth
from synth import gpu_loader
import paper_2407_11798_amd as pi
from gpu_common import forward, verify, max_rel_rowwise, TieBudget

pytestmark = pytest.mark.gpu

ODD_SHAPES = {
    "odd_f32_gqa3": synth.ModelShape("odd_f32_gqa3", 1, 160, 6, 2, 32, 144, 48, dtype="f32"),
    "odd_bf16_hd64": synth.ModelShape("odd_bf16_hd64", 2, 160, 5, 5, 64, 176, 112, dtype="bf16"),
    "odd_bf16_hd128": synth.ModelShape("odd_bf16_hd128", 1, 384, 3, 3, 128, 1040, 2000, dtype="bf16"),
    "odd_f32_gqa8": synth.ModelShape("odd_f32_gqa8", 2, 512, 16, 2, 32, 1376, 1024, dtype="f32"),
    # 8-bit weight matrices (64-column tiles): feature counts that end inside a tile's first and second half
    "odd_w8_hd128": synth.ModelShape("odd_w8_hd128", 1, 384, 3, 3, 128, 1040, 2000, dtype="bf16", weight_format="fp8",
                                     weight_scale_exp2=-11),
    "odd_w8_gqa8": synth.ModelShape("odd_w8_gqa8", 2, 512, 16, 2, 32, 1376, 1024, dtype="bf16", weight_format="fp8",
                                    weight_scale_exp2=-9),
    # 4-bit weight matrices (128-column tiles, tile counts padded to a multiple of eight)
    "odd_w4_hd128": synth.ModelShape("odd_w4_hd128", 1, 384, 3, 3, 128, 1040, 2000, dtype="bf16", weight_format="fp4",
                                     weight_scale_exp2=-6),
    "odd_w4_gqa8": synth.ModelShape("odd_w4_gqa8", 2, 512, 16, 2, 32, 1376, 1024, dtype="bf16", weight_format="fp4",
                                    weight_scale_exp2=-5),
    # 4-bit weight matrices with a scale per 32 columns: rows that end in a half block (1040 = 32 * 32 + 16)
    "odd_w4b_hd128": synth.ModelShape("odd_w4b_hd128", 1, 384, 3, 3, 128, 1040, 2000, dtype="bf16", weight_format="fp4b"),
    "odd_w4b_gqa8": synth.ModelShape("odd_w4b_gqa8", 2, 512, 16, 2, 32, 1376, 1024, dtype="bf16", weight_format="fp4b"),
}


def _tol_ok(gpu, ref, dtype):
    if dtype == "f32":
        return float(np.max(np.abs(gpu - ref))) <= 1e-4
    return max_rel_rowwise(gpu, ref) <= 2e-2


@pytest.mark.parametrize("name", sorted(ODD_SHAPES))
def test_ragged_shapes_match_oracle(name):
    sh = ODD_SHAPES[name]
    seed, n_cells = 3, 160
    om = from_synth.model_from_seed(sh, seed, 0.1)
    gm = gpu_loader.load_model(sh, seed, 0.1)
    ties = TieBudget(1)
    for T in (0, 31, 33, 96):
        okv = from_synth.kv_synthetic(sh, seed, n_cells, T)
        gkv = pi.KVCache(gm, n_cells)
        if T > 0:
            gpu_loader.prefill_kv_synthetic(gkv, sh, seed, T)
        for trial, (n, offset) in enumerate([(1, 0), (5, 7), (16, 48)]):
            parent = synth.random_tree(2, 10 * T + trial, n)
            toks = synth.sibling_distinct_tokens(sh, 2, 10 * T + trial, parent)
            rd = synth.tree_run(parent, T, T, offset=offset)
            ref = oracle.stage_forward(om, okv.clone(), rd, 0, sh.n_layers, tokens=toks)["logits"]
            st, done, lg, _, grun = forward(gm, gkv, rd, toks)
            assert (st, done) == (pi.PI_OK, sh.n_layers), (name, T, n)
            assert np.all(np.isfinite(lg))
            assert _tol_ok(lg, ref, sh.dtype), (name, T, n)
            root_expected = int(toks[0])
            a, acc, bonus = oracle.verify_greedy(toks, parent, ref.astype(np.float32), root_expected)
            gacc, gres = verify(grun, toks, lg, sh.vocab, root_expected)
            if ties.decisive([oracle.top2_gap(ref[i]) for i in acc]):
                assert gres.cpu().tolist() == [a, bonus]
            pi.kv_rollback(gkv, grun.slots, n)
            assert len(gkv) == T
    gm.free()


# Contractions long enough that every wave has several tiles of one row block at the start of its
# range in every projection (32 to 88 tiles per row, one or two row blocks per workgroup).
PARK_SHAPES = {
    "park_bf16": synth.ModelShape("park_bf16", 2, 2048, 16, 4, 128, 2816, 1024, dtype="bf16"),
    "park_w8": synth.ModelShape("park_w8", 2, 2048, 16, 4, 128, 2816, 1024, dtype="bf16", weight_format="fp8",
                                weight_scale_exp2=-10),
    "park_w4": synth.ModelShape("park_w4", 2, 4096, 32, 8, 128, 5632, 1024, dtype="bf16", weight_format="fp4",
                                weight_scale_exp2=-6),
}


@pytest.mark.parametrize("name", sorted(PARK_SHAPES) + ["odd_bf16_hd64"])
def test_tiles_asked_for_ahead_of_a_phase_change_no_bit(name):
    """Weight tiles that a wave asks for ahead of a phase (into LDS, while it waits for the phase to
    begin) are the first tiles of its range and are consumed first, in the same order and on the same
    accumulators as when they come through the ring: logits and the run's K/V must not change by a
    bit whatever the number of such tiles (none, 2, 6, the built-in choice, more than LDS holds)."""
    sh = PARK_SHAPES.get(name) or ODD_SHAPES[name]
    seed, n_cells, T = 5, 160, 33
    gm = gpu_loader.load_model(sh, seed, 0.1)
    gkv = pi.KVCache(gm, n_cells)
    gpu_loader.prefill_kv_synthetic(gkv, sh, seed, T)
    for n in (1, 5, 16):
        parent = synth.random_tree(2, n, n)
        toks = synth.sibling_distinct_tokens(sh, 2, n, parent)
        rd = synth.tree_run(parent, T, T)
        first = None
        for cap in (1, 2, 6, 0, 64):
            gm.set_plan(7, cap)
            st, done, lg, _, grun = forward(gm, gkv, rd, toks)
            assert (st, done) == (pi.PI_OK, sh.n_layers), (n, cap)
            image = gkv.raw()  # the whole cache, the run's cells included
            pi.kv_rollback(gkv, grun.slots, n)
            if first is None:
                first = (lg, image)
                continue
            assert np.array_equal(lg, first[0]), (n, cap)
            assert np.array_equal(image, first[1]), (n, cap)
    gm.set_plan(7, 0)
    gm.free()


def test_a_contraction_shorter_than_the_smallest_ring_is_refused():
    """d_model = 96 is three 32-column tiles, fewer than the smallest ring of outstanding tiles:
    the forward refuses on the host (no launch), and the model is otherwise intact."""
    sh = synth.ModelShape("too_short", 1, 96, 3, 1, 32, 144, 48, dtype="f32")
    gm = gpu_loader.load_model(sh, 1, 0.1)
    gkv = pi.KVCache(gm, 96)
    rd = synth.linear_run(2, 0)
    run = gpu_loader.make_run(rd, np.array([1, 2], dtype=np.int32))
    logits = torch.full((2, sh.vocab), 3.0, device="cuda")
    with pytest.raises(pi.PiError) as err:
        pi.stage_forward(gm, gkv, run, 0, 1, logits_out=logits)
    assert err.value.status == pi.PI_E_SHAPE
    torch.cuda.synchronize()
    assert torch.all(logits == 3.0)
    gm.free()
