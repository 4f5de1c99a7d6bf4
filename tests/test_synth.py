"""Pins for the seeded input generator (CPU only)."""
import ctypes

import numpy as np

import synth


def test_box_muller_matches_library_functions():
    # The generator's hand-written ln / cos / sin against numpy's, on the same uniforms.
    out = (ctypes.c_double * 4)()
    worst = 0.0
    for p in range(4000):
        synth.host_lib().synth_debug_pair_host(11, synth.stream_id(synth.T_WQ, 3), p, out)
        u1, u2, z0, z1 = list(out)
        assert 0.0 < u1 <= 1.0 and 0.0 <= u2 < 1.0
        r = np.sqrt(-2.0 * np.log(u1))
        worst = max(worst, abs(z0 - r * np.cos(2 * np.pi * u2)), abs(z1 - r * np.sin(2 * np.pi * u2)))
    assert worst < 1e-13


def test_moments_and_independence_of_streams():
    n = 4_000_000
    x = synth.normal_host(n, 0, synth.stream_id(synth.T_WG, 1), 0.02, "f32").astype(np.float64)
    assert abs(x.mean()) < 4 * 0.02 / np.sqrt(n)
    assert abs(x.std() - 0.02) < 4 * 0.02 / np.sqrt(2 * n)
    # fourth moment of a Gaussian: 3 sigma^4
    assert abs(np.mean(x ** 4) / 0.02 ** 4 - 3.0) < 0.02
    y = synth.normal_host(n, 0, synth.stream_id(synth.T_WG, 2), 0.02, "f32").astype(np.float64)
    assert abs(np.corrcoef(x, y)[0, 1]) < 4 / np.sqrt(n)
    # even/odd elements come from the cos/sin halves of one pair: uncorrelated
    assert abs(np.corrcoef(x[0::2], x[1::2])[0, 1]) < 4 / np.sqrt(n / 2)


def test_seed_and_prefix_stability():
    a = synth.normal_host(1001, 5, 77, 1.0, "f32")
    b = synth.normal_host(64, 5, 77, 1.0, "f32")
    assert np.array_equal(a[:64], b)          # counter-based: a prefix is a prefix
    c = synth.normal_host(64, 6, 77, 1.0, "f32")
    assert not np.array_equal(b, c)


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1.0 and 1.0078125 -> even (1.0)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -1.0 - 2.0 ** -8],
                 dtype=np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    assert back.tolist() == [1.0, 1.015625, 1.0078125, -1.0]
    # the generator's bf16 output equals rounding its own fp32 output
    f = synth.normal_host(4096, 3, 9, 0.02, "f32")
    h = synth.normal_host(4096, 3, 9, 0.02, "bf16")
    assert np.array_equal(h, synth.f32_to_bf16_bits(f))
    assert np.max(np.abs(synth.bf16_bits_to_f32(h) - f) / np.abs(f)) <= 2.0 ** -8


def test_uniform_tokens_in_range():
    t = synth.tokens_host(synth.SHAPES["llama7b"], 0, 100000)
    assert t.min() >= 0 and t.max() < 32000
    assert abs(t.mean() - 16000) < 200


def test_tree_structure():
    for salt in range(20):
        parent = synth.random_tree(0, salt, 4)
        run = synth.tree_run(parent, prefix_len=1024, window_base=1024, offset=4 * (salt % 8))
        depth = run["positions"] - 1024
        assert parent[0] == -1 and depth.max() <= 3
        for i in range(4):
            assert np.sum(parent == i) <= 3
            # mask = self + ancestors only
            bits = [c - 4 * (salt % 8) for c in range(64) if (int(run["mask"][i]) >> c) & 1]
            anc, p = [i], int(parent[i])
            while p >= 0:
                anc.append(p)
                p = int(parent[p])
            assert sorted(bits) == sorted(anc)
        toks = synth.sibling_distinct_tokens(synth.SHAPES["tiny"], 0, salt, parent)
        for p in set(parent.tolist()):
            sib = toks[parent == p]
            assert len(set(sib.tolist())) == len(sib)


def test_cancel_schedule_half():
    s = synth.cancel_schedule(0, 8, 32)
    assert sum(1 for v in s if v >= 0) == 4 and all(-1 <= v < 32 for v in s)


# ---- 8-bit weights: rounding to FP8 E4M3 and its decode table --------------------------------------

def test_e4m3_decode_table_matches_library_type_and_closed_forms():
    import torch
    from oracle import from_synth
    t = from_synth.E4M3
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    finite = ~np.isnan(ref)
    assert np.array_equal(np.isnan(t), ~finite) and np.array_equal(t[finite], ref[finite])
    assert np.isnan(t[0x7f]) and np.isnan(t[0xff]) and finite.sum() == 254
    assert t[0x7e] == 448.0 and t[0x08] == 2.0 ** -6 and t[0x01] == 2.0 ** -9 and t[0x38] == 1.0
    assert np.all(np.diff(t[:0x7f]) > 0) and np.array_equal(t[0x80:0xff], -t[:0x7f])
    # exact in float32, scale included
    assert np.array_equal(from_synth.dequantise_fp8(np.arange(0x7f, dtype=np.uint8), -11).astype(np.float64), t[:0x7f] / 2048)


def test_e4m3_rounding_is_nearest_even_and_saturates():
    import torch
    from oracle import from_synth
    t = from_synth.E4M3
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.normal(size=20000) * s for s in (1e-3, 0.02, 1.0, 40.0, 150.0)]).astype(np.float32)
    x = np.concatenate([x, np.array([0.0, -0.0, 2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -6, 447.9, 448.0, 464.0, 479.9, 1e6, -1e6],
                                    dtype=np.float32)])
    got = synth.f32_to_e4m3_host(x)
    # brute force: the nearest finite code; ties go to the even code (even mantissa); beyond 448: 448
    vals = t[:0x7f]
    ax = np.abs(x.astype(np.float64))
    d = np.abs(ax[:, None] - vals[None, :])
    best = d.min(axis=1)
    want = np.empty(len(x), dtype=np.int64)
    for i in range(len(x)):
        c = np.flatnonzero(d[i] == best[i])
        want[i] = c[0] if len(c) == 1 else (c[0] if c[0] % 2 == 0 else c[1])
    want = want | np.where(np.signbit(x), 0x80, 0)
    assert np.array_equal(got.astype(np.int64), want)
    # the library's own conversion agrees wherever it does not overflow
    inr = ax <= 448.0
    lib = torch.from_numpy(x[inr]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got[inr], lib)
    # ties, written out: 2^-10 lies between 0 and 2^-9 -> even code 0; 3*2^-10 between codes 1 and 2 -> 2
    assert synth.f32_to_e4m3_host(np.array([2.0 ** -10, 3 * 2.0 ** -10, 464.0, -1e6], dtype=np.float32)).tolist() == [0, 2, 0x7e, 0xfe]


def test_fp8_weight_stream_is_the_rounded_float_stream():
    from oracle import from_synth
    sid = synth.stream_id(synth.T_WQ, 3)
    f = synth.normal_host(5001, 7, sid, 0.02, "f32")
    q = synth.normal_host(5001, 7, sid, 0.02 * 2048, "fp8")
    assert np.array_equal(q, synth.f32_to_e4m3_host(f * np.float32(2048)))
    w = from_synth.dequantise_fp8(q, -11)
    assert np.max(np.abs(w - f) / np.maximum(np.abs(f), 2.0 ** -17)) <= 2.0 ** -4     # half a step of three mantissa bits


# ---- 4-bit weights: FP4 E2M1 ---------------------------------------------------------------------------

def test_e2m1_codes_rounding_and_packing():
    from oracle import from_synth
    t = from_synth.E2M1
    assert t[:8].tolist() == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0] and np.array_equal(t[8:], -t[:8])
    # value = (-1)^s * 2^(e-1) * (1 + m/2) for e > 0, m/2 for e = 0: the format's definition, code by code
    for c in range(16):
        s_, e, m = c >> 3, (c >> 1) & 3, c & 1
        v = (m / 2.0 if e == 0 else 2.0 ** (e - 1) * (1 + m / 2.0)) * (-1.0 if s_ else 1.0)
        assert t[c] == v and np.signbit(t[c]) == bool(s_)
    # nearest code, ties to the code with mantissa bit 0 (even code), saturation at 6: by brute force
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.normal(size=20000) * s for s in (0.3, 1.3, 4.0)] +
                       [np.array([0.0, -0.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 5.0001, 6.0, 7.0, 1e9, -0.25, -5.0, -1e9])]).astype(np.float32)
    got = synth.f32_to_e2m1_host(x)
    ax = np.abs(x.astype(np.float64))
    d = np.abs(ax[:, None] - t[None, :8])
    want = np.empty(len(x), dtype=np.int64)
    for i in range(len(x)):
        c = np.flatnonzero(d[i] == d[i].min())
        want[i] = c[0] if len(c) == 1 else (c[0] if c[0] % 2 == 0 else c[1])
    want |= np.where(np.signbit(x), 8, 0)
    assert np.array_equal(got.astype(np.int64), want)
    # the ties written out
    ties = synth.f32_to_e2m1_host(np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 100.0, -0.75], dtype=np.float32))
    assert ties.tolist() == [0, 2, 2, 4, 4, 6, 6, 7, 10]
    # packing: element 2p in the low nibble, 2p+1 in the high nibble; the stream is the rounded float stream
    sid = synth.stream_id(synth.T_WU, 1)
    f = synth.normal_host(4000, 9, sid, 0.02, "f32")
    q = synth.normal_host(4000, 9, sid, 0.02 * 64, "fp4")
    codes = synth.f32_to_e2m1_host(f * np.float32(64))
    assert q.shape == (2000,) and np.array_equal(q & 0xF, codes[0::2]) and np.array_equal(q >> 4, codes[1::2])
    w = from_synth.dequantise_fp4(q.reshape(40, 50), -6)
    assert w.shape == (40, 100) and np.array_equal(w.reshape(-1).astype(np.float64), t[codes] / 64)


# ---- 4-bit weights with one scale per 32 columns ---------------------------------------------------------

def test_block_scaled_fp4_scale_rule_rounding_and_layout():
    """Per block of 32 columns of a row: scale byte - 127 = floor(log2(largest magnitude)) - 2, so
    the largest element lands in [4, 8) before rounding; every nibble is the nearest E2M1 code of
    value / 2^e (checked against the plain rounding, itself pinned by brute force above); the
    decoded weight is within half a step of the value, or saturated at 6 * 2^e."""
    from oracle import from_synth
    rows, cols = 24, 688                      # 21 whole blocks and one of 16 columns per row
    sid = synth.stream_id(synth.T_WD, 1)
    buf = synth.normal_fp4b_host(rows, cols, 7, sid, 0.02)
    codes, scales = synth.split_fp4b(buf, rows, cols)
    assert codes.shape == (rows, cols // 2) and scales.shape == (rows, 22) and buf.size == rows * (cols // 2 + 22)
    f = synth.normal_host(rows * cols, 7, sid, 0.02, "f32").reshape(rows, cols).astype(np.float64)
    w = from_synth.dequantise_fp4_blocks(codes, scales).astype(np.float64)
    assert w.shape == (rows, cols)
    for r in range(rows):
        for b in range(22):
            blk = f[r, 32 * b:32 * b + 32]
            e = int(np.floor(np.log2(np.max(np.abs(blk))))) - 2
            assert scales[r, b] == e + 127
            assert 4.0 <= np.max(np.abs(blk)) / 2.0 ** e < 8.0
            want = synth.f32_to_e2m1_host((blk / 2.0 ** e).astype(np.float32))
            got = np.empty(len(blk), dtype=np.uint8)
            got[0::2] = codes[r, 16 * b:16 * b + len(blk) // 2] & 0xF
            got[1::2] = codes[r, 16 * b:16 * b + len(blk) // 2] >> 4
            assert np.array_equal(got, want)
            dec = w[r, 32 * b:32 * b + 32]
            assert np.array_equal(dec, from_synth.E2M1[got] * 2.0 ** e)
            # error: half the local step (0.25, 0.5 or 1 in units of 2^e), or saturation above 6
            err = np.abs(dec - blk) / 2.0 ** e
            a = np.abs(blk) / 2.0 ** e
            bound = np.where(a <= 2.0, 0.25, np.where(a <= 4.0, 0.5, np.where(a <= 6.0, 1.0, a - 6.0)))
            assert np.all(err <= bound + 1e-12)
    # the quantiser keeps what a 4-bit format can: relative error of the whole matrix
    assert np.linalg.norm(w - f) / np.linalg.norm(f) < 0.12
    # known bytes -> known values (scale 125 = 2^-2, codes 0x7 = 6, 0x9 = -0.5; scale 130 = 2^3 in the next block)
    c = np.zeros((1, 32), dtype=np.uint8)
    c[0, 0] = 0x97
    c[0, 16] = 0x21
    s_ = np.array([[125, 130]], dtype=np.uint8)
    d = from_synth.dequantise_fp4_blocks(c, s_)
    assert d[0, :2].tolist() == [1.5, -0.125] and d[0, 32:34].tolist() == [4.0, 8.0] and not d[0, 2:32].any()


def test_block_scaled_model_decodes_through_the_oracle_loader():
    from oracle import from_synth
    sh = synth.SHAPES["tiny_w4b"]
    om = from_synth.model_from_seed(sh, 0)
    wd = om.w("wd", 1)
    assert wd.shape == (sh.d_model, sh.ffn)
    f = synth.normal_host(sh.d_model * sh.ffn, 0, synth.stream_id(synth.T_WD, 1), 0.02, "f32").reshape(sh.d_model, sh.ffn)
    assert np.linalg.norm(wd - f) / np.linalg.norm(f) < 0.12
    assert om.w("embed").dtype == np.float64 and om.w("embed").shape == (sh.vocab, sh.d_model)
