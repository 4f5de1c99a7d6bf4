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
