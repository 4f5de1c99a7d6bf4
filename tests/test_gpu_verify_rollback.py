"""GPU parity of greedy verification (argmax + tree walk) and KV commit/rollback: integer work,
compared bit-exactly with the CPU oracle on the same inputs."""
import numpy as np
import pytest
import torch

import synth
import oracle
from synth import gpu_loader
import paper_2407_11798_amd as pi

pytestmark = pytest.mark.gpu


def _gpu_verify(draft, parent, logits, root_expected):
    n, vocab = logits.shape
    d = torch.as_tensor(np.asarray(draft, dtype=np.int32), device="cuda")
    p = None if parent is None else torch.as_tensor(np.asarray(parent, dtype=np.int32), device="cuda")
    lg = torch.as_tensor(np.asarray(logits, dtype=np.float32), device="cuda")
    acc = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    res = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    pi.verify_greedy(d, p, n, lg, vocab, int(root_expected), acc, res)
    torch.cuda.synchronize()
    return acc.cpu().tolist(), res.cpu().tolist()


@pytest.mark.parametrize("vocab", [16, 1000, 32000, 50257])
def test_verify_matches_oracle_on_random_trees(vocab):
    rng = np.random.default_rng(vocab)
    for trial in range(40):
        n = int(rng.integers(1, 17))
        parent = synth.random_tree(trial, vocab % 97, n, max_children=3, max_depth=5)
        logits = rng.normal(size=(n, vocab)).astype(np.float32)
        # walk a planted path of random length so that non-trivial acceptance happens
        draft = rng.integers(0, vocab, size=n).astype(np.int32)
        root_expected = int(rng.integers(0, vocab))
        u, exp = -1, root_expected
        for _ in range(int(rng.integers(0, 6))):
            ch = [c for c in range(n) if parent[c] == u]
            if not ch:
                break
            c = ch[int(rng.integers(0, len(ch)))]
            draft[c] = exp
            u, exp = c, int(np.argmax(logits[c]))
        a, acc, bonus = oracle.verify_greedy(draft, parent, logits, root_expected)
        gacc, gres = _gpu_verify(draft, parent, logits, root_expected)
        assert gres == [a, bonus]
        assert gacc[:a] == acc and all(v == -1 for v in gacc[a:])


def test_chained_verification_matches_oracle():
    """Three runs queued back to back, each checked against the bonus token of the one before
    it, all on the device; every combination of: the earlier run accepted whole or not, this
    run's forward finished or cancelled."""
    rng = np.random.default_rng(5)
    vocab = 1000
    for trial in range(60):
        ns = [int(rng.integers(1, 6)) for _ in range(3)]
        logits = [rng.normal(size=(n, vocab)).astype(np.float32) for n in ns]
        drafts = [rng.integers(0, vocab, size=n).astype(np.int32) for n in ns]
        root_expected = int(rng.integers(0, vocab))
        # plant agreement: each token is right with probability 0.8, given that all before it were
        exp = root_expected
        for k in range(3):
            for i in range(ns[k]):
                if rng.random() < 0.8:
                    drafts[k][i] = exp
                exp = int(np.argmax(logits[k][i]))
        status = [[pi.PI_OK, 2] if rng.random() < 0.8 else [pi.PI_CANCELLED, 1] for _ in range(3)]
        # oracle
        want, prev = [], None
        for k in range(3):
            a, acc, bonus = oracle.verify_greedy_chained(drafts[k], None, logits[k], root_expected, prev,
                                                         ns[k - 1] if k else 0, status[k][0] == pi.PI_OK)
            want.append((a, acc, bonus))
            prev = (a, bonus)
        # device: results never leave the GPU between the three calls
        res = [torch.full((2,), -7, dtype=torch.int32, device="cuda") for _ in range(3)]
        acc = [torch.full((ns[k],), -7, dtype=torch.int32, device="cuda") for k in range(3)]
        for k in range(3):
            pi.verify_greedy_chained(torch.as_tensor(drafts[k], device="cuda"), None, ns[k],
                                     torch.as_tensor(logits[k], device="cuda"), vocab, root_expected,
                                     res[k - 1] if k else None, ns[k - 1] if k else 0,
                                     torch.as_tensor(np.asarray(status[k], dtype=np.int32), device="cuda"), acc[k], res[k])
        torch.cuda.synchronize()
        for k in range(3):
            a, path, bonus = want[k]
            assert res[k].cpu().tolist() == [a, bonus], (trial, k)
            assert acc[k].cpu().tolist() == path + [-1] * (ns[k] - a)
    assert pi.lib().pi_verify_greedy_chained(None, None, 1, None, 16, 0, None, 0, None, None, None, None) == pi.PI_E_ARG


def test_verify_linear_chain_without_parent_array_and_ties():
    vocab = 4096
    logits = np.zeros((4, vocab), dtype=np.float32)
    logits[0, [7, 9]] = 1.0          # tie: lowest id (7) is the target's choice
    logits[1, 100] = 2.0
    logits[2, 5] = 3.0
    logits[3, 4095] = 0.5
    draft = np.array([3, 7, 100, 6], dtype=np.int32)
    a, acc, bonus = oracle.verify_greedy(draft, None, logits, 3)
    assert (a, acc, bonus) == (3, [0, 1, 2], 5)
    gacc, gres = _gpu_verify(draft, None, logits, 3)
    assert gres == [3, 5] and gacc == [0, 1, 2, -1]
    # duplicate siblings: lowest node index wins
    gacc, gres = _gpu_verify(np.array([3, 3], dtype=np.int32), np.array([-1, -1]), logits[:2], 3)
    assert gres == [1, 7] and gacc == [0, -1]


def _filled_cache(shape_name, n_cells, seed=1):
    sh = synth.SHAPES[shape_name]
    m = gpu_loader.load_model(sh, 0)
    kv = pi.KVCache(m, n_cells)
    ok = oracle.OracleKV(sh, n_cells)
    rng = np.random.default_rng(seed)
    for l in range(sh.n_layers):
        k = rng.normal(size=(n_cells, sh.n_kv_heads, sh.head_dim)).astype(np.float32)
        v = rng.normal(size=(n_cells, sh.n_kv_heads, sh.head_dim)).astype(np.float32)
        kv.set_cells(l, 0, k, v)
        ok.set_cells(l, 0, k, v)
    return sh, m, kv, ok


def _cells_equal(sh, kv, ok):
    for l in range(sh.n_layers):
        k, v = kv.get_cells(l, 0, ok.n_cells)
        if not (np.array_equal(k.astype(np.float64), ok.K[l]) and np.array_equal(v.astype(np.float64), ok.V[l])):
            return False
    return True


@pytest.mark.parametrize("shape_name", ["tiny", "tiny_gqa"])
def test_rollback_commits_path_and_frees_the_rest(shape_name):
    sh, m, kv, ok = _filled_cache(shape_name, 64)
    kv.set_len(20)
    ok.kv_len = 20
    assert _cells_equal(sh, kv, ok)                       # set/get round trip incl. cache rounding
    cases = [
        (np.array([20, 21, 22, 23]), [0, 1, 2]),           # linear chain, slots already in place
        (np.array([30, 25, 41, 33, 28]), [1, 3, 4]),       # scattered slots, path in the middle
        (np.array([40, 41, 42]), []),                      # nothing accepted (cancelled run)
        (np.array([29, 28, 27, 26]), [3, 2, 0]),           # sources overlap destinations, reversed (kv_len is 26 by now)
    ]
    for slots, path in cases:
        n = len(slots)
        oracle.kv_rollback(ok, slots, path)
        s = torch.as_tensor(slots.astype(np.int32), device="cuda")
        acc = torch.full((n,), -1, dtype=torch.int32, device="cuda")
        acc[:len(path)] = torch.as_tensor(np.asarray(path, dtype=np.int32))
        res = torch.tensor([len(path), 0], dtype=torch.int32, device="cuda")
        if path:
            pi.kv_rollback(kv, s, n, acc, res)
        else:
            pi.kv_rollback(kv, s, n)                       # discard form
        assert len(kv) == ok.kv_len
        assert _cells_equal(sh, kv, ok)
    m.free()


def test_argument_errors_are_reported_not_launched():
    sh = synth.SHAPES["tiny"]
    m = gpu_loader.load_model(sh, 0)
    kv = pi.KVCache(m, 64)
    run = gpu_loader.make_run(synth.linear_run(2, 0), np.array([1, 2], dtype=np.int32))
    logits = torch.zeros((2, sh.vocab), device="cuda")
    with pytest.raises(pi.PiError) as e:
        pi.stage_forward(m, kv, run, 1, 1, logits_out=logits)          # empty layer range
    assert e.value.status == pi.PI_E_ARG
    with pytest.raises(pi.PiError) as e:
        pi.stage_forward(m, kv, run, 0, sh.n_layers)                    # no logits buffer
    assert e.value.status == pi.PI_E_ARG
    with pytest.raises(pi.PiError) as e:
        pi.KVCache(m, 50)                                               # not a multiple of 16
    assert e.value.status == pi.PI_E_SHAPE
    import dataclasses
    with pytest.raises(pi.PiError) as e:
        pi.Model(dataclasses.replace(sh, head_dim=48))
    assert e.value.status == pi.PI_E_SHAPE
    m2 = pi.Model(sh)                                                   # tensors never supplied
    kv2 = pi.KVCache(m2, 64)
    with pytest.raises(pi.PiError) as e:
        pi.stage_forward(m2, kv2, run, 0, sh.n_layers, logits_out=logits)
    assert e.value.status == pi.PI_E_STATE
    m.free()
    m2.free()
