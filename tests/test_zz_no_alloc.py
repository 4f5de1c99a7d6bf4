"""The verification entry point that allocates nothing (its scratch is a device array inside the
library) against the ordinary one: same accepted nodes, count and bonus token, bit for bit, on two
calls in a row, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import synth
import paper_2407_11798_amd as pi

pytestmark = pytest.mark.gpu


def _case(seed, n, vocab):
    rng = np.random.default_rng(seed)
    parent = synth.random_tree(seed, 3, n, max_children=3, max_depth=5)
    logits = rng.normal(size=(n, vocab)).astype(np.float32)
    draft = rng.integers(0, vocab, size=n).astype(np.int32)
    root_expected = int(rng.integers(0, vocab))
    u, exp = -1, root_expected                      # plant a path so that something is accepted
    for _ in range(4):
        ch = [c for c in range(n) if parent[c] == u]
        if not ch:
            break
        c = ch[int(rng.integers(0, len(ch)))]
        draft[c] = exp
        u, exp = c, int(np.argmax(logits[c]))
    return draft, parent, logits, root_expected


def _run(fn, draft, parent, logits, root_expected):
    n, vocab = logits.shape
    d = torch.as_tensor(draft, device="cuda")
    p = torch.as_tensor(np.asarray(parent, dtype=np.int32), device="cuda")
    lg = torch.as_tensor(logits, device="cuda")
    acc = torch.full((n,), -7, dtype=torch.int32, device="cuda")
    res = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    st = fn(pi.binding._ptr(d), pi.binding._ptr(p), n, pi.binding._ptr(lg), vocab, int(root_expected),
            pi.binding._ptr(acc), pi.binding._ptr(res), pi.binding._stream_handle(None))
    assert st == pi.PI_OK
    torch.cuda.synchronize()
    return acc.cpu().tolist(), res.cpu().tolist()


def test_no_alloc_verification_equals_the_ordinary_one():
    L = pi.lib()                                       # straight through the C ABI
    big = _case(1, 16, 32000)
    small = _case(2, 3, 1000)
    want_big = _run(L.pi_verify_greedy, *big)
    want_small = _run(L.pi_verify_greedy, *small)
    assert want_big[1][0] >= 1                         # the planted path was found
    torch.cuda.synchronize()
    got_big = _run(L.pi_verify_greedy_noalloc, *big)
    got_small = _run(L.pi_verify_greedy_noalloc, *small)      # right behind it, fewer rows, shorter rows
    assert got_big == want_big and got_small == want_small
    # back to back on the stream with no host wait in between, then once more the large one
    n, vocab = big[2].shape
    outs = []
    for draft, parent, logits, root in (big, small, big):
        nn, vv = logits.shape
        d = torch.as_tensor(draft, device="cuda")
        p = torch.as_tensor(np.asarray(parent, dtype=np.int32), device="cuda")
        lg = torch.as_tensor(logits, device="cuda")
        acc = torch.full((nn,), -7, dtype=torch.int32, device="cuda")
        res = torch.full((2,), -7, dtype=torch.int32, device="cuda")
        outs.append((d, p, lg, acc, res, nn, vv, root))
    torch.cuda.synchronize()
    for d, p, lg, acc, res, nn, vv, root in outs:
        assert L.pi_verify_greedy_noalloc(pi.binding._ptr(d), pi.binding._ptr(p), nn, pi.binding._ptr(lg), vv, int(root),
                                          pi.binding._ptr(acc), pi.binding._ptr(res), pi.binding._stream_handle(None)) == pi.PI_OK
    torch.cuda.synchronize()
    for (d, p, lg, acc, res, nn, vv, root), want in zip(outs, (want_big, want_small, want_big)):
        assert (acc.cpu().tolist(), res.cpu().tolist()) == want


def test_no_alloc_verification_refuses_more_rows_than_its_scratch_holds():
    L = pi.lib()
    draft, parent, logits, root = _case(3, 16, 64)
    d = torch.as_tensor(np.concatenate([draft, draft]), device="cuda")
    lg = torch.as_tensor(np.concatenate([logits, logits]), device="cuda")
    acc = torch.full((32,), -7, dtype=torch.int32, device="cuda")
    res = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    st = L.pi_verify_greedy_noalloc(pi.binding._ptr(d), None, pi.PI_MAX_BATCH + 1, pi.binding._ptr(lg), 64, root,
                                    pi.binding._ptr(acc), pi.binding._ptr(res), pi.binding._stream_handle(None))
    assert st == pi.PI_E_SHAPE
    torch.cuda.synchronize()
    assert acc.cpu().tolist() == [-7] * 32 and res.cpu().tolist() == [-7, -7]      # nothing was launched
