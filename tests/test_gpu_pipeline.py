"""Continuous asynchronous speculation end to end on the GPU: whatever the draft quality, queue
depth, micro-batch size and cutoff settings, the generated tokens must be exactly those of
plain greedy decoding (the paper's Section "Model Accuracy"), here the CPU oracle's one token
at a time; and the machinery must really have been used (runs cancelled mid-queue, entries
accepted through the metadata, compaction)."""
import numpy as np
import pytest
import torch

import synth
import oracle
from oracle import from_synth
from synth import gpu_loader
import paper_2407_11798_amd as pi
from paper_2407_11798_amd.pipeline import ContinuousSpeculation

pytestmark = pytest.mark.gpu


def _oracle_greedy(sh, om, okv, T, first_token, n_tokens):
    """Plain decoding, one token per forward; returns tokens and each step's top-2 logit gap."""
    toks, gaps, t = [], [], int(first_token)
    for i in range(n_tokens):
        run = synth.linear_run(1, T + i)
        lg = oracle.stage_forward(om, okv, run, 0, sh.n_layers, tokens=np.array([t]))["logits"][0]
        oracle.kv_rollback(okv, run["slots"], [0])
        t = int(np.argmax(lg))
        toks.append(t)
        gaps.append(oracle.top2_gap(lg))
    return toks, gaps


@pytest.fixture(scope="module")
def tiny_truth():
    sh = synth.SHAPES["tiny"]
    T, N = 24, 72
    om = from_synth.model_from_seed(sh, 0, 0.1)
    okv = from_synth.kv_synthetic(sh, 3, T + N + 8, T)
    first = int(synth.tokens_host(sh, 9, 1, synth.T_MISC)[0])
    G, gaps = _oracle_greedy(sh, om, okv, T, first, N)
    safe = next((i for i, g in enumerate(gaps) if g < 1e-3), N)   # beyond a near-tie either choice is legitimate
    assert safe >= 40
    gm = gpu_loader.load_model(sh, 0, 0.1)
    yield sh, T, first, G, safe, gm
    gm.free()


def _settings(*rows):
    return [r if len(r) == 6 else r + (None,) for r in rows]


@pytest.mark.parametrize("alpha,depth,mb,cutoff,rpp,beta", _settings(
    (0.7, 3, 4, (0.3, 0.05, 0.05), 1),
    (0.3, 2, 2, (0.5, 0.1, 0.2), 1),
    (1.0, 4, 4, (0.0, 0.0, 0.0), 1),        # every draft right, never a cutoff stop
    (0.0, 3, 3, (0.2, 0.0, 0.1), 1),        # every draft wrong: one token per non-speculative run
    (0.8, 2, 4, (0.3, 0.02, 0.05), 1),      # the shortest queue: one run behind the non-speculative one
    (0.7, 2, 4, (0.1, 0.03, 0.05), 4),      # several runs share a pass over the weights
    (0.9, 1, 3, (0.0, 0.0, 0.0), 6),        # one pass in flight, up to six runs and sixteen tokens in it
    (0.3, 3, 1, (0.2, 0.05, 0.05), 3),      # one-token micro-batches
    (0.5, 3, 4, (0.1, 0.03, 0.05), 1, 0.8), # token trees: a chain plus the draft's second choice as a sibling leaf
    (0.6, 2, 3, (0.0, 0.0, 0.0), 4, 0.5),   # trees, several per weight pass
    (0.0, 2, 4, (0.0, 0.0, 0.0), 1, 1.0),   # the chain is always wrong at once and the second choice always right
))
def test_output_equals_plain_greedy_decoding(tiny_truth, alpha, depth, mb, cutoff, rpp, beta):
    sh, T, first, G, safe, gm = tiny_truth
    n_gen = min(safe, 64)
    gkv = pi.KVCache(gm, 176)
    gpu_loader.prefill_kv_synthetic(gkv, sh, 3, T)
    u = synth.uniform_int_host(2 * (len(G) + 64), 17, synth.stream_id(synth.T_MISC, int(alpha * 100) + depth + 10 * rpp),
                               1 << 20)

    def draft(pos):
        i = pos - (T + 1)
        g = G[i] if i < len(G) else 0
        right = u[2 * i] < alpha * (1 << 20)
        return (g if right else (g + 1 + int(u[2 * i]) % 7) % sh.vocab), float(u[2 * i + 1]) / (1 << 20)

    u2 = synth.uniform_int_host(len(G) + 64, 23, synth.stream_id(synth.T_MISC, 7), 1 << 20)

    def alternative(pos):
        """The draft's second choice: where its first choice is wrong it is the target's token with
        probability beta; otherwise some other token (a sibling that will be rejected)."""
        i = pos - (T + 1)
        g = G[i] if i < len(G) else 0
        first_right = u[2 * i] < alpha * (1 << 20)
        if not first_right and u2[i] < beta * (1 << 20):
            return g
        return (g + 9 + int(u2[i]) % 5) % sh.vocab

    cs = ContinuousSpeculation(gm, gkv, T, first, draft, depth=depth, micro_batch=mb, base_cutoff=cutoff[0],
                               recovery=cutoff[1], decay=cutoff[2], runs_per_pass=rpp,
                               alternative=alternative if beta is not None else None)
    out = cs.generate(n_gen)
    assert out == G[:n_gen], "first difference at %d" % next(i for i in range(n_gen) if out[i] != G[i])
    # the canonical entries are exactly the accepted tokens' (all but the last, which has no entry yet)
    n_acc, dense = cs.settle()
    st = cs.stats
    pos, seq = cs.read_cells()
    assert n_acc >= T + 1 + n_gen and dense == n_acc - 1
    assert pos[:n_acc - 1].tolist() == list(range(n_acc - 1)) and not (pos[n_acc - 1:] >= 0).any()
    assert len(gkv) == n_acc - 1
    assert st["runs"] == st["speculative"] + st["non_speculative"]
    if rpp > 1:
        assert st["passes"] < st["runs"]
    if alpha == 1.0:
        assert st["cancelled"] == 0 and st["tokens_accepted_from_drafts"] >= n_gen - st["non_speculative"] - 4
    if alpha == 0.0 and beta is None:
        assert st["tokens_accepted_from_drafts"] == 0 and st["non_speculative"] >= n_gen
    if 0.0 < alpha < 1.0:
        assert st["tokens_accepted_from_drafts"] > 0
    if alpha < 1.0:
        assert st["discarded"] > 0                                    # runs built on a rejected token were thrown away
    assert st["compactions"] >= 1
    if beta is None:
        assert st["tree_runs"] == 0
    else:
        assert st["tree_runs"] > 0 and st["alternatives_accepted"] > 0   # second choices did stand in for wrong first ones
    cs.close()
    print("alpha %.1f depth %d mb %d runs/pass %d: %s" % (alpha, depth, mb, rpp, st))
