"""Helpers for the GPU parity tests: run the HIP path through the public binding."""
import numpy as np
import torch

import synth
from synth import gpu_loader
import paper_2407_11798_amd as pi


def forward(model, kv, run_dict, tokens, layer_begin=0, layer_end=None, hidden_in=None, cancel_flag=None):
    """One pi_stage_forward; returns (status, layers_done, logits|None, hidden|None) as numpy."""
    sh = model.shape
    layer_end = sh.n_layers if layer_end is None else layer_end
    run = gpu_loader.make_run(run_dict, tokens)
    n = run.n
    logits = torch.full((n, sh.vocab), float("nan"), device="cuda") if layer_end == sh.n_layers else None
    hidden = torch.full((n, sh.d_model), float("nan"), device="cuda") if layer_end < sh.n_layers else None
    status = torch.full((2,), -99, dtype=torch.int32, device="cuda")
    hin = None if hidden_in is None else torch.as_tensor(np.asarray(hidden_in, dtype=np.float32), device="cuda")
    pi.stage_forward(model, kv, run, layer_begin, layer_end, hidden_in=hin, hidden_out=hidden,
                     logits_out=logits, cancel_flag=cancel_flag, run_status=status)
    torch.cuda.synchronize()
    st = status.cpu().numpy()
    return (int(st[0]), int(st[1]), None if logits is None else logits.cpu().numpy(),
            None if hidden is None else hidden.cpu().numpy(), run)


def verify(run, draft, logits_dev_or_np, vocab, root_expected):
    lg = torch.as_tensor(np.asarray(logits_dev_or_np, dtype=np.float32), device="cuda")
    d = torch.as_tensor(np.asarray(draft, dtype=np.int32), device="cuda")
    acc = torch.full((run.n,), -7, dtype=torch.int32, device="cuda")
    res = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    pi.verify_greedy(d, run.parent, run.n, lg, vocab, root_expected, acc, res)
    torch.cuda.synchronize()
    return acc, res


def max_rel_rowwise(gpu, ref):
    """max over rows of max|gpu - ref| / max|ref_row|."""
    ref = np.asarray(ref, dtype=np.float64)
    err = np.max(np.abs(np.asarray(gpu, dtype=np.float64) - ref), axis=-1)
    return float(np.max(err / np.max(np.abs(ref), axis=-1)))


class TieBudget:
    """Counts the comparisons that the top-2 gap rule exempts.  An argmax (and what is accepted
    through it) is only compared with the oracle's where the oracle's two largest logits of every
    row involved are at least 1e-3 apart; a test may use that exemption `limit` times and fails on
    the next one, so a gap that is wrong (or a tolerance that quietly swallows the comparisons)
    cannot go unnoticed."""
    GAP = 1e-3

    def __init__(self, limit):
        self.limit = limit
        self.used = 0
        self.checks = 0

    def decisive(self, gaps) -> bool:
        self.checks += 1
        if all(g >= self.GAP for g in gaps):
            return True
        self.used += 1
        assert self.used <= self.limit, "top-2 gap exemption used %d times in %d checks (limit %d)" % (
            self.used, self.checks, self.limit)
        return False
