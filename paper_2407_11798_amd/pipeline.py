"""Continuous asynchronous speculation on one GPU: the Python face of pi_spec_*.

What the paper's head node does (Sections "Asynchronous Speculation", "Continuous Speculation",
"Pipelined KV Cache Multibuffering", "Early Inference Cancellation") is the library's own loop
(csrc/spec.hip, behind pi_spec_create / pi_spec_generate): verification runs are queued back to
back on one stream; while the oldest has not finished, further micro-batches of draft tokens are
issued, each a run with a sequence partition, a record and a cancel word of its own, each building
on the entries of the one before it; when a result arrives it is sampled (greedy), the accepted
entries join every sequence, and every queued run that the new tokens contradict is cancelled
through its cancel word, which the stage kernel polls at every layer boundary.  Several consecutive
runs can share one pass over the weights (`runs_per_pass` > 1).

This module marshals: it turns the caller's draft model -- any callable position -> (token,
confidence), and optionally position -> second choice or None, which makes runs small token trees
(Sections "Speculative Inference / Verification", "Continuous Speculation": a chain plus one
alternative leaf hanging at least two positions above the chain's end) -- into the C callbacks the
loop calls, and the statistics into a dict.
"""
from __future__ import annotations

import ctypes

import numpy as np
import torch

from . import binding as pi


class ContinuousSpeculation:
    """model/kv: the target and its cache, holding `prefix_len` canonical cells (positions
    0 .. prefix_len-1); first_token: the accepted token at position prefix_len whose entry
    is not in the cache yet; draft(pos) -> (token, confidence) for pos > prefix_len.
    depth: weight passes in flight; micro_batch: draft tokens per run (1..4); runs_per_pass:
    consecutive runs sharing one pass over the weights (1 = every run is a pass of its own);
    alternative(pos) -> token or None: the draft model's second choice for position pos; when
    given, runs become trees (chain + one alternative leaf) where there is room."""

    def __init__(self, model, kv, prefix_len: int, first_token: int, draft, depth: int = 3, micro_batch: int = 4,
                 base_cutoff: float = 0.3, recovery: float = 0.05, decay: float = 0.05, n_seq: int = 32,
                 runs_per_pass: int = 1, alternative=None):
        self.model, self.kv = model, kv
        self._error = None

        def draft_cb(_ctx, pos, token_out, conf_out):
            try:
                tok, conf = draft(int(pos))
                token_out[0] = int(tok)
                conf_out[0] = float(conf)
                return pi.PI_OK
            except BaseException as e:    # an exception must not cross the C frames: report it afterwards
                self._error = e
                return pi.PI_E_ARG

        def alt_cb(_ctx, pos, token_out):
            try:
                a = alternative(int(pos))
                if a is None:
                    return 0
                token_out[0] = int(a)
                return 1
            except BaseException as e:
                self._error = e
                return pi.PI_E_ARG

        # the callback objects must outlive the handle
        self._draft_cb = pi.PI_DRAFT_FN(draft_cb)
        self._alt_cb = pi.PI_ALTERNATIVE_FN(alt_cb) if alternative is not None else pi.PI_ALTERNATIVE_FN()
        cfg = pi.PiSpecConfig(prefix_len, int(first_token), depth, micro_batch, runs_per_pass, n_seq, base_cutoff,
                              recovery, decay, self._draft_cb, self._alt_cb, None)
        self.handle = ctypes.c_void_p()
        pi._check(pi.lib().pi_spec_create(model.handle, kv.handle, ctypes.byref(cfg), pi._stream_handle(None),
                                          ctypes.byref(self.handle)), "pi_spec_create")

    @property
    def stats(self):
        st = pi.PiSpecStats()
        pi._check(pi.lib().pi_spec_get_stats(self.handle, ctypes.byref(st)), "pi_spec_get_stats")
        return {name: int(getattr(st, name)) for name in pi.SPEC_STATS}

    def generate(self, n_tokens: int):
        """Run until n_tokens have been generated after first_token; returns them."""
        out = np.zeros(max(n_tokens, 1), dtype=np.int32)
        st = pi.lib().pi_spec_generate(self.handle, n_tokens, ctypes.c_void_p(out.ctypes.data))
        if self._error is not None:
            e, self._error = self._error, None
            raise e
        pi._check(st, "pi_spec_generate")
        return [int(t) for t in out[:n_tokens]]

    def settle(self):
        """Wait for everything in flight and fold the window into the dense prefix; returns
        (accepted tokens incl. the prompt's, length of the dense prefix)."""
        na, dense = ctypes.c_int32(), ctypes.c_int32()
        pi._check(pi.lib().pi_spec_settle(self.handle, ctypes.byref(na), ctypes.byref(dense)), "pi_spec_settle")
        return na.value, dense.value

    def read_cells(self):
        """The loop's cell metadata: (positions int32[n_cells], sequence sets uint32[n_cells])."""
        pos = np.empty(self.kv.n_cells, dtype=np.int32)
        seq = np.empty(self.kv.n_cells, dtype=np.uint32)
        pi._check(pi.lib().pi_spec_read_cells(self.handle, ctypes.c_void_p(pos.ctypes.data),
                                              ctypes.c_void_p(seq.ctypes.data)), "pi_spec_read_cells")
        return pos, seq

    def close(self):
        if self.handle:
            pi.lib().pi_spec_free(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
