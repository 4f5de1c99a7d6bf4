#!/usr/bin/env python3
"""Writes the stored expected values under tests/golden/ by running the CPU oracle only.

Usage: python tests/golden/make_golden.py [case ...]   (cases: llama7b_linear, llama7b_w8_linear, llama7b_w4_linear, llama7b_runs,
tinyllama_decode, llama70b_layer, llama70b_w8_layer, llama70b_w4_layer, llama7b_w4b_linear, llama70b_w4b_layer,
llama7b_full, llama70b_full)
Every value comes from oracle/ on the seeded synthetic inputs of synth/; nothing here touches
the HIP library.  The JSON files are small: per logits row the argmax, the top-2 gap, the row's
max |logit| and the logits at a fixed sample of columns.  The *_full cases store whole logits
rows (every column, float32) in an .npz next to a JSON with the per-row records.
"""
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np

import synth
import oracle
from oracle import from_synth

HERE = os.path.dirname(os.path.abspath(__file__))
N_SAMPLE_COLS = 48


def sample_cols(vocab, seed):
    return sorted(set(int(c) for c in synth.uniform_int_host(N_SAMPLE_COLS, seed, synth.stream_id(synth.T_MISC, 77), vocab)))


def row_record(logits_row, cols):
    lr = np.asarray(logits_row, dtype=np.float64)
    return {"argmax": int(np.argmax(lr)), "gap": oracle.top2_gap(lr), "maxabs": float(np.max(np.abs(lr))),
            "sample": [float(lr[c]) for c in cols]}


def llama7b_linear():
    """Llama-7B-shaped bf16 target, 512 synthetic prefix cells, linear runs of 1, 4, 8 and 16 draft tokens."""
    sh = synth.SHAPES["llama7b"]
    seed, T = 0, 512
    om = from_synth.model_from_seed(sh, seed)
    base = from_synth.kv_synthetic(sh, seed, T + 64, T)
    cols = sample_cols(sh.vocab, seed)
    out = {"shape": sh.name, "seed": seed, "prefix": T, "cols": cols, "runs": {}}
    for n in (1, 4, 8, 16):
        t0 = time.time()
        run = synth.linear_run(n, T)
        toks = synth.tokens_host(sh, seed, n, synth.T_DRAFT, salt=n)
        lg = oracle.stage_forward(om, base.clone(), run, 0, sh.n_layers, tokens=toks)["logits"]
        out["runs"][str(n)] = {"tokens": [int(t) for t in toks], "rows": [row_record(lg[i], cols) for i in range(n)]}
        print("llama7b_linear n=%d done in %.0fs" % (n, time.time() - t0), flush=True)
    return out


def llama7b_w8_linear(shape_name="llama7b_w8"):
    """The Llama-7B shape with 8-bit (FP8 E4M3) or 4-bit (FP4 E2M1) weight matrices under one
    power-of-two scale, bf16 activations and cache, 512 synthetic prefix cells, linear runs of 1
    and 8 draft tokens."""
    sh = synth.SHAPES[shape_name]
    seed, T = 0, 512
    om = from_synth.model_from_seed(sh, seed)
    base = from_synth.kv_synthetic(sh, seed, T + 64, T)
    cols = sample_cols(sh.vocab, seed)
    out = {"shape": sh.name, "seed": seed, "prefix": T, "cols": cols, "runs": {}}
    for n in (1, 8):
        t0 = time.time()
        run = synth.linear_run(n, T)
        toks = synth.tokens_host(sh, seed, n, synth.T_DRAFT, salt=n)
        lg = oracle.stage_forward(om, base.clone(), run, 0, sh.n_layers, tokens=toks)["logits"]
        out["runs"][str(n)] = {"tokens": [int(t) for t in toks], "rows": [row_record(lg[i], cols) for i in range(n)]}
        print("%s_linear n=%d done in %.0fs" % (shape_name, n, time.time() - t0), flush=True)
    return out


def llama7b_w4_linear():
    return llama7b_w8_linear("llama7b_w4")


def llama7b_w4b_linear():
    """4-bit weight matrices with one power-of-two scale per 32 columns of a row."""
    return llama7b_w8_linear("llama7b_w4b")


def llama7b_runs():
    """Eight in-flight runs of 4-token trees over a shared 1024-cell prefix with a seeded cancel
    schedule (half of the runs are cancelled before a uniform-random layer).  The draft tokens
    along each tree's first root-to-leaf path are planted to agree with the oracle's own choices
    for a seeded number of steps, so accepted counts are not all zero."""
    sh = synth.SHAPES["llama7b"]
    seed, T, n_runs, n = 0, 1024, 8, 4
    om = from_synth.model_from_seed(sh, seed)
    base = from_synth.kv_synthetic(sh, seed, T + 64, T)
    cols = sample_cols(sh.vocab, seed)
    cancel = synth.cancel_schedule(seed, n_runs, sh.n_layers)
    root_expected = int(synth.tokens_host(sh, seed, 1, synth.T_MISC, salt=1)[0])
    plant = [int(v) % (n + 1) for v in synth.uniform_int_host(n_runs, seed, synth.stream_id(synth.T_MISC, 5), 1 << 20)]
    out = {"shape": sh.name, "seed": seed, "prefix": T, "cols": cols, "root_expected": root_expected,
           "cancel_before_layer": cancel, "runs": []}
    for r in range(n_runs):
        t0 = time.time()
        parent = synth.random_tree(seed, r, n)
        toks = synth.sibling_distinct_tokens(sh, seed, r, parent)
        rd = synth.tree_run(parent, T, T, offset=n * r)
        # first root-to-leaf path: follow the lowest-index child
        path, u = [], -1
        while True:
            ch = [c for c in range(n) if parent[c] == u]
            if not ch:
                break
            path.append(ch[0])
            u = ch[0]
        k = min(plant[r], len(path))
        lg = None
        for step in range(k + 1):
            lg = oracle.stage_forward(om, base.clone(), rd, 0, sh.n_layers, tokens=toks)["logits"]
            if step == k:
                break
            node = path[step]
            want = root_expected if step == 0 else int(np.argmax(lg[path[step - 1]]))
            if int(toks[node]) == want:
                continue
            toks = toks.copy()
            toks[node] = want
            # keep siblings distinct
            for c in range(n):
                if c != node and parent[c] == parent[node] and int(toks[c]) == want:
                    toks[c] = (want + 1) % sh.vocab
        a, acc, bonus = oracle.verify_greedy(toks, parent, lg.astype(np.float32), root_expected)
        out["runs"].append({"parent": [int(p) for p in parent], "tokens": [int(t) for t in toks],
                            "accepted": a, "accepted_nodes": acc, "bonus": bonus,
                            "rows": [row_record(lg[i], cols) for i in range(n)]})
        print("llama7b_runs run %d (planted %d, accepted %d) done in %.0fs" % (r, k, a, time.time() - t0), flush=True)
    return out


def tinyllama_decode():
    """TinyLlama-shaped draft model (grouped-query attention, head_dim 64), bf16: single-token decode
    steps at 128 and 2048 synthetic prefix cells."""
    sh = synth.SHAPES["tinyllama"]
    seed = 0
    om = from_synth.model_from_seed(sh, seed)
    cols = sample_cols(sh.vocab, seed)
    out = {"shape": sh.name, "seed": seed, "cols": cols, "runs": {}}
    for T in (128, 2048):
        t0 = time.time()
        base = from_synth.kv_synthetic(sh, seed, T + 64, T)
        run = synth.linear_run(1, T)
        toks = synth.tokens_host(sh, seed, 1, synth.T_DRAFT, salt=T)
        lg = oracle.stage_forward(om, base, run, 0, sh.n_layers, tokens=toks)["logits"]
        out["runs"][str(T)] = {"tokens": [int(t) for t in toks], "rows": [row_record(lg[0], cols)]}
        print("tinyllama_decode T=%d done in %.0fs" % (T, time.time() - t0), flush=True)
    return out


def llama70b_layer(shape_name="llama70b"):
    """One layer plus the LM head of the Llama-70B shape (d 8192, 64 query / 8 KV heads x 128,
    FFN 28672), bf16 (or 8-bit / 4-bit weight matrices), 2048 synthetic prefix cells: speculative
    batches of 1 and 16 tokens."""
    import dataclasses
    sh = dataclasses.replace(synth.SHAPES[shape_name], n_layers=1, name=shape_name + "_l1")
    seed, T = 0, 2048
    om = from_synth.model_from_seed(sh, seed)
    base = from_synth.kv_synthetic(sh, seed, T + 64, T)
    cols = sample_cols(sh.vocab, seed)
    out = {"shape": shape_name, "n_layers": 1, "seed": seed, "prefix": T, "cols": cols, "runs": {}}
    for n in (1, 16):
        t0 = time.time()
        run = synth.linear_run(n, T)
        toks = synth.tokens_host(sh, seed, n, synth.T_DRAFT, salt=n)
        lg = oracle.stage_forward(om, base.clone(), run, 0, 1, tokens=toks)["logits"]
        out["runs"][str(n)] = {"tokens": [int(t) for t in toks], "rows": [row_record(lg[i], cols) for i in range(n)]}
        print("%s_layer n=%d done in %.0fs" % (shape_name, n, time.time() - t0), flush=True)
    return out


def llama70b_w8_layer():
    return llama70b_layer("llama70b_w8")


def llama70b_w4_layer():
    return llama70b_layer("llama70b_w4")


def llama70b_w4b_layer():
    return llama70b_layer("llama70b_w4b")


def _stack_layer_by_layer(sh, seed, T, batches, keep_hidden_after=(), keep_cells_of=()):
    """The whole stack for several batch sizes in ONE pass over the layers: a layer's weights
    are generated once, every batch goes through that layer as a stage of its own ([l, l+1),
    hidden state handed on), then the weights are dropped -- a 140 GB model never exists in
    memory.  Splitting a run into stages does not change the oracle's result (pinned in
    tests/test_oracle_pins.py), so this is stage_forward over [0, L) for each batch."""
    store = {}

    def weights(name, layer):
        key = (name, layer)
        if key not in store:
            kind = from_synth._NAME_TO_KIND[name]
            store[key] = from_synth.dequantise(sh, kind, synth.weight_host(sh, seed, kind, layer, 0.0))
        return store[key]

    om = oracle.OracleModel(sh, weights)
    state = {}
    for n in batches:
        kv = oracle.OracleKV(sh, T + 64)
        kv.kv_len = T
        state[n] = {"kv": kv, "run": synth.linear_run(n, T), "toks": synth.tokens_host(sh, seed, n, synth.T_DRAFT, salt=n),
                    "hidden": None, "hidden_after": {}, "cells": {}}
    out_logits = {}
    for l in range(sh.n_layers):
        t0 = time.time()
        k, v = synth.kv_prefill_host(sh, seed, l, T)
        for n in batches:
            st = state[n]
            st["kv"].set_cells(l, 0, k, v)
            r = oracle.stage_forward(om, st["kv"], st["run"], l, l + 1, tokens=st["toks"], hidden_in=st["hidden"])
            if l + 1 == sh.n_layers:
                out_logits[n] = r["logits"]
            else:
                st["hidden"] = r["hidden"]
                if l + 1 in keep_hidden_after:
                    st["hidden_after"][l + 1] = r["hidden"].astype(np.float32)
            if l in keep_cells_of:
                slots = st["run"]["slots"]
                st["cells"][l] = (st["kv"].K[l, slots].astype(np.float32), st["kv"].V[l, slots].astype(np.float32))
            # the layer's prefix cells are not needed again: keep the cache small
            st["kv"].K[l] = 0.0
            st["kv"].V[l] = 0.0
        for key in [k_ for k_ in store if k_[1] == l and k_[0] not in ("embed", "final_norm", "lm_head")]:
            del store[key]
        print("%s layer %d done in %.0fs" % (sh.name, l, time.time() - t0), flush=True)
    return state, out_logits


def _full_case(shape_name, T, batches, keep_hidden_after=(), keep_cells_of=()):
    sh = synth.SHAPES[shape_name]
    seed = 0
    state, logits = _stack_layer_by_layer(sh, seed, T, batches, keep_hidden_after, keep_cells_of)
    meta = {"shape": sh.name, "seed": seed, "prefix": T, "runs": {}}
    arrays = {}
    for n in batches:
        lg = logits[n]
        meta["runs"][str(n)] = {"tokens": [int(t) for t in state[n]["toks"]],
                                "rows": [{"argmax": int(np.argmax(lg[i])), "gap": oracle.top2_gap(lg[i]),
                                          "maxabs": float(np.max(np.abs(lg[i])))} for i in range(n)]}
        arrays["logits_n%d" % n] = lg.astype(np.float32)
        for l1, h in state[n]["hidden_after"].items():
            arrays["hidden_n%d_after%d" % (n, l1)] = h
        for l, (kc, vc) in state[n]["cells"].items():
            arrays["k_n%d_layer%d" % (n, l)] = kc
            arrays["v_n%d_layer%d" % (n, l)] = vc
    np.savez(os.path.join(HERE, shape_name + "_full.npz"), **arrays)
    return meta


def llama7b_full():
    """Llama-7B shape, 512 prefix cells, linear runs of 1 and 8 tokens: every logits column."""
    return _full_case("llama7b", 512, (1, 8), keep_cells_of=(0, 31))


def llama70b_full():
    """Llama-70B shape at full depth (80 layers), 2048 prefix cells, linear runs of 1 and 16
    tokens: every logits column, the hidden state after 20 layers (one pipeline stage's share)
    and the run's own K/V cells in three layers."""
    return _full_case("llama70b", 2048, (1, 16), keep_hidden_after=(20,), keep_cells_of=(0, 19, 79))


CASES = {"llama7b_full": llama7b_full, "llama70b_full": llama70b_full,
         "llama7b_linear": llama7b_linear, "llama7b_w8_linear": llama7b_w8_linear, "llama7b_w4_linear": llama7b_w4_linear, "llama7b_runs": llama7b_runs, "tinyllama_decode": tinyllama_decode,
         "llama70b_layer": llama70b_layer, "llama70b_w8_layer": llama70b_w8_layer,
         "llama70b_w4_layer": llama70b_w4_layer, "llama7b_w4b_linear": llama7b_w4b_linear,
         "llama70b_w4b_layer": llama70b_w4b_layer}

if __name__ == "__main__":
    for name in (sys.argv[1:] or list(CASES)):
        data = CASES[name]()
        with open(os.path.join(HERE, name + ".json"), "w") as f:
            json.dump(data, f)
        print("wrote", name)
