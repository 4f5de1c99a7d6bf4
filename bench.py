#!/usr/bin/env python3
"""Benchmark of the speculative-verification hot path on one MI355X.

A step = one verification run end to end: pi_stage_forward over all layers + LM head on a
micro-batch of n speculated tokens, pi_verify_greedy, pi_kv_rollback.  Workload: the
Llama-7B-shaped bf16 target with 512 prefilled KV positions (synthetic, seeded), speculative
batches of 1, 4 and 8 tokens with a linear causal mask and uniform-random draft tokens.
Prints ONE JSON line; `value` is verified tokens/s at the largest batch (n = 8), the other
batch sizes are listed under "per_batch".
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per stage_kernel launch measured with rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated
# against a device copy (profiles/stage_kernel_*.md give the commands).  Keyed by (shape, prefix, n).
# These are typed in from those runs, not read at run time: re-take them when the kernel changes.
MEASURED_TRAFFIC_BYTES = {("llama7b", 512, 8): 14.200e9, ("llama7b_w8", 512, 8): 7.397e9,
                          ("llama7b_w4", 512, 8): 4.068e9, ("llama7b_w4b", 512, 8): 4.276e9,
                          ("llama70b", 2048, 8): 141.915e9}


def algorithmic_bytes(shape, layer_bytes, lm_bytes, prefix_len, n):
    """Bytes one forward must move: every weight once, the n embedding rows, every visible
    KV cell once (the prefix; the n new cells are written and read once more)."""
    es = shape.bytes_per_weight
    kv = shape.n_layers * (prefix_len + n) * 2 * shape.n_kv_heads * shape.head_dim * es
    return shape.n_layers * layer_bytes + lm_bytes + n * shape.d_model * es + kv


def cpu_baseline(shape, prefix_len, n, seed, other_ns=()):
    """The CPU oracle timed on a bounded sample: a 2-layer and a 10-layer model of the same
    layer shape (KV prefix included), extrapolated linearly to the full depth; `n` is the batch size
    the headline figure is quoted on, `other_ns` are timed on the same two models."""
    import dataclasses
    import numpy as np
    import synth
    import oracle
    from oracle import from_synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    ns = [n] + [m for m in other_ns if m != n]
    times = {m: {} for m in ns}
    lo, hi = (2, 10) if shape.n_layers >= 10 else (1, shape.n_layers)
    for nl in (lo, hi):
        sh = dataclasses.replace(shape, n_layers=nl, name="%s_l%d" % (shape.name, nl))
        om = from_synth.model_from_seed(sh, seed)
        for name in ("embed", "final_norm", "lm_head"):
            om.weights(name, 0)
        for l in range(nl):
            for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "wg", "wu", "wd"):
                om.weights(name, l)          # generation is not part of the timed region
        for m in ns:
            okv = from_synth.kv_synthetic(sh, seed, prefix_len + 64, prefix_len)
            run = synth.linear_run(m, prefix_len)
            toks = synth.tokens_host(sh, seed, m, synth.T_DRAFT)
            t0 = time.perf_counter()
            out = oracle.stage_forward(om, okv, run, 0, nl, tokens=toks)
            oracle.verify_greedy(toks, run["parent"], out["logits"].astype(np.float32), int(toks[0]))
            times[m][nl] = time.perf_counter() - t0

    def full_forward(m):
        t = times[m]
        per_layer = (t[hi] - t[lo]) / float(hi - lo) if hi > lo else t[lo] / lo
        return t[lo] + per_layer * (shape.n_layers - lo)

    full = full_forward(n)
    return {"value": n / full, "unit": "verified tokens/s", "cores": cores, "kind": "oracle",
            "per_batch": {str(m): m / full_forward(m) for m in ns},
            "sample": "n=%d, T=%d: timed %d-layer (%.2fs) and %d-layer (%.2fs) models of the same layer shape, "
                      "extrapolated to %d layers (%.1fs per forward); per_batch: the same two models at n = %s"
                      % (n, prefix_len, lo, times[n][lo], hi, times[n][hi], shape.n_layers, full,
                         ", ".join(str(m) for m in ns))}


def time_forward(pi, torch, model, kv, run, n, layer_begin, layer_end, steps, warmup, shape):
    """Mean HIP-event time (ms) of one pi_stage_forward over [layer_begin, layer_end); the run's cells are
    discarded after every forward (outside the timed region)."""
    last = layer_end == shape.n_layers
    logits = torch.empty((n, shape.vocab), device="cuda") if last else None
    hidden = torch.empty((n, shape.d_model), device="cuda") if not last else None
    hin = torch.zeros((n, shape.d_model), device="cuda") if layer_begin > 0 else None
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for k in range(warmup + steps):
        e = evs[k - warmup] if k >= warmup else None
        if e:
            e[0].record()
        pi.stage_forward(model, kv, run, layer_begin, layer_end, hidden_in=hin, hidden_out=hidden, logits_out=logits,
                         run_status=status)
        if e:
            e[1].record()
        pi.kv_rollback(kv, run.slots, n)
    torch.cuda.synchronize()
    assert status.cpu().tolist() == [0, layer_end], status
    return sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps


def shape_leg(pi, torch, synth, gpu_loader, shape_name, prefixes, batches, seed, steps, warmup, slice_layers=0):
    """Forward-only timing of another model shape: per (prefix, n) the forward time, the algorithmic
    bytes and the fraction of the HBM peak; optionally also the first `slice_layers` layers alone
    (one pipeline stage's share)."""
    shape = synth.SHAPES[shape_name]
    need = shape.n_layers * shape.layer_params * shape.bytes_per_weight * 1.08 + 4e9
    free, _total = torch.cuda.mem_get_info()
    if free < need:
        return {"skipped": "needs %.0f GB of device memory, %.0f GB free" % (need / 1e9, free / 1e9)}
    model = gpu_loader.load_model(shape, seed)
    layer_bytes, lm_bytes = model.weight_bytes()
    leg = {"shape": shape.name, "layers": shape.n_layers, "weights": shape.dtype, "runs": []}
    try:
        for T in prefixes:
            kv = pi.KVCache(model, ((T + 64 + 15) // 16) * 16)
            gpu_loader.prefill_kv_synthetic(kv, shape, seed, T)
            for n in batches:
                run = gpu_loader.make_run(synth.linear_run(n, T), synth.tokens_host(shape, seed, n, synth.T_DRAFT, salt=n))
                ms = time_forward(pi, torch, model, kv, run, n, 0, shape.n_layers, steps, warmup, shape)
                ab = algorithmic_bytes(shape, layer_bytes, lm_bytes, T, n)
                rec = {"prefix": T, "n": n, "forward_ms": ms, "verified_tokens_per_s_forward_only": n / (ms * 1e-3),
                       "per_layer_us": ms * 1e3 / (shape.n_layers + lm_bytes / layer_bytes),
                       "algorithmic_GB": ab / 1e9, "achieved_GBps": ab / 1e9 / (ms * 1e-3),
                       "frac_of_peak": ab / 1e9 / (ms * 1e-3) / HBM_PEAK_GBS}
                if slice_layers:
                    sms = time_forward(pi, torch, model, kv, run, n, 0, slice_layers, steps, warmup, shape)
                    es = shape.bytes_per_weight
                    sb = (slice_layers * layer_bytes + n * shape.d_model * es
                          + slice_layers * (T + n) * 2 * shape.n_kv_heads * shape.head_dim * es)
                    rec["slice"] = {"layers": slice_layers, "forward_ms": sms, "algorithmic_GB": sb / 1e9,
                                    "achieved_GBps": sb / 1e9 / (sms * 1e-3), "frac_of_peak": sb / 1e9 / (sms * 1e-3) / HBM_PEAK_GBS}
                leg["runs"].append(rec)
            kv.free()
    finally:
        model.free()
    return leg


def cancellation_on_device_clock(pi, torch, np, model, kv, run, n, shape, layer_end, layers):
    """Early Inference Cancellation timed on the device's own clock: a workgroup in the middle of
    the grid raises the run's cancel word when it enters the gate/up phase of a chosen layer and
    stamps the 100 MHz clock; workgroup 0 stamps every barrier it passes.  The run must stop at the
    boundary that ends that layer (one layer at most after the signal)."""
    cap = 5 * shape.n_layers + 8
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    last = layer_end == shape.n_layers
    logits = torch.empty((n, shape.vocab), device="cuda") if last else None
    hidden = torch.empty((n, shape.d_model), device="cuda") if not last else None
    model.set_plan(5, 1)
    trials = []
    try:
        for layer in layers:
            flag.zero_()
            model.raise_cancel(layer, 3)
            pi.stage_forward(model, kv, run, 0, layer_end, hidden_out=hidden, logits_out=logits, cancel_flag=flag,
                             run_status=status)
            pi.kv_rollback(kv, run.slots, n)
            torch.cuda.synchronize()
            st = status.cpu().tolist()
            tr = model.read_trace(cap).astype(np.int64)
            rec = {"raised_in_layer": layer, "status": st[0], "layers_done": st[1]}
            if st[0] == 1 and st[1] >= 1:
                t_store, t_stop = int(tr[cap - 1]), int(tr[3 + 2 * (st[1] - 1)])   # boundary that ended layer layers_done - 1
                t_layer0 = int(tr[3 + 2 * (st[1] - 2)]) if st[1] >= 2 else int(tr[1])
                rec.update({"signal_to_stop_us": (t_stop - t_store) / 100.0, "layer_us": (t_stop - t_layer0) / 100.0,
                            "layers_started_after_signal": st[1] - (layer + 1)})
            trials.append(rec)
    finally:
        model.raise_cancel(-1, 3)
        model.set_plan(5, 0)
    ok = [t for t in trials if "signal_to_stop_us" in t]
    return {"trials": len(trials), "stopped": len(ok),
            "layers_started_after_signal_max": max((t["layers_started_after_signal"] for t in ok), default=None),
            "signal_to_stop_us_mean": float(np.mean([t["signal_to_stop_us"] for t in ok])) if ok else None,
            "signal_to_stop_us_max": float(np.max([t["signal_to_stop_us"] for t in ok])) if ok else None,
            "signal_to_stop_layers_max": float(np.max([t["signal_to_stop_us"] / t["layer_us"] for t in ok])) if ok else None,
            "signal": "cancel word stored by workgroup grid/2 on entering gate/up of the layer; clock: device, 100 MHz",
            "per_trial": trials}


def phase_timeline(pi, torch, np, model, kv, run, n, shape, layer):
    """Per-workgroup timestamps of the five phases of one layer (pi_debug_wgtrace), all from one
    forward, as min / mean / max over the workgroups in microseconds from the moment the first
    workgroup entered the layer's QKV phase."""
    logits = torch.empty((n, shape.vocab), device="cuda")
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    model.wgtrace(layer)
    for _ in range(3):
        pi.stage_forward(model, kv, run, 0, shape.n_layers, logits_out=logits, run_status=status)
        pi.kv_rollback(kv, run.slots, n)
    torch.cuda.synchronize()
    t = model.wgtrace(-1, read=True).astype(np.int64)
    t = (t - t[:, 0, 0].min()) / 100.0
    rows = {}
    for k, name in enumerate(["qkv", "attention", "o", "gate_up", "down"]):
        f = lambda j: [round(float(t[:, k, j].min()), 1), round(float(t[:, k, j].mean()), 1), round(float(t[:, k, j].max()), 1)]
        rows[name] = {"entered": f(0), "work_done": f(2)}
        if k in (2, 4):
            rows[name]["barrier_passed"] = f(5)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--shape", default="llama7b")
    ap.add_argument("--prefix", type=int, default=512)
    ap.add_argument("--batches", default="1,4,8")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cancel", action="store_true", help="skip the cancellation latency trials")
    ap.add_argument("--no-multi-run", action="store_true", help="skip the several-runs-per-pass comparison")
    ap.add_argument("--no-kv-metadata", action="store_true", help="skip the cell-metadata bookkeeping timing")
    ap.add_argument("--no-continuous", action="store_true", help="skip the continuous-speculation generation loop")
    ap.add_argument("--no-c4", action="store_true", help="skip the eight-runs-half-cancelled workload")
    ap.add_argument("--no-w8", action="store_true", help="skip the same workload with 8-bit weight matrices")
    ap.add_argument("--no-other-shapes", action="store_true",
                    help="skip the 70B-shaped (full depth and 20-layer slice) and TinyLlama-shaped decode legs")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the bare streaming probe (hbm_ceiling_GBps)")
    ap.add_argument("--phase-timeline", type=int, default=-1,
                    help="print per-phase workgroup timestamps of this layer for every batch size and exit")
    ap.add_argument("--slice-layers", type=int, default=0,
                    help="also time a pipeline stage's share: the first this-many layers as one stage call")
    ap.add_argument("--calibrate-copy", type=int, default=0,
                    help="only run a device copy of this many MiB (known traffic for counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (a pipeline stage is a layer slice on that GPU); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    from synth import gpu_loader
    import paper_2407_11798_amd as pi

    if args.calibrate_copy:
        nbytes = args.calibrate_copy << 20
        src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": nbytes, "calibrate_copy_bytes_written": nbytes, "copies": 3}))
        return
    shape = synth.SHAPES[args.shape]
    batches = [int(b) for b in args.batches.split(",")]
    T = args.prefix
    torch.cuda.set_device(0)
    model = gpu_loader.load_model(shape, args.seed)
    n_cells = ((T + 64 + 15) // 16) * 16
    kv = pi.KVCache(model, n_cells)
    gpu_loader.prefill_kv_synthetic(kv, shape, args.seed, T)
    layer_bytes, lm_bytes = model.weight_bytes()

    if args.phase_timeline >= 0:
        tl = {}
        for n in batches:
            run = gpu_loader.make_run(synth.linear_run(n, T), synth.tokens_host(shape, args.seed, n, synth.T_DRAFT, salt=n))
            tl[str(n)] = phase_timeline(pi, torch, np, model, kv, run, n, shape, args.phase_timeline)
        print(json.dumps({"phase_timeline_us": tl, "shape": shape.name, "prefix": T, "layer": args.phase_timeline,
                          "columns": "min / mean / max over the 256 workgroups, from the first workgroup's entry into the phase"}))
        return

    per_batch = {}
    for n in batches:
        rd = synth.linear_run(n, T)
        toks = synth.tokens_host(shape, args.seed, n, synth.T_DRAFT, salt=n)
        run = gpu_loader.make_run(rd, toks)
        root_expected = int(synth.tokens_host(shape, args.seed, 1, synth.T_MISC, salt=n)[0])
        logits = torch.empty((n, shape.vocab), device="cuda")
        status = torch.zeros(2, dtype=torch.int32, device="cuda")
        acc = torch.zeros(n, dtype=torch.int32, device="cuda")
        res = torch.zeros(2, dtype=torch.int32, device="cuda")

        def step(ev0=None, ev1=None):
            if ev0 is not None:
                ev0.record()
            pi.stage_forward(model, kv, run, 0, shape.n_layers, logits_out=logits, run_status=status)
            if ev1 is not None:
                ev1.record()
            pi.verify_greedy(run.tokens, run.parent, n, logits, shape.vocab, root_expected, acc, res)
            pi.kv_rollback(kv, run.slots, n, acc, res)

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e0, e1 in evs:
            step(e0, e1)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        fwd_ms = sum(e0.elapsed_time(e1) for e0, e1 in evs) / args.steps
        assert status.cpu().tolist() == [0, shape.n_layers]
        kv.set_len(T)  # an accepted draft token would have advanced the prefix; keep the workload fixed
        ms = wall * 1e3 / args.steps
        ab = algorithmic_bytes(shape, layer_bytes, lm_bytes, T, n)
        slice_ms = None
        if args.slice_layers:
            hidden = torch.empty((n, shape.d_model), device="cuda")
            sev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
            for e0, e1 in sev:
                e0.record()
                pi.stage_forward(model, kv, run, 0, args.slice_layers, hidden_out=hidden, run_status=status)
                e1.record()
                pi.kv_rollback(kv, run.slots, n)
            torch.cuda.synchronize()
            slice_ms = sum(e0.elapsed_time(e1) for e0, e1 in sev) / args.steps
        per_batch[str(n)] = {
            "slice_layers": args.slice_layers or None, "slice_forward_ms": slice_ms,
            "verified_tokens_per_s": n / (ms * 1e-3), "ms_per_step": ms, "forward_ms": fwd_ms,
            "per_layer_us": fwd_ms * 1e3 / (shape.n_layers + lm_bytes / layer_bytes),
            "algorithmic_GB": ab / 1e9, "achieved_GBps": ab / 1e9 / (fwd_ms * 1e-3),
            "frac_of_peak": ab / 1e9 / (fwd_ms * 1e-3) / HBM_PEAK_GBS,
        }

    head = str(max(batches))
    hb = per_batch[head]

    # Early Inference Cancellation latency: the host raises a mapped flag at a random moment of a
    # run and polls a mapped status word; latency = status visible - flag written (host clock).
    import ctypes
    import random
    hip = ctypes.CDLL("libamdhip64.so")
    flag_h = torch.zeros(1, dtype=torch.int32, pin_memory=True)
    stat_h = torch.zeros(2, dtype=torch.int32, pin_memory=True)
    fptr, sptr = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipHostGetDevicePointer(ctypes.byref(fptr), ctypes.c_void_p(flag_h.data_ptr()), 0) == 0
    assert hip.hipHostGetDevicePointer(ctypes.byref(sptr), ctypes.c_void_p(stat_h.data_ptr()), 0) == 0
    n = int(head)
    run = gpu_loader.make_run(synth.linear_run(n, T), synth.tokens_host(shape, args.seed, n, synth.T_DRAFT, salt=n))
    logits = torch.empty((n, shape.vocab), device="cuda")
    lat, stopped_at = [], []
    rnd = random.Random(args.seed)
    fwd_s = hb["forward_ms"] * 1e-3
    sv = stat_h.numpy()
    fv = flag_h.numpy()
    for trial in range(0 if args.no_cancel else 16):
        fv[0] = 0
        sv[0] = -99
        torch.cuda.synchronize()
        pi.binding.lib().pi_stage_forward(model.handle, kv.handle, ctypes.byref(run.desc()), 0, shape.n_layers, None,
                                          None, ctypes.c_void_p(logits.data_ptr()), fptr, sptr,
                                          ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        delay = rnd.uniform(0.1, 0.8) * fwd_s
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < delay:
            pass
        fv[0] = 1
        t_set = time.perf_counter()
        while sv[0] == -99 and time.perf_counter() - t_set < 1.0:
            pass
        t_seen = time.perf_counter()
        torch.cuda.synchronize()
        if sv[0] == 1:
            lat.append((t_seen - t_set) * 1e6)
            stopped_at.append(int(sv[1]))
        pi.kv_rollback(kv, run.slots, n)
    torch.cuda.synchronize()
    layer_us = hb["per_layer_us"]
    cancel = {"trials": 0 if args.no_cancel else 16, "cancelled": len(lat),
              "latency_us_mean": float(np.mean(lat)) if lat else None,
              "latency_us_max": float(np.max(lat)) if lat else None,
              "latency_layers_max": float(np.max(lat)) / layer_us if lat else None,
              "layers_done": stopped_at,
              "clock": "host (flag written -> status seen through mapped memory: includes PCIe visibility and host polling)"}
    if not args.no_cancel:
        cancel["device_clock"] = cancellation_on_device_clock(
            pi, torch, np, model, kv, run, n, shape, shape.n_layers,
            sorted(set(int(x) for x in np.linspace(0, shape.n_layers - 2, 8))))

    # Several runs per weight pass: eight 4-token speculation trees under the shared prefix (the
    # shape of the paper's continuous speculation: many small runs in flight), evaluated as eight
    # passes of one run each and as two passes of four runs each (pi_stage_forward_multi, every run
    # with its own cancel word; none is raised here).
    multi = None
    if not args.no_multi_run:
        trees = [synth.random_tree(args.seed, 100 + r, 4) for r in range(8)]
        singles, quads = [], []
        for r, parent in enumerate(trees):
            rd = synth.tree_run(parent, T, T, offset=4 * r)
            singles.append(gpu_loader.make_run(rd, synth.sibling_distinct_tokens(shape, args.seed, 100 + r, parent)))
        for q in range(2):
            parent = np.concatenate([np.where(trees[4 * q + j] >= 0, trees[4 * q + j] + 4 * j, -1) for j in range(4)]).astype(np.int32)
            toks = np.concatenate([synth.sibling_distinct_tokens(shape, args.seed, 100 + 4 * q + j, trees[4 * q + j])
                                   for j in range(4)]).astype(np.int32)
            quads.append((gpu_loader.make_run(synth.tree_run(parent, T, T, offset=16 * q), toks),
                          [j for j in range(4) for _ in range(4)]))
        lg4 = torch.empty((4, shape.vocab), device="cuda")
        lg16 = torch.empty((16, shape.vocab), device="cuda")
        flags = torch.zeros(4, dtype=torch.int32, device="cuda")
        gstat = torch.zeros((4, 2), dtype=torch.int32, device="cuda")

        def eight_passes():
            for run in singles:
                pi.stage_forward(model, kv, run, 0, shape.n_layers, logits_out=lg4, run_status=status)
                pi.kv_rollback(kv, run.slots, 4)

        def two_passes():
            for run, groups in quads:
                pi.stage_forward_multi(model, kv, run, groups, 0, shape.n_layers, logits_out=lg16,
                                       cancel_flags=flags, group_status=gstat, run_status=status)
                pi.kv_rollback(kv, run.slots, 16)

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps

        reps = max(2, args.steps // 10)
        t8, t2 = timed(eight_passes, reps), timed(two_passes, reps)
        assert gstat.cpu().tolist() == [[0, shape.n_layers]] * 4
        multi = {"runs": 8, "tokens_per_run": 4,
                 "one_run_per_pass": {"passes": 8, "ms": t8 * 1e3, "verified_tokens_per_s": 32 / t8},
                 "four_runs_per_pass": {"passes": 2, "ms": t2 * 1e3, "verified_tokens_per_s": 32 / t2}}

    # Eight runs in flight, half of them cancelled (Section "Early Inference Cancellation"): eight
    # 4-token tree runs over a 1024-cell prefix, one forward each; a seeded half of them has its
    # cancel word raised before a seeded layer (the stack is issued as two stage calls with the
    # store of the word in between, in stream order).  Timed with and without the cancellations.
    c4 = None
    if not args.no_c4:
        T4 = 1024
        kv4 = pi.KVCache(model, T4 + 64)
        gpu_loader.prefill_kv_synthetic(kv4, shape, args.seed, T4)
        stops = synth.cancel_schedule(args.seed, 8, shape.n_layers)
        runs4 = []
        for r in range(8):
            parent = synth.random_tree(args.seed, r, 4)
            runs4.append(gpu_loader.make_run(synth.tree_run(parent, T4, T4, offset=4 * r),
                                             synth.sibling_distinct_tokens(shape, args.seed, r, parent)))
        lg4 = torch.empty((4, shape.vocab), device="cuda")
        hid4 = torch.empty((4, shape.d_model), device="cuda")
        flag4 = torch.zeros(1, dtype=torch.int32, device="cuda")
        st4 = torch.zeros((8, 2), dtype=torch.int32, device="cuda")

        def eight_runs(cancel):
            for r, run in enumerate(runs4):
                stop = stops[r] if cancel else -1
                flag4.zero_()
                if stop > 0:
                    pi.stage_forward(model, kv4, run, 0, stop, hidden_out=hid4, cancel_flag=flag4, run_status=st4[r])
                if stop >= 0:
                    flag4.fill_(1)
                pi.stage_forward(model, kv4, run, max(stop, 0), shape.n_layers, hidden_in=hid4 if stop > 0 else None,
                                 logits_out=lg4, cancel_flag=flag4, run_status=st4[r])
                pi.kv_rollback(kv4, run.slots, 4)

        def timed4(cancel, reps):
            eight_runs(cancel)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                eight_runs(cancel)
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / reps

        reps = max(2, args.steps // 10)
        t_all = timed4(False, reps)
        t_cut = timed4(True, reps)
        done = st4.cpu().tolist()
        assert [d[0] for d in done] == [1 if s >= 0 else 0 for s in stops]
        assert [d[1] for d in done] == [s if s >= 0 else shape.n_layers for s in stops]
        layers_run = sum(d[1] for d in done)
        c4 = {"runs": 8, "tokens_per_run": 4, "prefix": T4, "cancel_before_layer": stops,
              "ms_without_cancellation": t_all * 1e3, "ms_with_cancellation": t_cut * 1e3,
              "layers_evaluated": layers_run, "layers_total": 8 * shape.n_layers,
              "weight_GB_streamed": (layers_run * layer_bytes + sum(1 for s in stops if s < 0) * lm_bytes) / 1e9,
              "weight_GB_without_cancellation": 8 * (shape.n_layers * layer_bytes + lm_bytes) / 1e9,
              "time_saved_fraction": 1.0 - t_cut / t_all, "layers_saved_fraction": 1.0 - layers_run / (8.0 * shape.n_layers)}
        kv4.free()

    # Cell metadata and sequence partitions: the bookkeeping of one round of eight 4-token tree
    # runs -- per run: partitions from the queue, cells from the window, window words from the
    # table; then the best run accepted, every partition given back, and the accepted entries
    # compacted into the dense prefix (K/V of all layers moved).  Device time per round by events
    # around the enqueued calls; the oracle's Python bookkeeping of the same round beside it.
    kvmeta = None
    if not args.no_kv_metadata:
        trees = [synth.random_tree(args.seed, 100 + r, 4) for r in range(8)]
        meta = pi.KVMeta(n_cells, 32)
        all_seq = (1 << 32) - 1
        pos_t = [torch.as_tensor(synth.tree_run(tr, T, T)["positions"], device="cuda") for tr in trees]
        slots_t = [torch.zeros(4, dtype=torch.int32, device="cuda") for _ in trees]
        mask_t = [torch.zeros(4, dtype=torch.int64, device="cuda") for _ in trees]
        stat_t = torch.zeros(1, dtype=torch.int32, device="cuda")
        bad_t = torch.zeros(1, dtype=torch.int32, device="cuda")
        res_t = torch.zeros(2, dtype=torch.int32, device="cuda")
        acc_t = torch.as_tensor(np.array([0, -1, -1, -1], dtype=np.int32), device="cuda")
        one_t = torch.as_tensor(np.array([1, 0], dtype=np.int32), device="cuda")

        def meta_round():
            meta.fill(0, T, 0, all_seq)
            meta.fill(T, n_cells - T, 0, 0)
            held, seqs_dev = [], []
            for r, tr in enumerate(trees):
                ids = [meta.acquire() for _ in range(synth.n_leaves(tr))]
                held += ids
                sq = torch.as_tensor(np.asarray([pi.seq_bits(x) for x in synth.tree_sequences(tr, ids)],
                                                dtype=np.uint32).view(np.int32), device="cuda")
                seqs_dev.append(sq)
                meta.place(4, pos_t[r], sq, T, slots_t[r], stat_t)
                meta.build_mask(4, pos_t[r], sq, T, T, mask_t[r], bad_t)
            meta.accept(4, pos_t[7], seqs_dev[7], acc_t, one_t)          # the last run's root is accepted
            for s in held:
                meta.release(s)
            meta.compact(kv, T, res_t)

        meta_round()
        torch.cuda.synchronize()
        assert res_t.cpu().tolist() == [0, T + 1] and int(bad_t.item()) == 0 and int(stat_t.item()) == 0
        reps = max(3, args.steps // 5)
        t0 = time.perf_counter()
        for _ in range(reps):
            meta_round()
        torch.cuda.synchronize()
        t_dev = (time.perf_counter() - t0) / reps
        kv.set_len(T)
        kvmeta = {"round": "8 tree runs x 4 tokens over %d cells: 8 x (place + build_mask), accept, %d releases, "
                           "compaction moving 1 cell of %d layers" % (n_cells, sum(synth.n_leaves(t) for t in trees),
                                                                      shape.n_layers),
                  "calls_per_round": 2 + 16 + 1 + sum(synth.n_leaves(t) for t in trees) + 2,
                  "us_per_round": t_dev * 1e6}
        if not args.no_cpu_baseline:
            from oracle import OracleKVMeta
            om = OracleKVMeta(n_cells, 32)
            t0 = time.perf_counter()
            om.fill(0, T, 0, range(32))
            held = []
            for r, tr in enumerate(trees):
                ids = [om.acquire() for _ in range(synth.n_leaves(tr))]
                held += ids
                sq = synth.tree_sequences(tr, ids)
                positions = synth.tree_run(tr, T, T)["positions"].tolist()
                om.place(positions, sq, T)
                om.build_mask(positions, sq, T, T)
                last = (positions, sq)
            om.accept(last[0], last[1], [0])
            for s_ in held:
                om.release(s_)
            om.compact(T)
            kvmeta["oracle_us_per_round"] = (time.perf_counter() - t0) * 1e6
        meta.free()

    # Continuous asynchronous speculation (the paper's end-to-end method on this one GPU): plain
    # greedy decoding of 64 tokens first (one token per forward: the baseline, and the sequence
    # the synthetic draft source is planted on), then the same 64 tokens generated by queued
    # speculative micro-batches whose draft tokens agree with the target with probability alpha.
    # No trained model pair exists here, so alpha stands in for the draft model's quality; the
    # paper's model pairs report acceptance rates of 0.52 to 0.79.
    contin = None
    if not args.no_continuous:
        from paper_2407_11798_amd.pipeline import ContinuousSpeculation
        n_gen = 64
        cells2 = ((T + 64 + 2 * n_gen + 15) // 16) * 16
        kv2 = pi.KVCache(model, cells2)
        first = int(synth.tokens_host(shape, args.seed, 1, synth.T_MISC, salt=77)[0])
        lg1 = torch.empty((1, shape.vocab), device="cuda")
        acc1 = torch.zeros(1, dtype=torch.int32, device="cuda")
        res1 = torch.zeros(2, dtype=torch.int32, device="cuda")
        res_h = torch.zeros(2, dtype=torch.int32, pin_memory=True)

        def naive():
            gpu_loader.prefill_kv_synthetic(kv2, shape, args.seed, T)
            torch.cuda.synchronize()
            toks, t = [], first
            t0 = time.perf_counter()
            for i in range(n_gen):
                run1 = gpu_loader.make_run(synth.linear_run(1, T + i), np.array([t], dtype=np.int32))
                pi.stage_forward(model, kv2, run1, 0, shape.n_layers, logits_out=lg1, run_status=status)
                pi.verify_greedy(run1.tokens, None, 1, lg1, shape.vocab, t, acc1, res1)
                pi.kv_rollback(kv2, run1.slots, 1, acc1, res1)
                res_h.copy_(res1, non_blocking=True)
                torch.cuda.synchronize()
                t = int(res_h[1])
                toks.append(t)
            return toks, time.perf_counter() - t0

        G, t_naive = naive()
        contin = {"tokens": n_gen, "depth": 3, "micro_batch": 4, "cutoff": {"base": 0.0, "recovery": 0.05, "decay": 0.05},
                  "plain_decoding": {"tokens_per_s": n_gen / t_naive, "ms_per_token": t_naive * 1e3 / n_gen},
                  "note": "by_alpha: every run is a pass over the weights (3 passes in flight); "
                          "by_alpha_four_runs_per_pass: up to four consecutive runs share a pass (2 passes in flight)"}
        for rpp, key in ((1, "by_alpha"), (4, "by_alpha_four_runs_per_pass")):
            contin[key] = {}
            for alpha in (0.52, 0.66, 0.79, 1.0):
                gpu_loader.prefill_kv_synthetic(kv2, shape, args.seed, T)
                u = synth.uniform_int_host(2 * (n_gen + 64), args.seed, synth.stream_id(synth.T_MISC, int(alpha * 100)), 1 << 20)

                def draft(pos, u=u, alpha=alpha):
                    i = pos - (T + 1)
                    g = G[i] if i < len(G) else 0
                    right = u[2 * i] < alpha * (1 << 20)
                    return (g if right else (g + 1 + int(u[2 * i]) % 7) % shape.vocab), float(u[2 * i + 1]) / (1 << 20)

                cs = ContinuousSpeculation(model, kv2, T, first, draft, depth=3 if rpp == 1 else 2, micro_batch=4,
                                           base_cutoff=0.0, recovery=0.05, decay=0.05, runs_per_pass=rpp)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                got = cs.generate(n_gen)
                dt = time.perf_counter() - t0
                st = dict(cs.stats)
                cs.close()
                contin[key]["%.2f" % alpha] = {
                    "tokens_per_s": n_gen / dt, "speedup_vs_plain": t_naive / dt, "same_tokens_as_plain": got == G,
                    "passes": st["passes"], "runs": st["runs"], "speculative_runs": st["speculative"],
                    "cancelled_runs": st["cancelled"], "layers_skipped": st["layers_skipped"],
                    "draft_tokens_accepted": st["tokens_accepted_from_drafts"], "draft_tokens_issued": st["tokens_speculated"]}
        kv2.free()

    # Quantised weight streaming: the same workload on the same shape with 8-bit (FP8 E4M3) and 4-bit
    # (FP4 E2M1) weight matrices, decoded in the projection kernels; bf16 activations and cache.
    w8 = None
    if not args.no_w8 and shape.weight_format == "native":
        w8 = {}
        for suffix in ("_w8", "_w4", "_w4b"):
            if shape.name + suffix not in synth.SHAPES:
                continue
            sh8 = synth.SHAPES[shape.name + suffix]
            m8 = gpu_loader.load_model(sh8, args.seed)
            kv8 = pi.KVCache(m8, n_cells)
            gpu_loader.prefill_kv_synthetic(kv8, sh8, args.seed, T)
            lb8, lm8 = m8.weight_bytes()
            leg = {"weights": "fp4-e2m1, one power-of-two scale per 32 columns of a row" if sh8.weight_format == "fp4b" else
                   "%s x 2^%d" % ({"fp8": "fp8-e4m3", "fp4": "fp4-e2m1"}[sh8.weight_format], sh8.weight_scale_exp2),
                   "per_batch": {}}
            for n in batches:
                run8 = gpu_loader.make_run(synth.linear_run(n, T), synth.tokens_host(sh8, args.seed, n, synth.T_DRAFT, salt=n))
                lg8 = torch.empty((n, sh8.vocab), device="cuda")
                evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
                for k in range(args.warmup + args.steps):
                    e = evs[k - args.warmup] if k >= args.warmup else None
                    if e:
                        e[0].record()
                    pi.stage_forward(m8, kv8, run8, 0, sh8.n_layers, logits_out=lg8, run_status=status)
                    if e:
                        e[1].record()
                    pi.kv_rollback(kv8, run8.slots, n)
                torch.cuda.synchronize()
                assert status.cpu().tolist() == [0, sh8.n_layers]
                f8 = sum(e0.elapsed_time(e1) for e0, e1 in evs) / args.steps
                ab8 = algorithmic_bytes(sh8, lb8, lm8, T, n)
                leg["per_batch"][str(n)] = {"forward_ms": f8, "verified_tokens_per_s_forward_only": n / (f8 * 1e-3),
                                            "algorithmic_GB": ab8 / 1e9, "achieved_GBps": ab8 / 1e9 / (f8 * 1e-3),
                                            "frac_of_peak": ab8 / 1e9 / (f8 * 1e-3) / HBM_PEAK_GBS,
                                            "speedup_vs_%s_weights" % shape.dtype: per_batch[str(n)]["forward_ms"] / f8}
            w8[sh8.weight_format] = leg
            kv8.free()
            m8.free()

    # The other model shapes of the workload list, forward only: the 70B-shaped target (80 layers,
    # 2048 prefix cells, batches of 1 / 4 / 8 / 16, and its first 20 layers alone: one pipeline
    # stage's share) and single-token decode steps of the TinyLlama-shaped draft model.
    other = None
    if not args.no_other_shapes and shape.name == "llama7b":
        kv.free()
        model.free()
        model = kv = None
        few = max(3, min(10, args.steps // 5))
        other = {"tinyllama_decode": shape_leg(pi, torch, synth, gpu_loader, "tinyllama", (128, 512, 2048), (1,),
                                               args.seed, max(few, 20), 5),
                 "llama70b": shape_leg(pi, torch, synth, gpu_loader, "llama70b", (2048,), (1, 4, 8, 16), args.seed, few, 2,
                                       slice_layers=20)}
    ceiling = None
    if not args.no_ceiling:
        ceiling = pi.binding.stream_probe(2 << 30, 5)

    out = {
        "metric": "verified tokens/sec per spec batch (1/4/8 tok) + achieved HBM GB/s vs peak",
        "value": hb["verified_tokens_per_s"], "unit": "verified tokens/s (n=%s)" % head,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": hb["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype,
        "data": "synthetic",
        "config": {"workload": "%s-shaped target, %s weights, %s KV, T=%d prefilled cells, speculative batches %s, "
                               "linear causal mask, uniform-random drafts"
                               % (shape.name, "fp8-e4m3" if shape.weight_format == "fp8" else shape.dtype, shape.dtype, T,
                                  args.batches),
                   "step": "pi_stage_forward(all layers + LM head) + pi_verify_greedy + pi_kv_rollback"},
        "per_batch": per_batch,
        "cancellation": cancel,
        "multi_run": multi,
        "eight_runs_half_cancelled": c4,
        "kv_metadata": kvmeta,
        "continuous_speculation": contin,
        "quantised_weights": w8,
        "other_shapes": other,
        "hbm_ceiling_GBps": ceiling,
        "roofline": {"bound": "hbm", "achieved": hb["achieved_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": hb["frac_of_peak"],
                     "traffic": MEASURED_TRAFFIC_BYTES.get((shape.name, T, int(head))),
                     "kernel": "stage_kernel (one launch per forward, n=%s)" % head,
                     "algorithmic_bytes_per_launch": hb["algorithmic_GB"] * 1e9},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, T, int(head), args.seed, [int(b) for b in batches])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
