#!/usr/bin/env python3
"""Benchmark of the sparse-DNN SGD hot path on one MI355X.

A step = one pass of the whole hot path on one training minibatch, through the
C ABI: sdnn_forward, loss gradient, sdnn_backward, sdnn_sgd_step.  Throughput
is edges/s = (sum of nnz over the layers) x samples / seconds, the throughput
definition of the paper's inference table (Section 6.4), applied to the full
training step and, in a second figure, to the inference forward pass.

The default workload is the largest configuration at full depth (config 4:
65536 neurons per layer, 120 layers, 251 M stored entries, minibatch 64,
8192 inference samples streamed in blocks of 1024).  The other four
configurations are measured in the same run, each at full depth, and carried in
the key "other_configs" of the same JSON line.

Prints ONE JSON line.  Inputs are resident in HBM before the timed region.
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
T_START = time.time()

# input density just above the point where the benchmark nets die (-bias): every activation stays non-zero
LIVE_DENSITY = {1: 0.40, 2: 0.40, 3: 0.40, 4: 0.60}


def log(msg):
    print(f"[bench {time.time() - T_START:6.1f}s] {msg}", file=sys.stderr, flush=True)


def layer_bytes(n, nnz, b, fused):
    """Algorithmic HBM bytes per layer of each pass (every array moved once; gathers served on chip).

    forward   index + values (8 nnz), row schedule (16 n), bias (4 n), X in and X out
    backward  separate: transposed index + position (8 nnz), values through it (4 nnz), schedule, Delta in, X mask,
              Delta out; fused sweep: transposed index + values in that order (8 nnz), gradient written (4 nnz), the rest
              the same
    update    separate: index (4 nnz), values read + written (8 nnz), schedule, bias r/w, Delta, X
              after a fused sweep: transposed-order values r/w + gradient read (12 nnz), then the CSR copy rebuilt
              (inverse position, value read, value written: 12 nnz), bias r/w, Delta (bias gradient)
    """
    act = 4 * n * b
    fwd = 8 * nnz + 16 * n + 4 * n + 2 * act
    bwd = 12 * nnz + 16 * n + 3 * act
    upd = (24 * nnz + 8 * n + act) if fused else (12 * nnz + 16 * n + 8 * n + 2 * act)
    return fwd, bwd, upd


def workload_name(cfg, n, n_layers):
    return (f"config {cfg}: N={n}, L={n_layers}, 32 nnz/row" if cfg < 5
            else f"config 5: N={n}, L={n_layers}, heavy-tailed rows")


def run_config(cfg, args, steps, warmup, headline):
    """Training step and inference of one configuration; returns the figures as a dict."""
    import numpy as np
    import torch
    from paper_2104_11805_amd import sdnn, workloads as wl

    dev = "cuda:0"
    layers_arg = args.layers if headline else None
    density_arg = args.density if headline else None
    t0 = time.time()
    work = wl.make_config(cfg, n_layers=layers_arg, density=density_arg)
    N, L, nnz_total = work.n, len(work.layers), work.total_nnz
    Bt, Bi = work.train_batch, work.x_infer.shape[1]
    gen_s = time.time() - t0
    log(f"config {cfg}: generated {L} layers, {nnz_total} entries, inputs {work.x_infer.shape} in {gen_s:.1f} s")

    def to_dev(a, dtype=None):
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t.to(dtype) if dtype is not None else t).to(dev)

    # ---- training step --------------------------------------------------
    t0 = time.time()
    opts = dict(panel_cols=args.panel_cols, fuse_gradient=args.fuse_gradient) if headline else {}
    net = sdnn.Net(work.layers, work.act_cap, Bt, training=True, **opts)
    torch.cuda.synchronize()
    create_s = time.time() - t0
    log(f"config {cfg}: training net created in {create_s:.1f} s, workspace {net.workspace_bytes / 2**30:.2f} GiB")
    # which kernels the library picks for this shape (its measured launch policy, restated here to name them):
    # short rows and small layers run as two half-batches on two streams; layers of >= 4096 rows form the gradient in
    # the backward sweep where a launch holds at most 64 samples (short rows) or the batch at most 256 (long rows)
    short_rows = nnz_total < 128 * N * L
    split = short_rows and Bt % 128 == 0 and N * Bt <= 2 ** 21
    fuse_opt = args.fuse_gradient if headline else 0
    fused = ((N >= 4096 or fuse_opt > 0) and fuse_opt >= 0
             and ((short_rows and ((split and Bt == 128) or (not split and 1 < Bt <= 64)))
                  or (not short_rows and Bt <= 256 and Bt % 4 == 0)))
    if split:
        v = 4 if Bt % 512 == 0 else 2 if Bt % 256 == 0 else 1
    else:
        v = 4 if (Bt % 4 == 0 and Bt > 128) else 2 if (Bt % 2 == 0 and Bt > 64) else 1
    x0 = to_dev(work.x_train)
    xl = torch.empty(work.layers[-1].n_out, Bt, device=dev)
    dl = torch.empty_like(xl)
    if work.loss == "mse":
        y = to_dev(work.targets)
        loss_grad = lambda: sdnn.sdnn_mse_dloss(xl, y, out=dl)
    else:
        lab = to_dev(work.labels, torch.int32)
        loss_grad = lambda: sdnn.sdnn_softmax_ce_dloss(xl, lab, work.n_classes, out=dl)

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(x, marks=None):
        e = [ev() for _ in range(4)] if marks is not None else None
        if e: e[0].record()
        net.sdnn_forward(x, xl)
        if e: e[1].record()
        loss_grad()
        net.sdnn_backward(dl)
        if e: e[2].record()
        net.sdnn_sgd_step(work.lr)
        if e: e[3].record()
        if e: marks.append(e)

    w_first = [t.clone() for t in net.sdnn_get_weights(1)]
    w_last = [t.clone() for t in net.sdnn_get_weights(L)]
    for _ in range(warmup):
        step(x0)
    marks = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(x0, marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / steps
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in marks) / len(marks)
    bwd_ms = sum(e[1].elapsed_time(e[2]) for e in marks) / len(marks)
    upd_ms = sum(e[2].elapsed_time(e[3]) for e in marks) / len(marks)
    per_step = sorted(e[0].elapsed_time(e[3]) for e in marks)       # event time of each single step
    train_eps = nnz_total * Bt / (ms_step * 1e-3)
    # did the timed steps change the weights?  (nominal inputs of configs 1-4: every gradient is exactly zero,
    # so every timed step saw the same weights; otherwise the steps are a real descent)
    unchanged = all(torch.equal(a, b) for a, b in zip(w_first + w_last,
                                                      list(net.sdnn_get_weights(1)) + list(net.sdnn_get_weights(L))))
    # share of non-zero activations after layers 1, 2 and L of the minibatch (the nominal inputs of configs 1-4
    # die out after the first layers; the kernels never skip zeros, so the timing does not profit from it)
    net.sdnn_forward(x0, xl)
    active = {f"layer_{k}": round(float((net.sdnn_get_activation(k, Bt) != 0).float().mean()), 4)
              for k in sorted({1, min(2, L), L})}
    log(f"config {cfg}: step {ms_step:.3f} ms (fwd {fwd_ms:.3f} bwd {bwd_ms:.3f} upd {upd_ms:.3f}), "
        f"{train_eps:.3e} edges/s")

    # ---- the same step on live inputs: every rep starts from the same weights, restored outside the events ----
    live = None
    if cfg in LIVE_DENSITY and density_arg is None and not args.no_live:
        d_live = LIVE_DENSITY[cfg]
        xlive = to_dev(wl.binary_inputs(1000 * cfg + 902, N, Bt, d_live))
        saved = [tuple(t.clone() for t in net.sdnn_get_weights(k)) for k in range(1, L + 1)]
        reps = max(3, steps // 4)
        lmarks = []
        for r in range(reps + 1):
            for k in range(1, L + 1):
                net.sdnn_set_weights(k, saved[k - 1][0], saved[k - 1][1])
            step(xlive, lmarks if r > 0 else None)                  # the first one warms up
        torch.cuda.synchronize()
        lms = sorted(e[0].elapsed_time(e[3]) for e in lmarks)
        net.sdnn_forward(xlive, xl)
        lact = {f"layer_{k}": round(float((net.sdnn_get_activation(k, Bt) != 0).float().mean()), 4)
                for k in sorted({1, min(2, L), L})}
        for k in range(1, L + 1):
            net.sdnn_set_weights(k, saved[k - 1][0], saved[k - 1][1])
        live = {"input_density": d_live, "step_ms_median": round(lms[len(lms) // 2], 4), "step_ms_min": round(lms[0], 4),
                "edges_per_s": nnz_total * Bt / (lms[len(lms) // 2] * 1e-3), "reps": reps,
                "weights_restored_between_reps": True, "active_fraction": lact}
        del saved, xlive
        log(f"config {cfg}: live inputs (density {d_live}) step {live['step_ms_median']:.3f} ms")

    # ---- roofline of the dominant kernel --------------------------------
    fb = bb = ub = 0
    for lay in work.layers:
        f, b, u = layer_bytes(lay.n_out, lay.nnz, Bt, fused)
        fb += f; bb += b; ub += u
    first = work.layers[0]
    # separate backward: layers L..2 only; fused sweep: all layers, the first one without a Delta output
    bb -= (4 * first.n_in * Bt) if fused else layer_bytes(first.n_out, first.nnz, Bt, fused)[1]
    panels = short_rows and N * 256 >= (8 << 20) and (args.panel_cols >= 0 or not headline)   # the library's policy
    kernels = {"forward": "k_spmm_panel<8,0>" if panels else f"k_spmm<{v},0,{8 if short_rows else 16}>",
               "backward": ("k_bwd_grad<8>" if short_rows else "k_bwd_grad4<8>") if fused else f"k_spmm<{v},1,{8 if short_rows else 16}>",
               "update": "k_apply + k_gather_vals + k_apply_bias" if fused else "k_update<4>"}
    passes = {"forward": (fwd_ms, fb, L), "backward": (bwd_ms, bb, L if fused else L - 1), "update": (upd_ms, ub, 1)}
    dom = max(passes, key=lambda k: passes[k][0])
    d_ms, d_bytes, d_units = passes[dom]
    achieved = d_bytes / (d_ms * 1e-3) / 1e9
    # measured HBM-side bytes per unit of that pass (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by the
    # copy-kernel calibration), from the committed counter summary of this same workload
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"config{cfg}_traffic.json")
    if os.path.exists(tpath) and density_arg is None:
        t = json.load(open(tpath))
        k = t["kernels"].get(dom)
        if k:
            traffic = int(1024 * (k["fetch_KiB"] * t["scale"]["FETCH_SIZE"] + k["write_KiB"] * t["scale"]["WRITE_SIZE"]))
    roofline = {"bound": "hbm", "kernel": kernels[dom], "pass": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "units_per_step": d_units, "unit_of_work": "one layer" if dom != "update" else "all layers",
                "avg_unit_us": round(d_ms * 1e3 / d_units, 3), "bytes_per_unit": int(d_bytes / d_units),
                "kernel_launches_per_unit": 2 if (dom != "update" and split) else 1,
                "per_pass_frac": {p: round(passes[p][1] / (passes[p][0] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) for p in passes},
                "step_frac": round((fb + bb + ub) / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    net.close()
    del net, x0
    torch.cuda.empty_cache()

    # ---- inference forward over the full sample set ----------------------
    infer = None
    if not args.no_inference:
        block = (args.infer_block if headline else 0) or min(Bi, 1024 if N >= 65536 else Bi)
        t0 = time.time()
        iopts = dict(panel_cols=args.panel_cols, lds_forward=args.lds_forward) if headline else {}
        inet = sdnn.Net(work.layers, work.act_cap, block, training=False, **iopts)
        torch.cuda.synchronize()
        icreate_s = time.time() - t0
        blocks = [(s, min(block, Bi - s)) for s in range(0, Bi, block)]
        xin = [to_dev(work.x_infer[:, s:s + w]) for s, w in blocks]
        xout = [torch.empty(work.layers[-1].n_out, w, device=dev) for s, w in blocks]

        def infer_pass():
            for a, o in zip(xin, xout):
                inet.sdnn_forward(a, o)

        infer_pass()
        torch.cuda.synchronize()
        k = max(3, steps // 4)
        t0 = time.perf_counter()
        for _ in range(k):
            infer_pass()
        torch.cuda.synchronize()
        ims = (time.perf_counter() - t0) * 1e3 / k
        ibytes = sum(layer_bytes(l.n_out, l.nnz, Bi, False)[0] for l in work.layers)
        infer = {"edges_per_s": nnz_total * Bi / (ims * 1e-3), "ms": round(ims, 3), "samples": Bi,
                 "block": block, "algorithmic_GBs": round(ibytes / (ims * 1e-3) / 1e9, 1),
                 "hbm_frac": round(ibytes / (ims * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "create_s": round(icreate_s, 2)}
        log(f"config {cfg}: inference {ims:.3f} ms for {Bi} samples, {infer['edges_per_s']:.3e} edges/s")
        # second figure, never the headline: the same inference with dead samples dropped (ReLU, biases <= 0);
        # the edge count in the numerator then includes edges that were never visited
        if not args.no_skip_dead and work.activation == "relu" and all((l.bias <= 0).all() for l in work.layers[1:]):
            n_live = torch.zeros(1, dtype=torch.int32, device=dev)
            xchk = [torch.empty_like(o) for o in xout]
            live_end = 0
            for a, o in zip(xin, xchk):
                inet.sdnn_forward_skip_dead(a, o, check_every=args.check_every, n_live=n_live)
                live_end += int(n_live.item())
            same = all(torch.equal(a, b) for a, b in zip(xout, xchk))
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(k):
                for a, o in zip(xin, xchk):
                    inet.sdnn_forward_skip_dead(a, o, check_every=args.check_every, n_live=n_live)
            torch.cuda.synchronize()
            sms = (time.perf_counter() - t0) * 1e3 / k
            infer["skip_dead"] = {"edges_per_s": nnz_total * Bi / (sms * 1e-3), "ms": round(sms, 3),
                                  "check_every": args.check_every, "live_samples_at_last_check": live_end,
                                  "identical_to_plain_forward": bool(same)}
            del xchk
        inet.close()
        del inet, xin, xout
        torch.cuda.empty_cache()

    # ---- the oracle on the host cores, as a baseline (headline workload only) ----------------------
    cpu = None
    if headline and not args.no_cpu_baseline:
        from oracle.sdnn_oracle import Oracle, mse_dloss, softmax_ce_dloss
        orc = Oracle(np.float32)
        if work.loss == "mse":
            dfn = lambda x: mse_dloss(x, work.targets)          # same shape at any depth: the net is square
        else:
            dfn = lambda x: softmax_ce_dloss(x, work.labels, work.n_classes)
        # bounded sample: a depth prefix worth about 1.5e10 edge visits (10-30 s of CPU work)
        per_layer = 3.0 * (nnz_total / L) * Bt
        Ls = int(max(1, min(L, args.cpu_edge_visits // per_layer)))
        sub = work.layers[:Ls]
        t0 = time.perf_counter()
        orc.train_step(sub, work.x_train, work.act_cap, dfn, work.lr)
        cs = time.perf_counter() - t0
        cpu = {"value": sum(l.nnz for l in sub) * Bt / cs, "unit": "edges/s", "cores": orc.threads(),
               "kind": "oracle",
               "sample": f"one training step on the first {Ls} of {L} layers, full minibatch {Bt} ({cs:.1f} s)"}
        # the same oracle on one thread, on a shorter depth prefix
        n_all = orc.threads()
        L1 = int(max(1, min(Ls, (args.cpu_edge_visits / 6) // per_layer)))
        orc.set_threads(1)
        t0 = time.perf_counter()
        orc.train_step(work.layers[:L1], work.x_train, work.act_cap, dfn, work.lr)
        c1 = time.perf_counter() - t0
        orc.set_threads(n_all)
        cpu["single_thread"] = {"value": sum(l.nnz for l in work.layers[:L1]) * Bt / c1, "unit": "edges/s",
                                "sample": f"first {L1} layers ({c1:.1f} s)"}
        log(f"config {cfg}: oracle {cpu['value']:.3e} edges/s on {cpu['cores']} threads ({cs:.1f} s)")

    return {
        "workload": workload_name(cfg, N, L), "train_batch": Bt, "infer_samples": Bi, "total_nnz": nnz_total,
        "input_density": work.meta.get("density"), "active_fraction": active,
        "ms_per_step": round(ms_step, 4), "step_ms_min": round(per_step[0], 4),
        "step_ms_median": round(per_step[len(per_step) // 2], 4), "edges_per_s": train_eps, "steps": steps,
        "weights_unchanged_by_the_timed_steps": bool(unchanged), "gradient_formed_in_backward_sweep": bool(fused),
        "pass_ms": {"forward": round(fwd_ms, 4), "backward": round(bwd_ms, 4), "update": round(upd_ms, 4)},
        "live_inputs": live, "inference": infer, "roofline": roofline, "cpu_baseline": cpu,
        "setup_s": {"generate": round(gen_s, 2), "create": round(create_s, 2)},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 1..5 (the headline workload)")
    ap.add_argument("--layers", type=int, default=None, help="depth prefix (default: full depth)")
    ap.add_argument("--density", type=float, default=None, help="input density override (live inputs)")
    ap.add_argument("--paper-setup", action="store_true",
                    help="the paper's own training experiment: sigmoid, weights U[-1,1], one input vector per step")
    ap.add_argument("--n", type=int, default=1024, help="neurons per layer for --paper-setup")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-edge-visits", type=float, default=1.5e10,
                    help="size of the oracle's bounded sample, in edge visits (3 per edge-sample of a step)")
    ap.add_argument("--check-every", type=int, default=4,
                    help="layers between two packings of the live samples in the skip-dead inference figure")
    ap.add_argument("--infer-block", type=int, default=0,
                    help="samples per sdnn_forward call of the inference figure (0: all, 1024 for N >= 65536)")
    ap.add_argument("--no-inference", action="store_true")
    ap.add_argument("--no-skip-dead", action="store_true", help="leave out the skip-dead inference figure")
    ap.add_argument("--no-live", action="store_true", help="leave out the live-input repetition of the step")
    ap.add_argument("--others", type=str, default=None,
                    help="comma-separated configurations for the key other_configs (default: the other four when "
                         "the headline runs at full depth with nominal inputs; 'none' for none)")
    ap.add_argument("--gather-ceiling", action="store_true",
                    help="what a pure stream of random row gathers reaches, by table size and row width (the ceiling "
                         "of the product kernels' operand gathers)")
    ap.add_argument("--reorder-study", action="store_true",
                    help="row order chosen for gather locality (reorder_rows) on and off: a structured topology "
                         "(rows in groups of 32 share their columns) and the random config-2 pattern")
    ap.add_argument("--reorder", choices=["both", "0", "1"], default="both",
                    help="--reorder-study: which settings of reorder_rows to run (one at a time for counter runs)")
    ap.add_argument("--panel-cols", type=int, default=0, help="sdnn_config.panel_cols of the headline nets and of --reorder-study (0 auto, -1 off)")
    ap.add_argument("--fuse-gradient", type=int, default=0, help="sdnn_config.fuse_gradient of the headline training net (0 auto, 1 on, -1 off)")
    ap.add_argument("--lds-forward", type=int, default=0, help="sdnn_config.lds_forward of the headline inference net (0 auto, 1 on, -1 off)")
    ap.add_argument("--time-budget", type=float, default=400.0,
                    help="seconds since program start after which no further other_configs entry is begun")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2104_11805_amd import sdnn, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    log("torch and the library are loaded")
    if args.paper_setup:
        return paper_setup_bench(args, np, torch, sdnn, wl)
    if args.reorder_study:
        return reorder_study(args, np, torch, sdnn, wl)
    if args.gather_ceiling:
        return gather_ceiling(args, np, torch, sdnn)

    head = run_config(args.config, args, args.steps, args.warmup, headline=True)
    if args.others is None:
        others = [c for c in (3, 5, 2, 1) if c != args.config] if (args.layers is None and args.density is None) else []
    else:
        others = [] if args.others == "none" else [int(c) for c in args.others.split(",")]
    other_configs = {}
    for c in others:
        if time.time() - T_START > args.time_budget:
            other_configs[f"config {c}"] = {"skipped": f"time budget of {args.time_budget:.0f} s used up"}
            continue
        r = run_config(c, args, max(5, args.steps // 2), max(1, args.warmup - 1), headline=False)
        r.pop("cpu_baseline")
        other_configs[f"config {c}"] = r

    out = {
        "metric": "edges/s, forward+backward+SGD step (nnz x samples / time)",
        "value": head["edges_per_s"], "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "step_ms_min": head["step_ms_min"],
        "step_ms_median": head["step_ms_median"], "edge_visits_per_s": 3.0 * head["edges_per_s"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": head["workload"], "train_batch": head["train_batch"],
                   "infer_samples": head["infer_samples"], "total_nnz": head["total_nnz"],
                   "storage": "fp32", "accumulate": "fp64", "input_density": head["input_density"],
                   "active_fraction": head["active_fraction"],
                   "weights_unchanged_by_the_timed_steps": head["weights_unchanged_by_the_timed_steps"],
                   "gradient_formed_in_backward_sweep": head["gradient_formed_in_backward_sweep"]},
        "pass_ms": head["pass_ms"], "live_inputs": head["live_inputs"],
        "inference": head["inference"], "roofline": head["roofline"], "cpu_baseline": head["cpu_baseline"],
        "setup_s": head["setup_s"], "other_configs": other_configs,
        "total_s": round(time.time() - T_START, 1),
    }
    print(json.dumps(out))


# Time per input vector of a full SGD step in the paper's strong-scaling figure (Section 6.3),
# hypergraph-partitioned runs on 32 and on 512 cores of a Haswell/InfiniBand cluster, in ms.  Context only:
# other hardware, the real benchmark nets, precision not stated.
PAPER_MS_PER_VECTOR = {1024: (95.2, 41.1), 4096: (272.4, 81.6), 16384: (1143.1, 199.5), 65536: (6624.7, 571.2)}


def paper_setup_bench(args, np, torch, sdnn, wl):
    """One input vector per SGD step (B = 1), sigmoid, MSE, weights U[-1,1], lr 0.01, 120 layers."""
    dev = "cuda:0"
    L = args.layers or 120
    work = wl.paper_training_setup(args.n, n_layers=L, n_inputs=64)
    net = sdnn.Net(work.layers, work.act_cap, 1, training=True, activation="sigmoid", fuse_gradient=args.fuse_gradient)
    xs = [torch.from_numpy(np.ascontiguousarray(work.x_infer[:, s:s + 1])).to(dev) for s in range(64)]
    ys = [torch.from_numpy(np.ascontiguousarray(work.targets[:, s:s + 1])).to(dev) for s in range(64)]
    xl = torch.empty(args.n, 1, device=dev)
    dl = torch.empty_like(xl)

    def step(i):
        net.sdnn_forward(xs[i % 64], xl)
        sdnn.sdnn_mse_dloss(xl, ys[i % 64], out=dl)
        net.sdnn_backward(dl)
        net.sdnn_sgd_step(work.lr)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    cpu = None
    if not args.no_cpu_baseline:
        from oracle.sdnn_oracle import Oracle, mse_dloss
        orc = Oracle(np.float32, "sigmoid")
        x0, y0 = work.x_infer[:, :1], work.targets[:, :1]
        orc.train_step(work.layers, x0, work.act_cap, lambda x: mse_dloss(x, y0), work.lr)
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            orc.train_step(work.layers, x0, work.act_cap, lambda x: mse_dloss(x, y0), work.lr)
        cs = (time.perf_counter() - t0) / reps
        cpu = {"value": cs * 1e3, "unit": "ms per input vector", "cores": orc.threads(), "kind": "oracle",
               "sample": f"{reps} full steps on one vector, all {L} layers"}
    ctx = PAPER_MS_PER_VECTOR.get(args.n) if L == 120 else None
    print(json.dumps({
        "metric": "ms per input vector, full SGD step (forward+backward+update), one vector per step",
        "value": ms, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"paper training setup: N={args.n}, L={L}, 32 nnz/row, sigmoid, B=1",
                   "total_nnz": work.total_nnz, "storage": "fp32", "accumulate": "fp64"},
        "edges_per_s": work.total_nnz / (ms * 1e-3),
        "paper_context_ms": None if ctx is None else {"32 cores": ctx[0], "512 cores": ctx[1],
                                                      "note": "paper Fig. 4, other hardware and the real nets: context only"},
        "cpu_baseline": cpu}))
    net.close()


def gather_ceiling(args, np, torch, sdnn):
    """Random gathers of rows of 64*v floats from tables of 1 MiB .. 256 MiB, 8 / 16 / 32 wavefronts per CU, each
    streaming 256 gathers with 8 in flight (sdnn_gather_probe): TB/s and rows per microsecond."""
    dev = "cuda:0"
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    per_wave, reps, rows_out = 256, 10, []
    for v in (1, 4):
        for mib in (1, 4, 16, 64, 256):
            n_rows = mib * 2 ** 20 // (256 * v)
            table = torch.zeros(n_rows, 64 * v, device=dev)
            for wpc in (8, 16, 32):
                n_waves = n_cu * wpc
                idx = torch.randint(0, n_rows, (n_waves * per_wave,), device=dev, dtype=torch.int32,
                                    generator=torch.Generator(device=dev).manual_seed(7))
                out = torch.empty(n_waves * 64, device=dev)
                for _ in range(3):
                    sdnn.sdnn_gather_probe(table, v, idx, n_waves, per_wave, out)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    sdnn.sdnn_gather_probe(table, v, idx, n_waves, per_wave, out)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / reps
                r = {"row_bytes": 256 * v, "table_MiB": mib, "waves_per_cu": wpc, "us": round(us, 2),
                     "TB_per_s": round(n_waves * per_wave * 256.0 * v / us * 1e-6, 2),
                     "rows_per_us": round(n_waves * per_wave / us, 1)}
                rows_out.append(r)
                log(str(r))
            del table
    print(json.dumps({"study": "ceiling of random row gathers (sdnn_gather_probe)", "gathers_per_wavefront": per_wave,
                      "in_flight_per_wavefront": 8, "results": rows_out}))


def reorder_study(args, np, torch, sdnn, wl):
    """Times the training step (minibatch 64) and the inference forward (1024 samples) of two nets with the
    rows in the default longest-first order and in the clustered order of reorder_rows = 1: a structured
    topology, where groups of 32 rows share their 32 columns, and the uniformly random pattern of config 2."""
    dev = "cuda:0"
    n = args.n if args.n != 1024 else 65536
    L = args.layers or 12
    nets = {f"structured (strided links), N={n}, L={L}": [wl.strided_layer(8000 + l, n, value=0.0625, bias=-0.3)
                                                          for l in range(L)],
            f"random (config 2 pattern), N=4096, L={4 * L}": wl.make_config(2, n_layers=4 * L, with_inputs=False).layers}
    out = {}
    for name, layers in nets.items():
        N = layers[0].n_in
        x = torch.from_numpy(wl.binary_inputs(8900, N, 1024, 0.3)).to(dev)
        xt = x[:, :64].contiguous()
        y = torch.rand(N, 64, device=dev)
        res = {}
        for reorder in ((False, True) if args.reorder == "both" else (args.reorder == "1",)):
            t0 = time.time()
            net = sdnn.Net(layers, 32.0, 64, training=True, reorder_rows=reorder, panel_cols=args.panel_cols)
            torch.cuda.synchronize()
            create_s = time.time() - t0
            xl = torch.empty(N, 64, device=dev)
            dl = torch.empty_like(xl)
            marks = []
            for i in range(args.warmup + args.steps):
                e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                e[0].record(); net.sdnn_forward(xt, xl)
                e[1].record(); sdnn.sdnn_mse_dloss(xl, y, out=dl); net.sdnn_backward(dl)
                e[2].record(); net.sdnn_sgd_step(0.0)
                e[3].record()
                if i >= args.warmup:
                    marks.append(e)
            torch.cuda.synchronize()
            avg = lambda a, b: sum(e[a].elapsed_time(e[b]) for e in marks) / len(marks)
            r = {"step_ms": round(avg(0, 3), 4), "forward_ms": round(avg(0, 1), 4), "backward_ms": round(avg(1, 2), 4),
                 "update_ms": round(avg(2, 3), 4), "create_s": round(create_s, 2)}
            net.close()
            inet = sdnn.Net(layers, 32.0, 1024, training=False, reorder_rows=reorder, panel_cols=args.panel_cols)
            o = torch.empty(N, 1024, device=dev)
            inet.sdnn_forward(x, o)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(max(3, args.steps // 2)):
                inet.sdnn_forward(x, o)
            torch.cuda.synchronize()
            r["inference_ms"] = round((time.perf_counter() - t0) * 1e3 / max(3, args.steps // 2), 4)
            r["checksum"] = float(o.double().sum())
            inet.close()
            res["reorder_rows=1" if reorder else "reorder_rows=0"] = r
        assert len({r["checksum"] for r in res.values()}) == 1
        out[name] = res
        log(f"{name}: {res}")
    print(json.dumps({"study": "row order for gather locality (reorder_rows)", "panel_cols": args.panel_cols, "train_batch": 64, "infer_samples": 1024,
                      "steps": args.steps, "results": out}))


if __name__ == "__main__":
    main()
