#!/usr/bin/env python3
"""Benchmark of the sparse-DNN SGD hot path on one MI355X.

A step = one pass of the whole hot path on one training minibatch, through the
C ABI: sdnn_forward, loss gradient, sdnn_backward, sdnn_sgd_step.  Throughput
is edges/s = (sum of nnz over the layers) x samples / seconds, the throughput
definition of the paper's inference table (Section 6.4), applied to the full
training step and, in a second figure, to the inference forward pass.

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


def layer_bytes(n, nnz, b):
    """Algorithmic HBM bytes of one launch per layer (each array moved once)."""
    act = 4 * n * b
    fwd = 8 * nnz + 4 * (n + 1) + 4 * n + 2 * act                 # W, row_ptr, bias, X in, X out
    bwd = 12 * nnz + 4 * (n + 1) + 3 * act                          # index+perm, values, D in, X mask, D out
    upd = 8 * nnz + 4 * nnz + 4 * (n + 1) + 8 * n + 2 * act         # W r/w, bias r/w, D, X
    return fwd, bwd, upd


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5")
    ap.add_argument("--layers", type=int, default=None, help="depth prefix (default: full depth)")
    ap.add_argument("--density", type=float, default=None, help="input density override (live inputs)")
    ap.add_argument("--paper-setup", action="store_true",
                    help="the paper's own training experiment: sigmoid, weights U[-1,1], one input vector per step")
    ap.add_argument("--n", type=int, default=1024, help="neurons per layer for --paper-setup")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--check-every", type=int, default=4,
                    help="layers between two packings of the live samples in the skip-dead inference figure")
    ap.add_argument("--infer-block", type=int, default=0,
                    help="samples per sdnn_forward call of the inference figure (0: all, 1024 for N >= 65536)")
    ap.add_argument("--no-inference", action="store_true")
    ap.add_argument("--no-skip-dead", action="store_true", help="leave out the skip-dead inference figure")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2104_11805_amd import sdnn, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    if args.paper_setup:
        return paper_setup_bench(args, np, torch, sdnn, wl)
    t0 = time.time()
    work = wl.make_config(args.config, n_layers=args.layers, density=args.density)
    N, L, nnz_total = work.n, len(work.layers), work.total_nnz
    Bt, Bi = work.train_batch, work.x_infer.shape[1]
    gen_s = time.time() - t0

    def to_dev(a, dtype=None):
        t = torch.from_numpy(np.ascontiguousarray(a))
        return (t.to(dtype) if dtype is not None else t).to(dev)

    # ---- training step --------------------------------------------------
    net = sdnn.Net(work.layers, work.act_cap, Bt, training=True)
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
    marks = []

    def step(record=False):
        e = [ev() for _ in range(4)] if record else None
        if record: e[0].record()
        net.sdnn_forward(x0, xl)
        if record: e[1].record()
        loss_grad()
        net.sdnn_backward(dl)
        if record: e[2].record()
        net.sdnn_sgd_step(work.lr)
        if record: e[3].record()
        if record: marks.append(e)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(record=True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in marks) / len(marks)
    bwd_ms = sum(e[1].elapsed_time(e[2]) for e in marks) / len(marks)
    upd_ms = sum(e[2].elapsed_time(e[3]) for e in marks) / len(marks)
    per_step = sorted(e[0].elapsed_time(e[3]) for e in marks)       # event time of each single step
    train_eps = nnz_total * Bt / (ms_step * 1e-3)
    # share of non-zero activations after layers 1, 2 and L of the minibatch (the nominal inputs of configs 1-4
    # die out after the first layers; the kernels never skip zeros, so the timing does not profit from it)
    net.sdnn_forward(x0, xl)
    active = {f"layer_{k}": round(float((net.sdnn_get_activation(k, Bt) != 0).float().mean()), 4)
              for k in sorted({1, min(2, L), L})}

    # ---- roofline of the dominant kernel --------------------------------
    fb = bb = ub = 0
    for lay in work.layers:
        f, b, u = layer_bytes(lay.n_out, lay.nnz, Bt)
        fb += f; bb += b; ub += u
    passes = {"forward": (fwd_ms, fb, L), "backward": (bwd_ms, bb - layer_bytes(N, work.layers[0].nnz, Bt)[1], L - 1),
              "update": (upd_ms, ub, 1)}
    dom = max(passes, key=lambda k: passes[k][0])
    d_ms, d_bytes, d_launches = passes[dom]
    achieved = d_bytes / (d_ms * 1e-3) / 1e9
    # measured HBM-side bytes per launch of that kernel (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by the
    # copy-kernel calibration), taken from the committed counter summary of this same workload
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"config{args.config}_traffic.json")
    if os.path.exists(tpath) and args.layers is None and args.density is None:
        t = json.load(open(tpath))
        k = t["kernels"][dom]
        traffic = int(1024 * (k["fetch_KiB"] * t["scale"]["FETCH_SIZE"] + k["write_KiB"] * t["scale"]["WRITE_SIZE"]))
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "binding_unit": "vector L1 gather path (~30 B/clk/CU, see profiles/config2_counters.md)",
                "units_per_step": d_launches, "unit_of_work": "one layer" if dom != "update" else "all layers",
                "avg_unit_us": round(d_ms * 1e3 / d_launches, 3), "bytes_per_unit": int(d_bytes / d_launches),
                # forward/backward over small layers: each layer is two half-batch launches on two streams
                "kernel_launches_per_unit": 2 if (dom != "update" and Bt % 128 == 0 and N * Bt <= 2 ** 21) else 1}
    net.close()
    del net

    # ---- inference forward over the full sample set ----------------------
    infer = None
    if not args.no_inference:
        block = args.infer_block or min(Bi, 1024 if N >= 65536 else Bi)
        inet = sdnn.Net(work.layers, work.act_cap, block, training=False)
        xi = to_dev(work.x_infer)
        blocks = [(s, min(block, Bi - s)) for s in range(0, Bi, block)]
        xin = [xi[:, s:s + w].contiguous() for s, w in blocks]
        xout = [torch.empty(work.layers[-1].n_out, w, device=dev) for s, w in blocks]

        def infer_pass():
            for a, o in zip(xin, xout):
                inet.sdnn_forward(a, o)

        for _ in range(max(1, args.warmup)):
            infer_pass()
        torch.cuda.synchronize()
        k = max(3, args.steps // 2)
        t0 = time.perf_counter()
        for _ in range(k):
            infer_pass()
        torch.cuda.synchronize()
        ims = (time.perf_counter() - t0) * 1e3 / k
        ibytes = sum(layer_bytes(l.n_out, l.nnz, Bi)[0] for l in work.layers)
        infer = {"edges_per_s": nnz_total * Bi / (ims * 1e-3), "ms": round(ims, 3), "samples": Bi,
                 "block": block, "algorithmic_GBs": round(ibytes / (ims * 1e-3) / 1e9, 1),
                 "hbm_frac": round(ibytes / (ims * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        # second figure, never the headline: the same inference with dead samples dropped (ReLU, biases <= 0);
        # the edge count in the numerator then includes edges that were never visited
        if not args.no_skip_dead and work.activation == "relu" and all((l.bias <= 0).all() for l in work.layers[1:]):
            n_live = torch.zeros(1, dtype=torch.int32, device=dev)
            xchk = [torch.empty_like(o) for o in xout]

            def skip_pass(outs):
                for a, o in zip(xin, outs):
                    inet.sdnn_forward_skip_dead(a, o, check_every=args.check_every, n_live=n_live)

            skip_pass(xchk)
            same = all(torch.equal(a, b) for a, b in zip(xout, xchk))
            live_end = 0
            for a, o in zip(xin, xchk):
                inet.sdnn_forward_skip_dead(a, o, check_every=args.check_every, n_live=n_live)
                live_end += int(n_live.item())
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(k):
                skip_pass(xchk)
            torch.cuda.synchronize()
            sms = (time.perf_counter() - t0) * 1e3 / k
            infer["skip_dead"] = {"edges_per_s": nnz_total * Bi / (sms * 1e-3), "ms": round(sms, 3),
                                  "check_every": args.check_every, "live_samples_at_last_check": live_end,
                                  "identical_to_plain_forward": bool(same)}
        inet.close()
        del inet

    # ---- the oracle on the host cores, as a baseline ----------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle.sdnn_oracle import Oracle, mse_dloss, softmax_ce_dloss
        orc = Oracle(np.float32)
        if work.loss == "mse":
            dfn = lambda x: mse_dloss(x, work.targets)
        else:
            dfn = lambda x: softmax_ce_dloss(x, work.labels, work.n_classes)
        # bounded sample: a depth prefix worth about 3e10 edge visits (10-30 s of CPU work)
        per_layer = 3.0 * (nnz_total / L) * Bt
        Ls = int(max(1, min(L, 3e10 // per_layer)))
        sub = work.layers[:Ls]
        if work.loss == "mse":
            dfn = lambda x: mse_dloss(x, work.targets)      # same shape: the net is square
        t0 = time.perf_counter()
        orc.train_step(sub, work.x_train, work.act_cap, dfn, work.lr)
        cs = time.perf_counter() - t0
        cpu = {"value": sum(l.nnz for l in sub) * Bt / cs, "unit": "edges/s", "cores": orc.threads(),
               "kind": "oracle",
               "sample": f"one training step on the first {Ls} of {L} layers, full minibatch {Bt} ({cs:.1f} s)"}
        # the same oracle on one thread, on a shorter depth prefix (about 1.5e9 edge visits)
        n_all = orc.threads()
        L1 = int(max(1, min(Ls, 1.5e9 // per_layer)))
        orc.set_threads(1)
        t0 = time.perf_counter()
        orc.train_step(work.layers[:L1], work.x_train, work.act_cap, dfn, work.lr)
        c1 = time.perf_counter() - t0
        orc.set_threads(n_all)
        cpu["single_thread"] = {"value": sum(l.nnz for l in work.layers[:L1]) * Bt / c1, "unit": "edges/s",
                                "sample": f"first {L1} layers ({c1:.1f} s)"}

    out = {
        "metric": "edges/s, forward+backward+SGD step (nnz x samples / time)",
        "value": train_eps, "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "step_ms_min": round(per_step[0], 4),
        "step_ms_median": round(per_step[len(per_step) // 2], 4), "edge_visits_per_s": 3.0 * train_eps,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"config {args.config}: N={N}, L={L}, 32 nnz/row" if args.config < 5
                   else f"config 5: N={N}, L={L}, heavy-tailed rows",
                   "train_batch": Bt, "infer_samples": Bi, "total_nnz": nnz_total,
                   "storage": "fp32", "accumulate": "fp64", "input_density": work.meta.get("density"), "active_fraction": active},
        "pass_ms": {"forward": round(fwd_ms, 4), "backward": round(bwd_ms, 4), "update": round(upd_ms, 4)},
        "inference": infer, "roofline": roofline, "cpu_baseline": cpu,
        "setup_s": {"generate": round(gen_s, 2)},
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
    net = sdnn.Net(work.layers, work.act_cap, 1, training=True, activation="sigmoid")
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


if __name__ == "__main__":
    main()
