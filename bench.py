#!/usr/bin/env python3
"""Benchmark of the LQ-SGD compressor on one MI355X.

A step is one whole iteration of the hot path (error-feedback add, both
power-iteration products, Gram-Schmidt, both quantised exchanges with the
on-device mean over W workers, reconstruction, residual update, and the plain
mean of the 1-D tensors) over one batch of synthetic gradients that is already
resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet18]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def sweep_bytes(kernel, w, ghat, eager, bf16=False):
    """Algorithmic HBM bytes of one launch of a streaming kernel: bytes per
    gradient element of one worker x elements (sweep 0: read G, read M/E, write M = 12 B; sweep 1: read M = 4 B;
    residual sweep: read M, write E = 8 B, plus G-hat once per layer = 4 B / W;
    with the residual deferred only the G-hat pass remains).  `ghat`: 0 = not
    written, 1 = stored, 2 = applied to the parameters (read w, write w)."""
    e1 = w.elements_per_worker
    e = w.workers * e1
    if kernel == "sweep0_add_project":
        return (10.0 if bf16 else 12.0) * e
    if kernel == "sweep1_back_project":
        return 4.0 * e
    if kernel == "sweep2_residual_ghat":
        return (8.0 * e if eager else 0.0) + 4.0 * e1 * ghat
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet18", choices=["fc_256x128", "small_cnn", "resnet18", "llm_stack", "sweep_8192"])
    ap.add_argument("--rank", type=int, default=None)
    ap.add_argument("--bits", type=int, default=None)
    ap.add_argument("--workers", type=int, default=None)
    ap.add_argument("--llm-layers", type=int, default=32)
    ap.add_argument("--no-ghat", action="store_true", help="do not write G-hat (state update only)")
    ap.add_argument("--eager", action="store_true",
                    help="apply the residual update at the end of every step (a third sweep) instead of "
                         "deferring it into the next step's first sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the benchmark, copy a 1 GiB tensor three times (a kernel of known HBM "
                         "traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--aggregate-first", action="store_true",
                    help="the PowerSGD order: exchange the raw P factors, orthonormalise the aggregate once")
    ap.add_argument("--bf16-grads", action="store_true",
                    help="hand the gradients over in bfloat16 (the first sweep then reads 10 instead of 12 bytes per element)")
    ap.add_argument("--update", type=float, default=None, metavar="ETA",
                    help="apply w <- w - ETA G-hat to synthetic parameters inside the step instead of storing G-hat")
    ap.add_argument("--no-cooperative-launch", action="store_true",
                    help="the Gram-Schmidt of tall factors takes its form of several ordinary launches instead of one "
                         "cooperative launch (for runs under rocprofv3, whose exit handler crashes after a cooperative launch)")
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph and time replays of it (for the small, launch-bound sets)")
    ap.add_argument("--rank-sweep", action="store_true",
                    help="after the main measurement, time every point of the rank / bit-width sweep on the "
                         "8192 x 8192 matrix (r in 1..32, b in 2, 4, 8, W = 16) and add the table to the JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (W simulated workers share it; "
              "no collectives are built) -- run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2506_17974_amd import binding as B
    from paper_2506_17974_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the compressor has no CPU path", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    mk = {"fc_256x128": wl.fc_256x128, "small_cnn": wl.small_cnn, "resnet18": wl.resnet18,
          "llm_stack": lambda: wl.llm_stack(args.llm_layers), "sweep_8192": wl.sweep_8192}[args.workload]
    w = mk()
    over = {}
    if args.rank is not None:
        over["rank"] = args.rank
    if args.bits is not None:
        over["bits"] = args.bits
    if args.workers is not None:
        over["workers"] = args.workers
    if over:
        w = wl.scaled(w, **over)
    L, V, W = len(w.layers), len(w.vectors), w.workers

    if args.calibration_copy:
        src = torch.ones(1 << 28, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- synthetic inputs, resident in HBM before anything is timed -----
    grads = []
    for k in range(W):
        row = [wl.device_gradient(w, 0, l, k) for l in range(L)]
        row += [torch.from_numpy(wl.vector_gradient(w, 0, v, k)).cuda() for v in range(V)]
        grads.append(row)
    if args.bf16_grads:
        grads = [[t.to(torch.bfloat16) for t in row] for row in grads]
    ghat = None
    if not args.no_ghat:
        ghat = [torch.empty(s, device="cuda") for s in w.layers] + [torch.empty(n, device="cuda") for n in w.vectors]
    side = torch.cuda.Stream() if args.graph else None      # a graph cannot be recorded on the default stream
    torch.cuda.synchronize()
    comp = B.Compressor(B.layer_list(w.layers, w.vectors), w.rank, w.bits, w.bits, W, w.alpha,
                        (B.FLAG_EAGER_RESIDUAL if args.eager else 0) |
                        (B.FLAG_AGGREGATE_FIRST if args.aggregate_first else 0) |
                        (B.FLAG_BF16_GRADIENTS if args.bf16_grads else 0) |
                        (B.FLAG_NO_COOPERATIVE_LAUNCH if args.no_cooperative_launch else 0),
                        stream=side.cuda_stream if side is not None else None)
    q0 = [wl.initial_q(w, l) for l in range(L)]
    for l in range(L):
        comp.set_q(l, q0[l])
    tab = comp.pointer_table(grads)
    import ctypes as C
    gt = None
    if ghat is not None:
        gt = (C.c_void_p * (L + V))()
        for i, t in enumerate(ghat):
            gt[i] = t.data_ptr()

    def run(n):
        if args.update is not None and gt is not None:
            for _ in range(n):       # `ghat` holds the parameters (whatever torch.empty left there), updated in place
                comp._check(B.lib().lqsgd_step_update(comp._h, tab, gt, args.update))
            return
        for _ in range(n):
            comp.step_raw(tab, gt)

    run(max(args.warmup, 2 if args.graph else 0))
    torch.cuda.synchronize()
    timed = run
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            run(1)
        torch.cuda.synchronize()

        def timed(n):
            for _ in range(n):
                graph.replay()
        timed(2)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    timed(args.steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    grad_bytes = w.gradient_bytes
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9

    ghat_mode = 0 if ghat is None else (2 if args.update is not None else 1)
    # ---- per-kernel durations: HIP events on the library's own stream ----
    roofline = None
    kernels = {}
    if not args.no_kernel_timing:
        comp.timing_enable(True)
        run(args.steps)
        ms, cnt = comp.timing_read()
        comp.timing_enable(False)
        elems = W * w.elements_per_worker
        for k in range(B.KERNEL_COUNT):
            if cnt[k]:
                # keyed by the stage of the iteration; "function" is the device function that served it
                # (template arguments included, as rocprofv3's kernel list names it)
                kernels[B.kernel_name(k)] = {"function": comp.launched_kernel(k), "avg_us": 1e3 * ms[k] / cnt[k],
                                             "launches": cnt[k]}
        dom = max((k for k in kernels), key=lambda n: kernels[n]["avg_us"])
        alg = sweep_bytes(dom, w, ghat_mode, args.eager, args.bf16_grads)
        if alg:
            achieved = alg / (kernels[dom]["avg_us"] * 1e-6) / 1e9
            traffic = _measured_traffic(dom, "%s_r%d_b%d_W%d" % (w.name, w.rank, w.bits, W))
            roofline = {"bound": "hbm", "kernel": kernels[dom]["function"], "stage": dom, "achieved": round(achieved, 1),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                        "traffic": traffic,
                        "traffic_source": ("rocprofv3 FETCH_SIZE + WRITE_SIZE counter runs committed under profiles/ "
                                           "(hbm_traffic.txt), not measured by this run") if traffic else None,
                        "algorithmic_bytes_per_launch": alg,
                        "avg_launch_us": round(kernels[dom]["avg_us"], 2)}
        for n, d in kernels.items():
            alg = sweep_bytes(n, w, ghat_mode, args.eager, args.bf16_grads)
            if alg:
                d["hbm_frac"] = round(alg / (d["avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
            d["avg_us"] = round(d["avg_us"], 2)

    # ---- the oracle on the host cores, same inputs, bounded sample -------
    cpu = None
    if not args.no_cpu_baseline:
        cpu = _cpu_baseline(w, grads, q0)

    step_bytes = sum(sweep_bytes(k, w, ghat_mode, args.eager, args.bf16_grads)
                     for k in ("sweep0_add_project", "sweep1_back_project", "sweep2_residual_ghat"))
    out = {
        "metric": "compressed gradient GB/s per LQ-SGD step (ResNet-18 set, r=4) and % HBM peak",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d matrices + %d vectors, %d elements/worker, r=%d, b=%d, W=%d, alpha=%g, %s gradients, G-hat %s, residual update %s"
                   % (w.name, L, V, w.elements_per_worker, w.rank, w.bits, W, w.alpha, w.dist,
                      ("applied to parameters (eta=%g)" % args.update) if (ghat is not None and args.update is not None)
                      else "written" if ghat is not None else "not written",
                      "at the end of each step" if args.eager else "fused into the next step's first sweep"),
                   "gradient_dtype": "bf16" if args.bf16_grads else "f32",
                   "launch": "replays of a HIP graph holding one step" if args.graph else "eager launches",
                   "order": "aggregate, then orthonormalise" if args.aggregate_first else "orthonormalise, then aggregate (Algorithm 1)",
                   "cooperative_launch": not args.no_cooperative_launch,
                   "rank": w.rank, "bits": w.bits, "workers": W, "gradient_bytes_per_step": grad_bytes},
        "step_algorithmic_bytes": step_bytes,
        "step_hbm_frac": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels,
        "wire_bytes_per_worker_step": comp.wire_bytes(),
        "matrix_cores": _matrix_cores(B, w, W),
        "paper_context": PAPER_CONTEXT,
    }
    comp.close()
    if args.rank_sweep:
        del grads, ghat
        torch.cuda.empty_cache()
        out["rank_sweep"] = _rank_sweep(B, wl, torch)
    print(json.dumps(out))


# Table 1 of the paper (the only timing it prints): whole-epoch figures on other hardware.
PAPER_CONTEXT = ("paper, Table 1: ResNet-18 / CIFAR-10, compression rank 1, 5 x RTX 4090 workers + 1 central node, "
                 "precision unstated: computing time per EPOCH (communication excluded) 2.5714 s LQ-SGD, 2.3359 s PowerSGD, "
                 "2.2937 s SGD; 3 / 14 / 3325 MB sent per epoch.  Context only: no per-step or per-kernel figure is published.")


def _matrix_cores(B, w, W):
    """Which sweeps of this configuration run on the matrix cores (decided by the rank pad)."""
    info = B.plan_query(B.layer_list(w.layers, w.vectors), w.rank, w.bits, w.bits, W, w.alpha)
    return {"rank_pad": int(info.rank_pad), "sweeps_0_and_2": bool(info.rank_pad >= 16), "sweep_1": bool(info.rank_pad >= 32)}


def _rank_sweep(B, wl, torch):
    """Every point of the rank / bit-width sweep on one 8192 x 8192 matrix, W = 16: step time, gradient
    GB/s, the fraction of the HBM peak the first sweep reaches (12 B per element), matrix-core use."""
    rows = []
    base = wl.sweep_8192()
    W = base.workers
    grads = [[wl.device_gradient(base, 0, 0, k)] for k in range(W)]
    ghat = [torch.empty(base.layers[0], device="cuda")]
    elems = W * base.elements_per_worker
    for r in (1, 2, 4, 8, 16, 32):
        for b in (2, 4, 8):
            w = wl.scaled(base, rank=r, bits=b)
            comp = B.Compressor(B.layer_list(w.layers, w.vectors), r, b, b, W, w.alpha)
            comp.set_q(0, wl.initial_q(w, 0))
            for _ in range(3):
                comp.step(grads, ghat)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                comp.step(grads, ghat)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / 20
            comp.timing_enable(True)
            for _ in range(5):
                comp.step(grads, ghat)
            tms, cnt = comp.timing_read()
            comp.timing_enable(False)
            a_us = 1e3 * tms[B.KERNEL_ADD_PROJECT] / max(1, cnt[B.KERNEL_ADD_PROJECT])
            mc = _matrix_cores(B, w, W)
            rows.append({"rank": r, "bits": b, "ms_per_step": round(ms, 4),
                         "gradient_GBps": round(4.0 * elems / (ms * 1e-3) / 1e9, 1),
                         "sweep0_us": round(a_us, 1), "sweep0_hbm_frac": round(12.0 * elems / (a_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                         "step_hbm_frac": round((16.0 * elems + 4.0 * base.elements_per_worker) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         "matrix_cores_sweeps_0_2": mc["sweeps_0_and_2"], "matrix_cores_sweep_1": mc["sweep_1"]})
            comp.close()
            print("rank_sweep r=%d b=%d: %.3f ms" % (r, b, ms), file=sys.stderr, flush=True)
    return rows


def _measured_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if one
    exists for this kernel and workload (a line `<kernel> <workload>_r<r>_b<b>_W<W> hbm_bytes_per_launch <number>`)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        with open(path) as fh:
            for line in fh:
                p = line.split()
                if len(p) == 4 and p[0] == kernel and p[1] == workload and p[2] == "hbm_bytes_per_launch":
                    return float(p[3])
    except OSError:
        pass
    return None


def _cpu_baseline(w, grads, q0):
    """The oracle as it stands, on the host cores, on a bounded sample of the
    same inputs: layers are taken in order until about 25 s have been spent."""
    import numpy as np
    import oracle.lqsgd_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    L, W = len(w.layers), w.workers
    budget_s = 25.0
    done_elems = 0
    done_layers = 0
    t_spent = 0.0
    order = sorted(range(L), key=lambda l: w.layers[l][0] * w.layers[l][1])
    host = {}
    passes = 0
    # whole passes over the layer set are repeated until about 10 s have been spent (a small set
    # takes well under a second per pass); a large set stops inside its first pass at the budget
    while t_spent < 10.0 and passes < 50:
        stopped = False
        for n, l in enumerate(order):
            if l not in host:
                host[l] = [grads[k][l].float().cpu().numpy() for k in range(W)]
            G = host[l]
            E = [np.zeros(w.layers[l], np.float32) for _ in range(W)]
            t0 = time.perf_counter()
            orc.layer_step(G, E, q0[l], w.rank, w.bits, w.bits, w.alpha)
            t_spent += time.perf_counter() - t0
            done_elems += W * w.layers[l][0] * w.layers[l][1]
            if passes == 0:
                done_layers += 1
            if t_spent > budget_s:
                stopped = True
                break
        passes += 1
        if stopped or done_layers < L:
            break
    return {"value": round(4.0 * done_elems / t_spent / 1e9, 4), "unit": "GB/s", "cores": int(threads),
            "kind": "oracle",
            "sample": "%d of %d layers (smallest first), all %d workers, %d pass(es) of one step: %d gradient elements in %.1f s"
                      % (done_layers, L, W, passes, done_elems, t_spent)}


if __name__ == "__main__":
    main()
