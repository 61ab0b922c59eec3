#!/usr/bin/env python3
"""Benchmark of the PowerSGD step on one MI355X.

A "step" is one psgd_step over one batch of synthetic gradients: error-feedback
add, P = M Q, orthogonalisation, Q = M^T P_hat, decompression and the new error
memory for every matrix of the model (plus the uncompressed vector tensors),
for W simulated workers.  Inputs are generated on the GPU before the timed
region (planted low rank + Gaussian noise in the model's tensor shapes) and a
ring of several gradient buffers is cycled so that the gradient is not simply
re-read from cache.

Prints ONE JSON line: gradient GB/s for the whole job, the HBM roofline of the
dominant kernel (duration measured here with HIP events on the library's
stream) and the CPU oracle's throughput on the host cores as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

# HBM bytes per launch of a kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by a
# copy kernel of known size (see profiles/); keyed by (workload, rank, workers, kernel).  None = not
# measured for that configuration.
METRIC = "PowerSGD step gradient GB/s + % HBM peak, ResNet18 shapes r=2"   # the headline metric and its workload

MEASURED_TRAFFIC = {
    # (workload, rank, workers, kernel slot of kernel_ms): FETCH_SIZE + WRITE_SIZE, scaled, bytes per launch
    ("resnet18", 2, 1, "k_resident"): 200345914,      # profiles/resident_resnet18_r2.md
    ("lstm", 4, 1, "k_ef_right"): 391825784,          # profiles/streaming_lstm_r4.md
    ("lstm", 4, 1, "k_left"): 132707849,
    ("lstm", 4, 1, "k_decomp"): 400357535,
    ("resnet18", 2, 16, "k_ef_right"): 2169938454,    # profiles/streaming_resnet18_w16_r2.md
    ("resnet18", 2, 16, "k_left"): 726187992,
    ("resnet18", 2, 16, "k_decomp"): 1479685687,
    ("resnet18", 2, 1, "k_ef_add_zero"): 178776239,   # profiles/baseline_random_*_resnet18_r2.md
}
# The 24-layer transformer-shaped set: the counter runs end in a crash of the profiler once the process holds
# several GB of device memory, so the counters were taken on the embedding + 4 layers (same kernels and tiles,
# profiles/transformer_4layers_bf16_r*_counters.md); here: measured traffic / algorithmic bytes of that subset,
# applied to the full set's algorithmic bytes.
TRANSFORMER_TRAFFIC_RATIO = {
    (4, "k_ef_right"): 3170481503 / 3043491840, (4, "k_left"): 1271433450 / 1217396736, (4, "k_decomp"): 3181641715 / 3043934208,
    (16, "k_ef_right"): 3183008586 / 3043491840, (16, "k_left"): 1285809725 / 1217396736, (16, "k_decomp"): 3207991556 / 3043934208,
    (32, "k_ef_right"): 3222822593 / 3043491840, (32, "k_left"): 1305035561 / 1217396736, (32, "k_decomp"): 3201981824 / 3043934208,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet18", choices=["tiny", "resnet18", "lstm", "transformer"])
    ap.add_argument("--layers", type=int, default=24, help="transformer workload: number of layers")
    ap.add_argument("--grad-dtype", default=None, choices=["f32", "bf16"], help="default: the workload's")
    ap.add_argument("--out-dtype", default=None, choices=["f32", "bf16"], help="default: same as the gradient")
    ap.add_argument("--rank", type=int, default=None)
    ap.add_argument("--workers", type=int, default=1)
    ap.add_argument("--grad-buffers", type=int, default=4, help="distinct gradient batches cycled through")
    ap.add_argument("--profile-steps", type=int, default=50, help="steps of the per-kernel HIP-event pass")
    ap.add_argument("--cold-steps", type=int, default=20,
                    help="steps of the cold-cache pass (caches flushed before each step, outside the timing)")
    ap.add_argument("--update", choices=["none", "fused", "separate"], default="none",
                    help="also apply the momentum / parameter update of Algorithm 2: fused into the step "
                         "(psgd_step_update) or as separate elementwise kernels after psgd_step")
    ap.add_argument("--iterations", type=int, default=1,
                    help="subspace iterations per step (psgd_compress, then psgd_iterate, then psgd_decompress)")
    ap.add_argument("--compressor", choices=["powersgd", "random_block", "random_k"], default="powersgd",
                    help="powersgd (the headline), or one of the linear baselines of Appendix G run in the same "
                         "error-feedback loop (their random draws are made before the timed region)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle timing")
    ap.add_argument("--tune", action="append", default=[], help="key=value planner tuning (experiments)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="also run a plain device copy of this many MiB five times (a kernel of known traffic "
                         "against which rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings are scaled)")
    return ap.parse_args()


def device_gradients(wl, lay, plan, workers, seed, torch, dev, dtype=None):
    """One flat [W][grad_stride] gradient batch generated on the GPU: planted low rank + noise."""
    s = plan.sizes
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    grad = torch.zeros(workers * s.grad_stride, dtype=dtype or torch.float32, device=dev)
    fac_gen = torch.Generator(device=dev)
    fac_gen.manual_seed(12345)
    sv = torch.tensor(np.asarray(wl.singular_values), dtype=torch.float32, device=dev)
    for t, shape in enumerate(wl.shapes):
        off = lay.flat_off[t]
        if len(shape) == 1:
            for w in range(workers):
                grad[w * s.grad_stride + off: w * s.grad_stride + off + shape[0]] = \
                    (wl.sigma * torch.randn(shape[0], generator=gen, device=dev)).to(grad.dtype)
            continue
        n, m = shape
        k = min(wl.planted_rank, n, m)
        U, _ = torch.linalg.qr(torch.randn(n, k, generator=fac_gen, device=dev))
        V, _ = torch.linalg.qr(torch.randn(m, k, generator=fac_gen, device=dev))
        base = (U * sv[:k]) @ V.T
        dens = wl.row_density.get(t)
        mask = None
        if dens is not None:
            mask = (torch.rand(n, 1, generator=gen, device=dev) < dens).to(torch.float32)
        for w in range(workers):
            g = base + wl.sigma * torch.randn(n, m, generator=gen, device=dev)
            if mask is not None:
                g = g * mask
            grad[w * s.grad_stride + off: w * s.grad_stride + off + n * m] = g.reshape(-1).to(grad.dtype)
    return grad


def cpu_baseline(wl, rank, workers, budget_s, compressor="powersgd"):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    from oracle import powersgd_oracle as O
    from paper_1905_13727_amd import workloads as WL
    if compressor != "powersgd":
        return cpu_baseline_sparse(wl, rank, workers, budget_s, compressor)
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    factors = WL.planted_factors(wl, 0)
    q = [None if x is None else x.astype(np.float64) for x in WL.initial_q(wl, rank, 0)]
    errs = [[None if len(s) == 1 else np.zeros(s) for s in wl.shapes] for _ in range(workers)]
    grads = [WL.gradients(wl, factors, 0, 0, w) for w in range(workers)]
    n_elems = sum(int(np.prod(s)) for s in wl.shapes)
    steps, spent = 0, 0.0
    while True:
        t0 = time.perf_counter()
        res = O.powersgd_step(grads, errs, q, rank)
        spent += time.perf_counter() - t0
        q, errs = res["Q"], res["err"]
        steps += 1
        if spent >= budget_s or steps >= 1000:
            break
    gbs = workers * n_elems * 4 / (spent / steps) / 1e9
    rec = {"value": round(gbs, 4), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
           "ms_per_step": round(1e3 * spent / steps, 3),
           "sample": "%d full steps of the %s workload (W=%d, r=%d), numpy fp64, same gradient each step"
                     % (steps, wl.name, workers, rank)}
    # the same with the numerical library held to one thread (a few steps, at most a fifth of the budget again)
    try:
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            n1, spent1 = 0, 0.0
            while True:
                t0 = time.perf_counter()
                res = O.powersgd_step(grads, errs, q, rank)
                spent1 += time.perf_counter() - t0
                q, errs = res["Q"], res["err"]
                n1 += 1
                if spent1 >= budget_s / 5 or n1 >= 10:
                    break
        rec["single_thread"] = {"value": round(workers * n_elems * 4 / (spent1 / n1) / 1e9, 4), "unit": "GB/s",
                                "ms_per_step": round(1e3 * spent1 / n1, 3), "steps": n1}
    except Exception:
        rec["single_thread"] = None
    return rec


def cpu_baseline_sparse(wl, rank, workers, budget_s, compressor):
    """The oracle's Random Block / Random K step on the same workload (numpy fp64; the draws are not timed)."""
    from oracle import powersgd_oracle as O
    from paper_1905_13727_amd import workloads as WL
    factors = WL.planted_factors(wl, 0)
    errs = [[None if len(s) == 1 else np.zeros(s) for s in wl.shapes] for _ in range(workers)]
    grads = [WL.gradients(wl, factors, 0, 0, w) for w in range(workers)]
    n_elems = sum(int(np.prod(s)) for s in wl.shapes)
    steps, spent = 0, 0.0
    while True:
        draw = WL.block_starts(wl, rank, 0, steps) if compressor == "random_block" else WL.random_indices(wl, rank, 0, steps)
        t0 = time.perf_counter()
        res = (O.random_block_step if compressor == "random_block" else O.random_k_step)(grads, errs, draw, rank)
        spent += time.perf_counter() - t0
        errs = res["err"]
        steps += 1
        if spent >= budget_s or steps >= 1000:
            break
    return {"value": round(workers * n_elems * 4 / (spent / steps) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "ms_per_step": round(1e3 * spent / steps, 3),
            "sample": "%d full %s steps of the %s workload (W=%d, r=%d), numpy fp64 elementwise (one thread), same "
                      "gradient each step, draws not timed" % (steps, compressor, wl.name, workers, rank)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (W simulated workers share it); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        return 2
    import torch
    from paper_1905_13727_amd import binding as B
    from paper_1905_13727_amd import workloads as WL
    from paper_1905_13727_amd.flat import FlatLayout

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    wl = WL.transformer(args.layers) if args.workload == "transformer" else WL.by_name(args.workload)
    rank = args.rank if args.rank is not None else (4 if args.workload in ("lstm", "transformer") else 2)
    W = args.workers
    gdt = args.grad_dtype or wl.grad_dtype
    odt = args.out_dtype or gdt
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16}
    plan = B.Plan(wl.shapes, rank, W, B.PSGD_BF16 if gdt == "bf16" else B.PSGD_F32,
                  B.PSGD_BF16 if odt == "bf16" else B.PSGD_F32)
    tune = {}
    for kv in args.tune:
        k, v = kv.split("=")
        plan.set_tuning(k, int(v))
        tune[k] = int(v)
    lay = FlatLayout(plan, wl.shapes)
    s = plan.sizes

    grads = [device_gradients(wl, lay, plan, W, 100 + i, torch, dev, tdt[gdt]) for i in range(args.grad_buffers)]
    err = torch.zeros(W * s.err_stride, dtype=torch.float32, device=dev)
    q0 = WL.initial_q(wl, rank, 0)
    q = torch.from_numpy(lay.pack_q(q0)).to(dev)
    p = torch.zeros(s.p_elems, dtype=torch.float32, device=dev)
    out = torch.zeros(s.out_elems, dtype=tdt[odt], device=dev)
    ws = torch.empty(s.workspace_bytes // 4 + 64, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream(dev)
    sh = stream.cuda_stream

    if args.update != "none":   # Algorithm 2's last two lines: momentum and parameter buffers shaped like `out`
        mom = torch.zeros(s.out_elems, dtype=torch.float32, device=dev)
        par = torch.randn(s.out_elems, dtype=torch.float32, device=dev)
        if args.update == "separate" and odt != "f32":
            print("bench.py: --update separate needs an f32 output", file=sys.stderr)
            return 2

    sparse = args.compressor != "powersgd"
    if sparse:
        if gdt != "f32" or odt != "f32" or args.update != "none" or args.iterations != 1:
            print("bench.py: the baselines run in fp32, without fused update or iterations", file=sys.stderr)
            return 2
        vals = torch.zeros(max(1, s.kept_elems), dtype=torch.float32, device=dev)
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        draws = []
        for _ in range(len(grads)):      # one draw per gradient batch, made before the timed region
            if args.compressor == "random_block":
                st = torch.zeros(len(wl.shapes), dtype=torch.int64, device=dev)
                for t, shp in enumerate(wl.shapes):
                    if len(shp) == 2:
                        st[t] = int(torch.randint(0, shp[0] * shp[1], (1,), generator=gen, device=dev))
                draws.append(st)
            else:
                ix = torch.zeros(max(1, s.kept_elems), dtype=torch.int64, device=dev)
                for t, shp in enumerate(wl.shapes):
                    if len(shp) == 2:
                        off, n = plan.kept(t)
                        ix[off: off + n] = torch.randperm(shp[0] * shp[1], generator=gen, device=dev)[:n]
                draws.append(ix)

    def step(i):
        if sparse:
            if args.compressor == "random_block":
                plan.random_block_step(grads[i % len(grads)], err, draws[i % len(draws)], vals, out, sh)
            else:
                plan.random_k_step(grads[i % len(grads)], err, draws[i % len(draws)], vals, out, sh)
            return
        if args.iterations > 1:   # Appendix G.7: several subspace iterations per step (on chip when the plan is resident)
            plan.step_iterations(grads[i % len(grads)], err, q, p, out, ws, args.iterations, sh)
            return
        if args.update == "fused":
            plan.step_update(grads[i % len(grads)], err, q, p, mom, par, 0.01, 0.9, ws, sh)
        else:
            plan.step(grads[i % len(grads)], err, q, p, out, ws, sh)
            if args.update == "separate":   # the same update as three elementwise torch kernels on Delta'
                mom.mul_(0.9).add_(out)
                par.add_(out + mom, alpha=-0.01)

    if args.copy_calibration > 0:
        n = args.copy_calibration * 1024 * 1024 // 4
        src = torch.randn(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)      # reads and writes args.copy_calibration MiB each
        torch.cuda.synchronize(dev)
        del src, dst

    for i in range(args.warmup):
        step(i)
    resident = plan.check(sh)     # synchronises; raises if a resident step ever timed out
    torch.cuda.synchronize(dev)
    # HIP events on the stream the kernels are launched on, around the whole timed region
    ev_begin, ev_end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev_begin.record(stream)
    for i in range(args.steps):
        step(i)
    ev_end.record(stream)
    torch.cuda.synchronize(dev)
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / args.steps
    event_ms_per_step = ev_begin.elapsed_time(ev_end) / args.steps
    plan.check(sh)

    # per-kernel durations: HIP events recorded by the library on its own stream
    plan.set_profiling(True)
    for i in range(args.profile_steps):
        step(i)
    kms, ksteps = plan.kernel_times()
    plan.set_profiling(False)
    kavg = {k: v / max(1, ksteps) for k, v in kms.items()}
    # A resident step is one launch, so the events around the timed region give that kernel's average launch
    # duration directly (back to back, as timed); the per-launch event pairs of the profiling pass add about 3 us
    # each and stay in `kernel_ms` for reference.  Multi-kernel steps keep the per-kernel pairs.
    if sparse:
        resident = False
    kavg_events = dict(kavg)
    if resident and args.update != "separate":
        kavg = {k: 0.0 for k in kavg}
        kavg["k_resident"] = event_ms_per_step
    elif args.update != "separate" and sum(kavg.values()) > 0:
        # Multi-kernel steps: the pass above waits for the stream after every step, so each of its event pairs also
        # holds the start-up of a kernel launched onto an idle GPU (the pairs add up to 10-40 % more than a step of
        # the timed region takes).  A kernel's launch duration over the timed region is therefore taken as the
        # region's time per step (events around the K back-to-back steps) times that kernel's share of the pairs.
        total = sum(kavg.values())
        kavg = {k: event_ms_per_step * v / total for k, v in kavg.items()}

    # Cold-cache passes: before every step (outside its timing) 1 GiB of other data is pushed through L2 and the
    # memory-side cache, so that gradients and error memory come from HBM as after a real backward pass.  Two
    # variants: the caches are left full of DIRTY foreign lines (a 1 GiB fill; the step's own traffic then also
    # pays for their write-back: the harsher figure, reported as `cold`), or of CLEAN ones (a read-only sum over
    # the same 1 GiB: `cold_clean`).
    cold_ms = cold_clean_ms = None
    if args.cold_steps > 0:
        flush = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev)
        flush.fill_(1.0)
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        for dirty in (True, False):
            ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.cold_steps)]
            ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(args.cold_steps)]
            for i in range(args.cold_steps):
                if dirty:
                    flush.fill_(float(i))
                else:
                    sink += flush.sum()
                ev0[i].record(stream)
                step(i)
                ev1[i].record(stream)
            torch.cuda.synchronize(dev)
            ts = sorted(a.elapsed_time(b) for a, b in zip(ev0, ev1))
            res = {"median": round(ts[len(ts) // 2], 4), "min": round(ts[0], 4)}
            if dirty:
                cold_ms = res
            else:
                cold_clean_ms = res
        del flush

    # the dominant kernel's duration in the cold pass: a resident step is that one kernel; a multi-kernel step
    # gets the per-kernel event pairs again, with the caches flushed before every step
    cold_kavg = None
    if cold_ms is not None and not (resident and args.update != "separate") and args.profile_steps > 0:
        flush = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev)
        plan.set_profiling(True)
        for i in range(args.cold_steps):
            flush.fill_(float(i))
            step(i)
        ckms, csteps = plan.kernel_times()
        plan.set_profiling(False)
        cold_kavg = {k: v / max(1, csteps) for k, v in ckms.items()}
        ctotal = sum(cold_kavg.values())
        if ctotal > 0:   # the same apportioning, of the cold pass's own time per step
            cold_kavg = {k: cold_ms["median"] * v / ctotal for k, v in cold_kavg.items()}
        del flush

    payload_mat = s.payload_elems - s.n_vec_elems
    L = s.n_vec_elems
    # algorithmic bytes per launch of each kernel (fp32): what the kernel itself has to move
    gsz, osz = (2 if gdt == "bf16" else 4), (2 if odt == "bf16" else 4)
    kernel_bytes = {
        "k_ef_right": payload_mat * W * (gsz + 8),                          # read g, read e, write M
        "k_left": payload_mat * W * 4,                                      # read M
        "k_decomp": payload_mat * (W * 8 + osz) + L * (W * gsz + osz),      # read M, write e', write Delta' once
        "k_resident": int(s.bytes_min),                           # read g, e; write e', Delta': each once
        "k_ef_add_zero": int(s.bytes_min),                        # baselines: read g, e; write M; write Delta' = 0 once
        "k_kept_entries": int(s.kept_elems) * (W * 8 + 8),        # read, write M at the kept entries; Delta', values
    }
    if args.update == "fused":   # Delta' is not stored; momentum and parameters are read and written instead
        extra = (payload_mat + L) * (16 - osz)
        kernel_bytes["k_resident"] += extra
        kernel_bytes["k_decomp"] += extra
    if args.iterations > 1:      # the library's event pairs then hold the last round, whose P = M Q only reads M
        kernel_bytes["k_ef_right"] = payload_mat * W * 4
    dom = max(kernel_bytes, key=lambda k: kavg.get(k, 0.0))
    achieved = kernel_bytes[dom] / (kavg[dom] * 1e-3) / 1e9 if kavg[dom] > 0 else 0.0
    grad_bytes = W * (payload_mat + L) * gsz
    value = grad_bytes / (ms_per_step * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC.get((wl.name, rank, W, dom))
    traffic_source = "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on this configuration (profiles/)" if traffic else None
    if wl.name.startswith("transformer") and gdt == "bf16" and odt == "bf16" and W == 1 and (rank, dom) in TRANSFORMER_TRAFFIC_RATIO:
        traffic = int(TRANSFORMER_TRAFFIC_RATIO[(rank, dom)] * kernel_bytes[dom])
        traffic_source = ("counters of the embedding + 4 layers subset (profiles/transformer_4layers_bf16_r%d_counters.md), "
                          "traffic / algorithmic bytes applied to this set" % rank)
    if (sparse and dom != "k_ef_add_zero") or (not sparse and dom == "k_ef_add_zero"):
        traffic = None
    compressor_label = {"powersgd": "PowerSGD", "random_block": "Random Block", "random_k": "Random K"}[args.compressor]
    if args.update != "none" or args.iterations != 1 or tune:
        traffic, traffic_source = None, None   # the counters were taken on the plain step with the planner's own choices
    if resident and args.update != "separate":
        cold_dom_ms = cold_ms["median"] if cold_ms else None
    else:
        cold_dom_ms = cold_kavg[dom] if cold_kavg and cold_kavg.get(dom, 0.0) > 0 else None
    achieved_cold = kernel_bytes[dom] / (cold_dom_ms * 1e-3) / 1e9 if cold_dom_ms else None

    rec = {
        "metric": METRIC if (wl.name, rank, W) == ("resnet18", 2, 1) and gdt == "f32" and odt == "f32" and not sparse
                  else "%s step gradient GB/s + %% HBM peak, %s shapes W=%d r=%d" % (compressor_label, wl.name, W, rank),
        "value": round(value, 3),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if gdt == "f32" else "f32 (bf16 gradients)",
        "data": "synthetic",
        "config": {"workload": "%s-shaped gradient set, W=%d simulated worker(s), rank %d, gradients %s, output %s"
                               % (wl.name, W, rank, gdt, odt),
                   "compressor": args.compressor,
                   "mode": "elementwise sweep + kept entries (two kernels)" if sparse else
                           "resident (one kernel, M kept in registers)" if resident else
                           ("matrix cores (one kernel per phase)" if plan.path() == "matrix cores"
                            else "streaming (one kernel per phase)"),
                   "matrices": int(s.n_matrices), "matrix_elems": int(payload_mat), "vector_elems": int(L),
                   "grad_buffers": len(grads), "update": args.update,
                   "iterations": args.iterations},
        # Byte models of the whole step over the timed (warm, back-to-back) steps.  min_model: every element of g, e
        # read once and of e', Delta' written once - what a resident step moves.  stream_model: the same plus the two
        # re-reads of M that the method's two global reductions force on kernels that cannot keep M on chip - what a
        # streaming or matrix-core step moves; a resident step does not move these bytes, so the model is not
        # reported for it.
        "min_model": {"bytes_per_step": int(s.bytes_min),
                      "GBps": round(s.bytes_min / (ms_per_step * 1e-3) / 1e9, 2),
                      "frac_of_hbm_peak": round(s.bytes_min / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "stream_model": None if (resident or sparse) else {
            "bytes_per_step": int(s.bytes_stream),
            "GBps": round(s.bytes_stream / (ms_per_step * 1e-3) / 1e9, 2),
            "frac_of_hbm_peak": round(s.bytes_stream / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        # cold: caches flushed before every step, outside the timing - gradients and error memory come from HBM as
        # they would after a real backward pass.  The primary regime; `value` and `roofline.frac` are the timed
        # region's (warm), the cold fractions stand beside them.
        "cold_ms_per_step": cold_ms,
        "cold_clean_ms_per_step": cold_clean_ms,
        "cold": None if not cold_ms else {
            "value": round(grad_bytes / (cold_ms["median"] * 1e-3) / 1e9, 3), "unit": "GB/s",
            "min_model_frac_of_hbm_peak": round(s.bytes_min / (cold_ms["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "stream_model_frac_of_hbm_peak": None if (resident or sparse) else
                round(s.bytes_stream / (cold_ms["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "event_ms_per_step": round(event_ms_per_step, 5),
        "kernel_ms": {k: round(v, 5) for k, v in kavg.items()},
        "kernel_ms_event_pairs": {k: round(v, 5) for k, v in kavg_events.items()},
        "cold_kernel_ms": None if not cold_kavg else {k: round(v, 5) for k, v in cold_kavg.items()},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                     "traffic_source": traffic_source,
                     "algorithmic_bytes_per_launch": int(kernel_bytes[dom]),
                     "avg_launch_ms": round(kavg[dom], 5),
                     "regime": "warm (the timed region: steps back to back)",
                     "achieved_cold": None if achieved_cold is None else round(achieved_cold, 2),
                     "frac_cold": None if achieved_cold is None else round(achieved_cold / HBM_PEAK_GBS, 4),
                     "avg_launch_ms_cold": None if cold_dom_ms is None else round(cold_dom_ms, 5),
                     "frac_cold_clean": None if not (resident and cold_clean_ms and args.update != "separate") else
                         round(kernel_bytes[dom] / (cold_clean_ms["median"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(wl, rank, W, args.cpu_seconds, args.compressor)
    print(json.dumps(rec), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
