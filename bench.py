#!/usr/bin/env python3
"""Benchmark: one K-FAC preconditioner step (factor update + eigendecomposition + preconditioning) over
the ResNet-50-shaped layer set (53 convs + FC, 224x224 inputs, per-GPU batch 32, fp32) on one MI355X.

A step = every layer: unfold -> A and G factor update folded into the running average; then the
eigendecomposition of all 108 factors; then the eigenbasis-preconditioned gradient of all 54 layers.
Inputs are seeded synthetic tensors resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_F32 = 157.3e12   # MI355X dense fp32 matrix FLOP/s
PEAK_MFMA_F16 = 2.5e15     # dense fp16 matrix FLOP/s
PEAK_VALU_F32 = 157.3e12   # fp32 vector FLOP/s (256 CUs x 128 lanes x 2 flops x 2.4 GHz)
PEAK_HBM = 8.0e12          # bytes/s

BOUNDS = {  # kernel class -> (bound, peak, unit, which work figure)
    "unfold": ("hbm", PEAK_HBM, "GB/s", "bytes"),
    "syrk": ("mfma", PEAK_MFMA_F32, "TFLOP/s", "flops"),
    "syrk_bf16": ("mfma", PEAK_MFMA_F16, "TFLOP/s", "flops"),   # bf16 and fp16 share the dense matrix peak
    "syrk_reduce": ("hbm", PEAK_HBM, "GB/s", "bytes"),
    "precond_gemm": ("mfma", PEAK_MFMA_F32, "TFLOP/s", "flops"),
    "precond_scale": ("hbm", PEAK_HBM, "GB/s", "bytes"),
    # three fp16 matrix products per algorithmic fp32 product: the issued rate against the fp16 peak
    "precond_gemm_split": ("mfma", PEAK_MFMA_F16 / 3.0, "TFLOP/s", "flops"),
    "eig_small": ("alu", PEAK_VALU_F32, "TFLOP/s", "flops"),
    "eig_pivot_solve": ("alu", PEAK_VALU_F32, "TFLOP/s", "flops"),
    # K = 64 contraction per pass over W and Q: 16 flop/byte, below the fp32 ridge of 19.7
    "eig_apply": ("hbm", PEAK_HBM, "GB/s", "bytes"),
    "eig_misc": ("hbm", PEAK_HBM, "GB/s", "bytes"),
    "eig_post_gemm": ("mfma", PEAK_MFMA_F32, "TFLOP/s", "flops"),
    "eig_copy": ("hbm", PEAK_HBM, "GB/s", "bytes"),
    # split-fp16 engine, three fp16 MFMA products per algorithmic fp32 product: 56 algorithmic flop/byte, i.e.
    # 168 issued fp16 flop/byte against an fp16 ridge of 312, so the HBM roof is the one that binds
    "eig_outer_cols": ("hbm", PEAK_HBM, "GB/s", "bytes"),
    "eig_outer_rows": ("hbm", PEAK_HBM, "GB/s", "bytes"),
}


def measured_traffic(kernel):
    """HBM bytes per launch of a kernel class on the default workload, from the committed counter summary
    (rocprofv3 FETCH_SIZE / WRITE_SIZE runs); None where no figure was taken."""
    path = os.path.join(ROOT, "profiles", "resnet50_step_hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel:
                return float(f[2])
    except OSError:
        pass
    return None


def distinct_shape_layers(wl):
    """First layer of every distinct shape of the set, with the number of layers of that shape."""
    first, count = {}, {}
    for i, l in enumerate(wl.layers):
        key = (l.c_in, l.c_out, l.k, l.stride, l.pad, l.h_in, l.fc)
        first.setdefault(key, i)
        count[key] = count.get(key, 0) + 1
    return [(first[k], count[k]) for k in first]


def cpu_baseline(wl_name):
    """The fp64 oracle, as it stands, timed on this host on the workload of `value`: one K-FAC step (unfold + both
    factors + both eigendecompositions + preconditioning) of one layer of every distinct shape of the set, each
    time multiplied by the number of layers of that shape (layers of one shape cost the oracle the same: its
    loops and its eigensolver's operation count depend on the sizes only)."""
    import oracle
    from paper_2007_00784_amd import synthetic as S
    wl = S.workload(wl_name)
    ph = {"factors": 0.0, "eig": 0.0, "precondition": 0.0}
    measured = 0.0
    picks = distinct_shape_layers(wl)
    for li, mult in picks:
        lay = wl.layers[li]
        t = S.layer_inputs(wl, li, update=0)
        R = wl.batch * lay.T
        t0 = time.perf_counter()
        if lay.fc:
            P, g = t["x"], t["g"]
        else:
            P = oracle.unfold(t["x"], lay.k, lay.k, lay.stride, lay.stride, lay.pad, lay.pad)
            g = t["g"].transpose(0, 2, 3, 1).reshape(R, lay.c_out)
        A = oracle.gram(P, 1, 1.0 / R)
        G = oracle.gram(g, 0, 1.0 / R)
        t1 = time.perf_counter()
        la, qa = oracle.eigh(A)
        lg, qg = oracle.eigh(G)
        t2 = time.perf_counter()
        oracle.precondition(qa, la, qg, lg, wl.damping, t["gradw"])
        t3 = time.perf_counter()
        ph["factors"] += mult * (t1 - t0) * 1e3
        ph["eig"] += mult * (t2 - t1) * 1e3
        ph["precondition"] += mult * (t3 - t2) * 1e3
        measured += (t3 - t0) * 1e3
        print("[bench] oracle: %s x%d in %.1f s" % (lay.name, mult, t3 - t0), file=sys.stderr, flush=True)
    return {
        "value": round(sum(ph.values()), 1), "unit": "ms", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "one K-FAC step of the whole set (%d layers), composed: one layer of each of the %d distinct shapes "
                  "timed once and multiplied by the number of layers of that shape; %.1f s of CPU work measured"
                  % (len(wl.layers), len(picks), measured / 1e3),
        "phases_ms": {k: round(v, 1) for k, v in ph.items()},
        "measured_ms": round(measured, 1),
    }


def gpu_same_sample_ms(wl, torch, KfacRunner):
    """The HIP path on exactly the layers the CPU baseline times, one of each distinct shape (one step, after one
    warm-up step): compare with cpu_baseline.measured_ms."""
    run = KfacRunner(wl, "cuda:0", n_updates=1, layers=[li for li, _ in distinct_shape_layers(wl)])
    for _ in range(2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run.update_factors(0, 0.0)
        run.eig(raise_on_noconv=False)
        run.precondition()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3
    run.close()
    return round(ms, 3)


def config_step_ms(name, torch, K, S, KfacRunner):
    """Step time of one of the other benchmark configurations, after two warm-up steps: one factor update folded
    into the running average + eigendecomposition of every factor + preconditioning of every gradient.  For the
    bf16 configuration the update-decoupled schedule over 200 iterations instead (factors every 10 iterations,
    eigendecompositions every 100 -- the second started from the eigenvectors of the first --, preconditioning
    every iteration), amortised per iteration."""
    wl = S.workload(name)
    run = KfacRunner(wl, "cuda:0", n_updates=2)
    run.update_factors(0, 0.0)
    out = {}
    if not wl.bf16:
        ms = []
        for it in range(5):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run.update_factors(1, wl.decay)
            info = run.eig(raise_on_noconv=False)
            run.precondition()
            torch.cuda.synchronize()
            ms.append((time.perf_counter() - t0) * 1e3)
        out = {"step_ms": round(min(ms[2:]), 3), "layers": len(wl.layers), "batch": wl.batch,
               "eig_converged": "%d/%d" % (sum(1 for (_, _, c) in info if c), len(info))}
    else:
        per_it = []
        for rep in range(2):      # the first pass is the warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            n_fac = n_eig = 0
            t_eig = 0.0
            for k in range(200):
                do_f, do_e = K.kfac_schedule_due(k, 10, 100)
                if do_f:
                    run.update_factors(n_fac % 2, wl.decay)
                    n_fac += 1
                if do_e:
                    te = time.perf_counter()
                    info = run.eig(raise_on_noconv=False, warm_start=n_eig > 0)
                    t_eig += time.perf_counter() - te
                    n_eig += 1
                run.precondition()
            torch.cuda.synchronize()
            per_it.append((time.perf_counter() - t0) * 1e3 / 200)
        out = {"ms_per_iteration_200": round(per_it[-1], 3), "layers": len(wl.layers), "batch": wl.batch,
               "eig_ms_total": round(t_eig * 1e3, 1), "factor_updates": n_fac, "eigendecompositions": n_eig,
               "eig_converged": "%d/%d" % (sum(1 for (_, _, c) in info if c), len(info))}
    run.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the measurements that are not part of `value` (warm start, decoupled schedule, split-fp16 "
                         "preconditioner): for short profiler runs")
    ap.add_argument("--eig-serial", action="store_true",
                    help="run the eigensolver's groups one after another on one stream, so that a profiler's kernel "
                         "durations are the kernels' own (as in the instrumented step); `value` is then NOT the "
                         "product's figure and the line says so in config.eig_serial")
    args = ap.parse_args()
    if args.eig_serial:
        os.environ["KFAC_EIG_SERIAL"] = "1"
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every GPU box here has one GPU); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2007_00784_amd import kfac as K
    from paper_2007_00784_amd import synthetic as S
    from paper_2007_00784_amd.runner import KfacRunner

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = S.workload(args.workload)
    t_setup = time.time()
    run = KfacRunner(wl, "cuda:0", n_updates=2)
    print("[bench] inputs generated and resident in %.1f s" % (time.time() - t_setup), file=sys.stderr, flush=True)
    # warm state: the first factor update has no history (decay 0)
    run.update_factors(0, 0.0)
    torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step(marks=None):
        run.restore_gradients()      # the backward pass's part: fresh gradients (inside the step, outside the phases)
        if marks is not None:
            marks[0].record()
        run.update_factors(1, wl.decay)
        if marks is not None:
            marks[1].record()
        run.eig(raise_on_noconv=False)
        if marks is not None:
            marks[2].record()
        run.precondition(restore=False)
        if marks is not None:
            marks[3].record()

    for i in range(args.warmup):
        step()
        torch.cuda.synchronize()
        print("[bench] warmup step %d done" % i, file=sys.stderr, flush=True)
    all_marks = [[ev() for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(all_marks[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    phases = {"factors": 0.0, "eig": 0.0, "precondition": 0.0}
    for m in all_marks:
        phases["factors"] += m[0].elapsed_time(m[1]) / args.steps
        phases["eig"] += m[1].elapsed_time(m[2]) / args.steps
        phases["precondition"] += m[2].elapsed_time(m[3]) / args.steps
    step_ms = sorted(m[0].elapsed_time(m[3]) for m in all_marks)
    info = run.eig_info
    sweeps = [s for (s, _, _) in info]
    nconv = sum(1 for (_, _, c) in info if c)

    # what a training loop would do from its second decomposition on: start from the previous eigenvectors
    # (two more steps, each folding another batch into the factors; not part of `value`)
    warm_ms = []
    for upd in (() if args.no_extras else (0, 1)):
        run.update_factors(upd, wl.decay)
        e0, e1 = ev(), ev()
        e0.record()
        run.eig(raise_on_noconv=False, warm_start=True)
        e1.record()
        torch.cuda.synchronize()
        warm_ms.append(e0.elapsed_time(e1))
    warm_sweeps = max(s for (s, _, _) in run.eig_info)
    if args.no_extras:
        warm_ms, warm_sweeps = [0.0], None

    # the eigendecomposition with every product on the fp32 matrix instructions (the default runs the rank-256 passes of
    # factors with d >= 2048 on split-fp16 products until it recomputes W = Q^T F Q in fp32): not part of `value`
    fp32_ms, fp32_sweeps = None, None
    if not args.no_extras:
        run.update_factors(1, wl.decay)
        ts_ = []
        for _ in range(2):
            e0, e1 = ev(), ev()
            e0.record()
            run.eig(raise_on_noconv=False, fp32_only=True)
            e1.record()
            torch.cuda.synchronize()
            ts_.append(e0.elapsed_time(e1))
        fp32_ms, fp32_sweeps = round(min(ts_), 3), max(s for (s, _, _) in run.eig_info)

    # the update-decoupled schedule (factors every 10 iterations, eigendecompositions every 100, preconditioning
    # every iteration) over 200 iterations, amortised; not part of `value`
    torch.cuda.synchronize()
    ts = time.perf_counter()
    n_fac = 0
    for k in range(0 if args.no_extras else 200):
        do_f, do_e = K.kfac_schedule_due(k, 10, 100)
        if do_f:
            run.update_factors(n_fac % 2, wl.decay)
            n_fac += 1
        if do_e:
            run.eig(raise_on_noconv=False)
        run.precondition()
    torch.cuda.synchronize()
    sched_ms = (time.perf_counter() - ts) * 1e3 / 200

    # the preconditioner with its GEMM chain on the split-fp16 engine (an option of the call; the default above is
    # what the workload's gradient type selects: fp32 chain for fp32 gradients), five calls, best
    split_ms = []
    for _ in range(1 if args.no_extras else 5):
        e0, e1 = ev(), ev()
        e0.record()
        run.precondition(split_f16=True)
        e1.record()
        torch.cuda.synchronize()
        split_ms.append(e0.elapsed_time(e1))

    # the paper's other method (Sec. II-C, Eq. (kfac-damped); Table I sets it against the eigendecomposition): damped
    # factors inverted by blocked Cholesky, gradients preconditioned by two plain products; not part of `value`
    inv_ms, invp_ms = None, None
    if not args.no_extras:
        ti, tp = [], []
        for _ in range(3):
            e0, e1, e2 = ev(), ev(), ev()
            run.restore_gradients()
            e0.record()
            run.invert_factors()
            e1.record()
            run.precondition_inverse(restore=False)
            e2.record()
            torch.cuda.synchronize()
            ti.append(e0.elapsed_time(e1))
            tp.append(e1.elapsed_time(e2))
        inv_ms, invp_ms = round(min(ti), 3), round(min(tp), 3)

    # one more, instrumented step: every kernel launch bracketed by hipEvents on the library's stream
    K.kfac_profile_begin(run.ctx)
    step()
    stats = K.kfac_profile_end(run.ctx)
    kernels = {}
    for name, st in stats.items():
        bound, peak, unit, which = BOUNDS[name]
        work = st[which]
        avg_ms = st["ms"] / max(st["launches"], 1)
        ach = work / (st["ms"] * 1e-3) if st["ms"] > 0 else 0.0
        kernels[name] = {"launches": st["launches"], "total_ms": round(st["ms"], 3), "avg_ms": round(avg_ms, 5),
                         "bound": bound, "achieved": round(ach / (1e9 if unit == "GB/s" else 1e12), 3),
                         "peak": peak / (1e9 if unit == "GB/s" else 1e12), "unit": unit,
                         "frac": round(ach / peak, 4)}
        if st["launches"] and st["bytes"] > 0:
            kernels[name]["algorithmic_bytes_per_launch"] = round(st["bytes"] / st["launches"])
        if st["ms"] > 0 and st["flops"] > 0:
            kernels[name]["algorithmic_tflops"] = round(st["flops"] / (st["ms"] * 1e-3) / 1e12, 3)
    dom = max(stats, key=lambda k: stats[k]["ms"])
    roofline = dict(kernels[dom])
    roofline["kernel"] = dom
    roofline["traffic"] = measured_traffic(dom) if args.workload == "resnet50" else None
    roofline["timing"] = ("hipEvents around every launch of the class, over one instrumented step in which the eigensolver's "
                          "groups run one after another on one stream (the kernel's own duration, no waiting behind other "
                          "streams); in the timed steps the groups overlap on four streams")
    roofline = {k: roofline[k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic",
                                         "launches", "avg_ms", "total_ms", "algorithmic_bytes_per_launch", "algorithmic_tflops",
                                         "timing") if k in roofline}
    w = run.work()
    peak_syrk = PEAK_MFMA_F16 if wl.bf16 else PEAK_MFMA_F32     # bf16 samples run on the bf16 matrix instructions
    derived = {
        "syrk_tflops": round(w["syrk_flops"] / (phases["factors"] * 1e-3) / 1e12, 2),
        "syrk_frac_of_mfma_peak": round(w["syrk_flops"] / (phases["factors"] * 1e-3) / peak_syrk, 4),
        "precondition_tflops": round(w["precond_flops"] / (phases["precondition"] * 1e-3) / 1e12, 2),
        "precondition_frac_of_mfma_peak": round(w["precond_flops"] / (phases["precondition"] * 1e-3) / PEAK_MFMA_F32, 4),
        "eig_sum_d3_per_s": round(w["sum_d3"] / (phases["eig"] * 1e-3), 1),
        "eig_sweeps_max": max(sweeps), "eig_converged": "%d/%d" % (nconv, len(info)),
        "eig_warm_start_ms": None if args.no_extras else round(min(warm_ms), 3), "eig_warm_start_sweeps_max": warm_sweeps,
        "eig_fp32_only_ms": fp32_ms, "eig_fp32_only_sweeps_max": fp32_sweeps,
        "decoupled_schedule_ms_per_iteration": None if args.no_extras else round(sched_ms, 3),
        "inverse_method_invert_factors_ms": inv_ms, "inverse_method_precondition_ms": invp_ms,
        "precondition_split_f16_ms": round(min(split_ms), 3),
        "precondition_split_f16_tflops": round(w["precond_flops"] / (min(split_ms) * 1e-3) / 1e12, 2),
    }
    out = {
        "metric": "kfac_step_ms", "value": round(ms_per_step, 3), "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if not wl.bf16 else "bf16",
        "data": "synthetic",
        "config": {"workload": "%s: %d layers, batch %d, %s; factor update + eig of %d factors + precondition"
                               % (wl.name, len(wl.layers), wl.batch, "bf16 in / fp32 factors" if wl.bf16 else "fp32",
                                  2 * len(wl.layers)),
                   "arithmetic": "factors, pivot solves, round applications, W = Q^T F Q, eigenvalues, preconditioner: fp32 "
                                 "(fp32 MFMA); rank-256 update passes of the eigensolver for factors with d >= 2048: "
                                 "split-fp16 MFMA (hi + lo halves, 3 products, fp32 accumulation), followed by a recomputation "
                                 "of W = Q^T F Q in fp32; derived.eig_fp32_only_ms is the same step's eigensolve with "
                                 "every product in fp32"},
        "phases_ms": {k: round(v, 3) for k, v in phases.items()},
        "step_ms_median": round(step_ms[len(step_ms) // 2], 3), "step_ms_min": round(step_ms[0], 3),
        "derived": derived,
        "roofline": roofline,
        "kernels": kernels,
    }
    if args.eig_serial:
        out["config"]["eig_serial"] = True      # profiling mode: the eigensolver's groups ran one after another
    run.close()
    if not args.no_extras and args.workload == "resnet50":
        # the other four benchmark configurations, each after two warm-up steps
        out["configs"] = {}
        for name in ("single_conv", "resnet32_cifar", "largest_factor", "resnet50_bf16"):
            out["configs"][name] = config_step_ms(name, torch, K, S, KfacRunner)
            print("[bench] config %s: %s" % (name, out["configs"][name]), file=sys.stderr, flush=True)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
        out["cpu_baseline"]["gpu_same_sample_ms"] = gpu_same_sample_ms(wl, torch, KfacRunner)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
