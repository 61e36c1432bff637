#!/usr/bin/env python3
"""Benchmark of the integer linear-layer step (scale -> map -> int8 GEMM x3 -> inverse map)
on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5]

A "step" is one forward + backward pass of every linear layer of the workload through
fxp_linear_fwd / fxp_linear_bwd on synthetic inputs already resident in HBM.  Prints ONE
JSON line: whole-step throughput in TOPS (3 GEMMs x 2MNK integer ops per layer), a
`roofline` object for the kernel class that takes the most time (per-launch durations
measured with HIP events on the launching stream, same kernels and arguments as the
step), a `kernels` table for all classes, and `cpu_baseline`: the CPU oracle timed on a
bounded sample of the same workload on the host cores.  The default workload is the largest
configuration (c5, 8192^3, sigma 1): the one whose products are bound by the matrix cores and whose 268 MB
tensors are read from HBM, so the line's `targets` object carries the three rates the build's targets are
stated on (int8 MFMA fraction with the core clock the products ran at, map and scale HBM fractions).
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published
PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, published (5.0 POP/s)
RIDGE_OPS_PER_BYTE = PEAK_INT8_TOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
PEAK_CLOCK_MHZ = 2400.0      # the clock the published peaks are quoted at


def measured_ceilings():
    """(copy GB/s beyond the Infinity Cache, register-only int8 MFMA TOP/s) as profiles/ceilings.md records them for
    this machine's MI355X: the best streaming copy over the working sets of 1 GiB and more, and the MFMA loop.  (None,
    None) when the file is missing."""
    hbm, mfma = None, None
    try:
        with open(os.path.join(ROOT, "profiles", "ceilings.md")) as f:
            for line in f:
                w = line.split()
                if len(w) > 3 and w[0] == "hbm" and "best:" in w and int(w[1]) >= 1024:
                    v = float(w[w.index("copy") + 1])
                    hbm = v if hbm is None else max(hbm, v)
                elif len(w) > 3 and w[0] == "int8" and w[1] == "mfma" and w[-1] == "TOP/s":
                    mfma = float(w[-2])
    except (OSError, ValueError):
        pass
    return hbm, mfma


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c5", choices=["c1", "c2", "c3", "c4", "c5", "c2conv", "vitb_attn", "sgd16", "sgd16_multi"])
    ap.add_argument("--sigma", type=float, default=1.0, help="c5 only")
    ap.add_argument("--bits", type=int, default=8, help="width of the fixed-point values (8 = the paper's int8; 4..7 = its ablation)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--step-only", action="store_true",
                    help="time the steps and stop: no per-kernel section, no CPU baseline (for kernel-trace profiles, "
                         "where every traced launch is then a launch of the step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a 256 MiB elementwise copy (for scaling rocprofv3 byte counters)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def read_traffic(workload, kernel_class):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None.

    File format (profiles/layer_step_<workload>.txt): lines `traffic_bytes_per_launch <row> <bytes>`."""
    path = os.path.join(ROOT, "profiles", f"layer_step_{workload}.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel_class:
                    return float(parts[2])
    except OSError:
        pass
    return None


def read_step_traffic(name):
    """HBM bytes per whole step from profiles/<name>.txt (line `HBM bytes per step (...): <bytes>; ...`), or None."""
    try:
        with open(os.path.join(ROOT, "profiles", name + ".txt")) as f:
            for line in f:
                if line.startswith("HBM bytes per step"):
                    return float(line.split(":", 1)[1].split(";")[0])
    except (OSError, ValueError, IndexError):
        pass
    return None


def repeat_to_target(run_once, target_seconds, most=64):
    """Run the (whole-workload) CPU sample once; when that is far below the target time, repeat it.  Returns
    (repetitions, total seconds)."""
    first = run_once(0)
    reps = int(max(1, min(most, target_seconds / max(first, 1e-9))))
    if reps == 1:
        return 1, first
    total = 0.0
    for r in range(reps):
        total += run_once(r)
    return reps, total


def copy_calibration(torch, dev):
    """A plain elementwise copy of known size (256 MiB read, 256 MiB written, three launches) for scaling the
    FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this program."""
    src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()


def step_only_line(args, torch, dev, metric, unit, value, ms, dtype, workload):
    """--step-only: nothing but the steps has run (what a profiler should see); print the bare line and stop."""
    if args.copy_calibration:
        copy_calibration(torch, dev)
    print(json.dumps({"metric": metric, "value": round(value, 3), "unit": unit, "n_gpus": 1, "steps": args.steps,
                      "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
                      "vs_baseline": None, "dtype": dtype, "data": "synthetic", "config": {"workload": workload},
                      "roofline": None, "cpu_baseline": None}))


def bench_conv(args, torch, fxp, synth, dev):
    """The c2 layer given as a convolution (channels-last): map the activation once, int8 im2col, GEMMs,
    gather col2im.  Same integer work as c2 (3 x 2*M*K*Cout), far fewer fp32 bytes."""
    X, Wt, dY, g = synth.conv_tensors()
    buf = fxp.ConvBuffers(g["N"], g["H"], g["W"], g["C"], g["Cout"], g["KH"], g["KW"], g["stride"], g["pad"], device=dev)
    Xd, Wd, dYd = (torch.from_numpy(a).to(dev) for a in (X, Wt, dY))

    def step(i):
        fxp.conv2d_fwd(Xd, Wd, buf, seed=0, step=i, bits=args.bits)
        fxp.conv2d_bwd(dYd, buf, seed=0, step=i, bits=args.bits)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    M, K, Cout = g["N"] * buf.Ho * buf.Wo, g["KH"] * g["KW"] * g["C"], g["Cout"]
    ops = 3 * 2.0 * M * K * Cout
    if args.step_only:
        return step_only_line(args, torch, dev, "int8 fixed-point layer fwd+bwd TOPS", "TOPS", ops / (ms * 1e-3) / 1e12, ms,
                              "int8", "c2conv")
    nx, nw, ny = X.size, Wt.size, dY.size
    # algorithmic HBM bytes of every kernel of the step: scale + map of X (one
    # copy), W and dY (both copies); forward GEMM reading the image and the weights; transposed patches of X and the
    # weight flip; weight-gradient GEMM; input-gradient GEMM reading the gradient image and the flipped weights
    step_bytes = (4 * nx + 5 * nx) + (4 * nw + 6 * nw) + (nx + nw + 4 * ny) \
        + (4 * ny + 6 * ny) + (nx + M * K) + 2 * nw + (M * K + ny + 4 * nw) + (ny + nw + 4 * nx)
    gbs = step_bytes / (ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        def run(rows):
            t = time.perf_counter()
            _, sv = oracle.conv2d_fwd(X[:rows], Wt, g["stride"], g["pad"], 0, 0)
            oracle.conv2d_bwd(dY[:rows], sv, 0, 0)
            return time.perf_counter() - t

        per_image = run(1)      # one image first, to size the sample to about --cpu-seconds of CPU work
        rows = int(max(1, min(g["N"], args.cpu_seconds / max(per_image, 1e-9))))
        reps_cpu, dt = repeat_to_target(lambda r: run(rows), args.cpu_seconds) if rows == g["N"] else (1, run(rows))
        cpu = dict(value=round(ops * rows / g["N"] * reps_cpu / dt / 1e12, 6), unit="TOPS", cores=oracle.num_threads(), kind="oracle",
                   seconds=round(dt, 2), sample=f"first {rows} of {g['N']} images, fwd+bwd" + (f", {reps_cpu} times" if reps_cpu > 1 else ""))
    print(json.dumps({
        "metric": "int8 fixed-point layer fwd+bwd TOPS", "value": round(ops / (ms * 1e-3) / 1e12, 3), "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "c2conv: the c2 ResNet-18 3x3 convolution as a channels-last convolution layer "
                               f"N={g['N']} H=W={g['H']} C={g['C']} Cout={g['Cout']} (M={M} K={K})",
                   "pass": "scale+map X, W, dY; forward and input-gradient GEMMs read their patches from the int8 images; "
                           "transposed int8 patches + GEMM for the weight gradient",
                   "rounding": "stochastic (Philox-4x32-10)", "bits": args.bits},
        "roofline": dict(bound="hbm", achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                         frac=round(gbs / PEAK_HBM_GBS, 4), kernel="whole step (7 launches, all HBM- or launch-bound)",
                         algorithmic_per_launch=step_bytes, traffic=read_step_traffic("layer_step_c2conv")),
        "cpu_baseline": cpu,
    }))


def bench_attn(args, torch, fxp, synth, dev):
    """The two attention products of one ViT-B/16 block at batch 64 (768 heads, 197 tokens padded to 208, head
    width 64), forward + backward each: scores = Q K^T and context = P V as batched product layers."""
    t, g = synth.attention_tensors()
    b, S, d = g["batch"], g["S"], g["d"]
    qk = fxp.BmmBuffers(b, S, d, S, True, device=dev)
    pv = fxp.BmmBuffers(b, S, S, d, False, device=dev)
    td = {k: torch.from_numpy(v).to(dev) for k, v in t.items()}

    def step(i):
        fxp.bmm_fwd(td["Q"], td["K"], qk, seed=0, step=i, bits=args.bits)
        fxp.bmm_bwd(td["dS"], qk, seed=0, step=i, bits=args.bits)
        fxp.bmm_fwd(td["P"], td["V"], pv, seed=0, step=i, bits=args.bits)
        fxp.bmm_bwd(td["dO"], pv, seed=0, step=i, bits=args.bits)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ops = 2 * 3 * 2.0 * b * S * S * d
    nq, ns = b * S * d, b * S * S
    if args.step_only:
        return step_only_line(args, torch, dev, "int8 fixed-point layer fwd+bwd TOPS", "TOPS", ops / (ms * 1e-3) / 1e12, ms,
                              "int8", "vitb_attn")

    # the same steps with every tensor's previous scale as its (right) guess: one pass for scale + map
    def step_guess(i):
        fxp.bmm_fwd(td["Q"], td["K"], qk, seed=0, step=i, bits=args.bits, guess=True)
        fxp.bmm_bwd(td["dS"], qk, seed=0, step=i, bits=args.bits, guess=True)
        fxp.bmm_fwd(td["P"], td["V"], pv, seed=0, step=i, bits=args.bits, guess=True)
        fxp.bmm_bwd(td["dO"], pv, seed=0, step=i, bits=args.bits, guess=True)

    for i in range(args.warmup):
        step_guess(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step_guess(args.warmup + i)
    torch.cuda.synchronize()
    ms_guess = (time.perf_counter() - t0) * 1e3 / args.steps

    def layer_bytes(na, nb, ny):   # three tensors scaled + mapped to both orientations, three products
        return 10 * (na + nb + ny) + (na + nb + 4 * ny) + (ny + nb + 4 * na) + (na + ny + 4 * nb)

    step_bytes = layer_bytes(nq, nq, ns) + layer_bytes(ns, nq, nq)
    gbs = step_bytes / (ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        def run(nb):
            tt = time.perf_counter()
            _, sv = oracle.bmm_fwd(t["Q"][:nb], t["K"][:nb], True, 0, 0)
            oracle.bmm_bwd(t["dS"][:nb], sv, 0, 0)
            _, sv = oracle.bmm_fwd(t["P"][:nb], t["V"][:nb], False, 0, 0)
            oracle.bmm_bwd(t["dO"][:nb], sv, 0, 0)
            return time.perf_counter() - tt

        per_head = run(8) / 8   # a few heads first, to size the sample to about --cpu-seconds of CPU work
        nb = int(max(8, min(b, args.cpu_seconds / max(per_head, 1e-9))))
        reps_cpu, dt = repeat_to_target(lambda r: run(nb), args.cpu_seconds) if nb == b else (1, run(nb))
        cpu = dict(value=round(ops * nb / b * reps_cpu / dt / 1e12, 6), unit="TOPS", cores=oracle.num_threads(), kind="oracle",
                   seconds=round(dt, 2), sample=f"first {nb} of {b} heads, both products fwd+bwd" + (f", {reps_cpu} times" if reps_cpu > 1 else ""))
    print(json.dumps({
        "metric": "int8 fixed-point layer fwd+bwd TOPS", "value": round(ops / (ms * 1e-3) / 1e12, 3), "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"vitb_attn: attention products of one ViT-B/16 block, batch 64 x 12 heads = {b}, "
                               f"S={g['S_real']} padded to {S}, d={d}: Q K^T and P V, forward + backward",
                   "pass": "per product: scale+map 3 tensors (both orientations), 3 batched int8 GEMMs with fused inverse map",
                   "rounding": "stochastic (Philox-4x32-10)", "bits": args.bits},
        "with_scale_guesses": {"ms_per_step": round(ms_guess, 4), "value": round(ops / (ms_guess * 1e-3) / 1e12, 3),
                               "note": "fxp_bmm_fwd_guess / _bwd_guess, every guess right (same inputs every step)"},
        "roofline": dict(bound="hbm", achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                         frac=round(gbs / PEAK_HBM_GBS, 4), kernel="whole step (15 kernels, all HBM-bound)",
                         algorithmic_per_launch=step_bytes, traffic=read_step_traffic("layer_step_vitb_attn")),
        "cpu_baseline": cpu,
    }))


def bench_sgd(args, torch, fxp, synth, dev):
    """int16 SGD step (weight decay 5e-4, momentum 0.9: the paper's classification optimiser) on a flat
    parameter vector of ResNet-18's size."""
    n = synth.RESNET18_PARAMS
    w, g, v = synth.sgd_tensors(n)
    wd_, gd, vd = (torch.from_numpy(a).to(dev) for a in (w, g, v))
    buf = fxp.SgdBuffers(n, device=dev)

    def step(i):
        fxp.sgd16_step(wd_, gd, vd, buf, 0.1, 0.9, 5e-4, seed=0, step=i)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    if args.step_only:
        return step_only_line(args, torch, dev, "int16 SGD step (weight decay + momentum) G elements/s", "G elements/s",
                              n / (ms * 1e-3) / 1e9, ms, "int16", "sgd16")
    # scales of w, g, v (4 B each) + three lines of 8 B read, 4 B written
    step_bytes = 48 * n
    gbs = step_bytes / (ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        tt = time.perf_counter()
        oracle.sgd16_step(w, g, v, 0.1, 0.9, 5e-4, seed=0, step=0)
        one = time.perf_counter() - tt
        reps = int(max(1, min(400, args.cpu_seconds / max(one, 1e-9))))   # whole-vector steps, about --cpu-seconds
        tt = time.perf_counter()
        wc, vc = w, v
        for r in range(reps):
            wc, vc = oracle.sgd16_step(wc, g, vc, 0.1, 0.9, 5e-4, seed=0, step=r)
        dt = time.perf_counter() - tt
        cpu = dict(value=round(n * reps / dt / 1e9, 6), unit="G elements/s", cores=oracle.num_threads(), kind="oracle",
                   seconds=round(dt, 2), sample=f"{reps} consecutive steps on all {n} parameters")
    print(json.dumps({
        "metric": "int16 SGD step (weight decay + momentum) G elements/s", "value": round(n / (ms * 1e-3) / 1e9, 3),
        "unit": "G elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int16", "data": "synthetic",
        "config": {"workload": f"sgd16: flat parameter vector of ResNet-18's size, n={n}, lr 0.1, momentum 0.9, "
                               "weight decay 5e-4",
                   "pass": "3 scale reductions (w, g, v) + 3 fixed-point axpy lines (8 B read, 4 B written each)",
                   "rounding": "stochastic (Philox-4x32-10)", "bits": 16},
        "roofline": dict(bound="hbm", achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                         frac=round(gbs / PEAK_HBM_GBS, 4), kernel="whole step (3 x k_absmax_partials, 3 x k_axpy16)",
                         algorithmic_per_launch=step_bytes, traffic=read_step_traffic("sgd16_step")),
        "cpu_baseline": cpu,
    }))


def bench_sgd_multi(args, torch, fxp, synth, dev):
    """int16 SGD step over the 62 parameter tensors of a ResNet-18 (own scales per tensor) through the multi-tensor
    entry point; the same tensors through one fxp_sgd16_step call each are timed beside it."""
    ws, gs, vs = synth.sgd_tensor_list()
    wd_, gd, vd = ([torch.from_numpy(a).to(dev) for a in lst] for lst in (ws, gs, vs))
    buf = fxp.SgdMultiBuffers(wd_, gd, vd)
    n = sum(w.numel() for w in wd_)
    single = fxp.SgdBuffers(max(w.numel() for w in wd_), device=dev)

    def step(i):
        fxp.sgd16_step_multi(buf, 0.1, 0.9, 5e-4, seed=0, step=i)

    def step_per_tensor(i):
        for t in range(len(wd_)):
            fxp.sgd16_step(wd_[t], gd[t], vd[t], single, 0.1, 0.9, 5e-4, seed=0, step=(i << 16) | t)

    def run(fn, steps):
        for i in range(args.warmup):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(args.warmup + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms = run(step, args.steps)
    if args.step_only:
        return step_only_line(args, torch, dev, "int16 SGD step (weight decay + momentum) G elements/s", "G elements/s",
                              n / (ms * 1e-3) / 1e9, ms, "int16", "sgd16_multi")
    ms_loop = run(step_per_tensor, max(3, args.steps // 5))
    step_bytes = 48 * n
    gbs = step_bytes / (ms * 1e-3) / 1e9
    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        def once(r):
            tt = time.perf_counter()
            oracle.sgd16_step_multi(ws, gs, vs, 0.1, 0.9, 5e-4, seed=0, step=r)
            return time.perf_counter() - tt

        reps, dt = repeat_to_target(once, args.cpu_seconds, most=400)
        cpu = dict(value=round(n * reps / dt / 1e9, 6), unit="G elements/s", cores=oracle.num_threads(), kind="oracle",
                   seconds=round(dt, 2), sample=f"{reps} steps over all {len(ws)} tensors ({n} parameters)")
    print(json.dumps({
        "metric": "int16 SGD step (weight decay + momentum) G elements/s", "value": round(n / (ms * 1e-3) / 1e9, 3),
        "unit": "G elements/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int16", "data": "synthetic",
        "config": {"workload": f"sgd16_multi: the {len(ws)} parameter tensors of a ResNet-18 ({n} parameters), one scale "
                               "per tensor, lr 0.1, momentum 0.9, weight decay 5e-4",
                   "pass": "4 launches: block maxima of w, g, v of every tensor; 3 fixed-point axpy lines over every tensor",
                   "rounding": "stochastic (Philox-4x32-10)", "bits": 16},
        "ms_per_step_one_call_per_tensor": round(ms_loop, 4),
        "roofline": dict(bound="hbm", achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                         frac=round(gbs / PEAK_HBM_GBS, 4), kernel="whole step (k_absmax_multi, 3 x k_axpy16_multi)",
                         algorithmic_per_launch=step_bytes, traffic=None),
        "cpu_baseline": cpu,
    }))


def main():
    args = parse_args()
    world = int(os.environ.get("WORLD_SIZE", "1"))
    if args.gpus != 1 or world != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2207_08822_amd import fxp, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libfxp has no CPU path", file=sys.stderr)
        sys.exit(3)
    fxp.lib()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.workload == "c2conv":
        return bench_conv(args, torch, fxp, synth, dev)
    if args.workload == "vitb_attn":
        return bench_attn(args, torch, fxp, synth, dev)
    if args.workload == "sgd16":
        return bench_sgd(args, torch, fxp, synth, dev)
    if args.workload == "sgd16_multi":
        return bench_sgd_multi(args, torch, fxp, synth, dev)
    layers = synth.WORKLOADS[args.workload]
    host_inputs, dev_inputs, bufs = [], [], []
    for li, layer in enumerate(layers):
        X, W, dY = synth.layer_tensors(args.workload, li, sigma=args.sigma)
        host_inputs.append((X, W, dY))
        dev_inputs.append(tuple(torch.from_numpy(a).to(dev) for a in (X, W, dY)))
        bufs.append(fxp.LayerBuffers(layer.M, layer.K, layer.N, device=dev))
    seed = 0

    def step(i):
        for (X, W, dY), buf in zip(dev_inputs, bufs):
            fxp.linear_fwd(X, W, buf, seed=seed, step=i, bits=args.bits)
            fxp.linear_bwd(dY, buf, seed=seed, step=i, bits=args.bits)

    # ------------------------------------------------------------------ whole step
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ops_per_step = sum(synth.ops_per_layer(l) for l in layers)
    tops = ops_per_step / (ms_per_step * 1e-3) / 1e12

    config = {"workload": f"{args.workload}: " + ", ".join(f"{l.name} M={l.M} K={l.K} N={l.N}" for l in layers)
              + (f", sigma={args.sigma}" if args.workload == "c5" else ""),
              "pass": "scale+map X,W,dY (int8, both orientations) + 3 int8 GEMMs with fused inverse map",
              "rounding": "stochastic (Philox-4x32-10)", "bits": args.bits}
    if args.step_only:
        if args.copy_calibration:
            copy_calibration(torch, dev)
        print(json.dumps({"metric": "int8 fixed-point layer fwd+bwd TOPS", "value": round(tops, 3), "unit": "TOPS", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
                          "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8",
                          "data": "synthetic", "config": config, "roofline": None, "cpu_baseline": None}))
        return

    # the same steps through fxp_linear_fwd_guess / _bwd_guess: every tensor's scale of the previous step is its guess
    # and, the inputs being the same every step, every guess is right - the best case of that path (one pass over
    # each large tensor instead of two); reported beside `value`, which stays the two-pass step
    def step_guess(i):
        for (X, W, dY), buf in zip(dev_inputs, bufs):
            fxp.linear_fwd(X, W, buf, seed=seed, step=i, bits=args.bits, guess=True)
            fxp.linear_bwd(dY, buf, seed=seed, step=i, bits=args.bits, guess=True)

    for i in range(args.warmup):
        step_guess(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step_guess(args.warmup + i)
    torch.cuda.synchronize()
    ms_guess = (time.perf_counter() - t0) * 1e3 / args.steps

    # ------------------------------------------------------------------ per-kernel durations
    # Same kernels, same arguments as the step, launched back to back on the current
    # stream between two HIP events (torch.cuda.Event on the current stream, which is the
    # stream the binding hands to the library).
    reps = max(5, min(args.steps, 50))

    def timed(fn):
        """Median over five batches of `reps` back-to-back launches (seconds per launch); the minimum is kept too."""
        fn()
        torch.cuda.synchronize()
        batch = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            e1.synchronize()
            batch.append(e0.elapsed_time(e1) * 1e-3 / reps)
        batch.sort()
        timed.last_min = batch[0]
        return batch[2]

    rows = {}   # kernel row -> totals over one step

    def add(row, kernel, dt, nbytes, ops=0.0, tmin=None):
        r = rows.setdefault(row, dict(kernel=kernel, t=0.0, tmin=0.0, launches=0, bytes=0.0, ops=0.0))
        r["t"] += dt; r["tmin"] += timed.last_min if tmin is None else tmin
        r["launches"] += 1; r["bytes"] += nbytes; r["ops"] += ops

    gemm_rows = []
    map_rotating_gbs = None
    lib, p = fxp.lib(), (lambda z: z.data_ptr())
    st = torch.cuda.current_stream().cuda_stream
    side = torch.cuda.Stream()                      # default priority; carries only the clock probe
    probe_out = torch.zeros(2, dtype=torch.int64, device=dev)

    def clock_during(fn, seconds_per_launch):
        """Core clock in MHz while `fn` is launched back to back: a one-wave probe on a second stream counts core
        cycles against the constant 100 MHz counter for about 1 ms (at least four launches) in the middle of a
        run of launches."""
        window_us = int(min(20000, max(1000, 4 * seconds_per_launch * 1e6)))
        n = int(window_us * 1e-6 / max(seconds_per_launch, 1e-7)) + 2
        for _ in range(max(2, n // 2)):
            fn()
        side.wait_stream(torch.cuda.current_stream())      # the probe starts when the lead-in launches are done
        lib.fxp_clock_probe(p(probe_out), window_us, side.cuda_stream)
        for _ in range(2 * n):
            fn()
        torch.cuda.synchronize()
        ticks, cycles = probe_out.cpu().tolist()
        return 100.0 * cycles / ticks if ticks > 0 else None
    for layer, (X, W, dY), buf in zip(layers, dev_inputs, bufs):
        M, K, N = layer.M, layer.K, layer.N
        # map: 4 B read + 1 B written per copy (both orientations) per element; launched as the step launches it:
        # activation and weight in one launch, the gradient in one of its own
        outs = [(torch.empty(t.shape, dtype=torch.int8, device=dev),
                 torch.empty((t.shape[1], t.shape[0]), dtype=torch.int8, device=dev)) for t in (X, W, dY)]
        dX_, dW_ = (fxp._desc(t, e, o[0], o[1], tag) for t, e, o, tag in ((X, buf.eX, outs[0], 0), (W, buf.eW, outs[1], 1)))
        t_map_xw = timed(lambda: lib.fxp_map2(ctypes.byref(dX_), ctypes.byref(dW_), seed, 0, args.bits, st))
        tmin_map_xw = timed.last_min
        add("map", "k_map_tile<true, *>", t_map_xw, 6.0 * (X.numel() + W.numel()))
        # scale: 4 B read per element.  The step launches the reduction (k_absmax_partials, activation and weight in
        # one launch) and the map kernel, which finishes the reduction, back to back: the row is the time of that
        # pair of launches minus the time of the map launch alone (the stand-alone fxp_scale would add a finishing
        # launch per tensor that the step does not have)
        ws2 = torch.empty(2 * max(256, fxp.workspace_bytes(fxp.OP_SCALE, 0)), dtype=torch.uint8, device=dev)
        t_pair = timed(lambda: lib.fxp_scale_map2(ctypes.byref(dX_), ctypes.byref(dW_), seed, 0, args.bits, p(ws2),
                                                  ws2.numel(), st))
        add("scale", "k_absmax_partials", max(t_pair - t_map_xw, 0.0), 4.0 * (X.numel() + W.numel()),
            tmin=max(timed.last_min - tmin_map_xw, 0.0))
        if layer is layers[0] and not args.copy_calibration:      # (counter runs keep to the launches of the step)
            # the same launch over a rotating set of inputs larger than the 256 MB Infinity Cache: every launch reads
            # its tensor from HBM ("rotating"); the row above re-reads one tensor ("warm", as inside a training step,
            # where the scale reduction has just read it)
            copies = max(2, -(-640 * 1024 * 1024 // (4 * X.numel())))
            Xs = [X] + [X.clone() for _ in range(copies - 1)]
            descs = [fxp._desc(x, buf.eX, outs[0][0], outs[0][1], 0) for x in Xs]
            turn = [0]

            def rotating():
                turn[0] = (turn[0] + 1) % copies
                lib.fxp_map2(ctypes.byref(descs[turn[0]]), ctypes.byref(dW_), seed, 0, args.bits, st)

            map_rotating_gbs = 6.0 * (X.numel() + W.numel()) / timed(rotating) / 1e9
            del Xs, descs
        t_map_g = timed(lambda: lib.fxp_map(p(dY), dY.shape[0], dY.shape[1], p(buf.e_dY), p(outs[2][0]), p(outs[2][1]), seed, 2,
                                            0, args.bits, st))
        tmin_map_g = timed.last_min
        add("map", "k_map_tile<true, *>", t_map_g, 6.0 * dY.numel())
        t_pair = timed(lambda: lib.fxp_scale_map(p(dY), dY.shape[0], dY.shape[1], p(buf.e_dY), p(outs[2][0]), p(outs[2][1]),
                                                 seed, 2, 0, args.bits, p(ws2), ws2.numel(), st))
        add("scale", "k_absmax_partials", max(t_pair - t_map_g, 0.0), 4.0 * dY.numel(), tmin=max(timed.last_min - tmin_map_g, 0.0))
        del outs, ws2
        gemms = [("fwd", M, N, K, buf.Xq, buf.WqT, buf.eX, buf.eW, buf.Y),
                 ("dX", M, K, N, buf.dYq, buf.Wq, buf.e_dY, buf.eW, buf.dX),
                 ("dW", K, N, M, buf.XqT, buf.dYqT, buf.eX, buf.e_dY, buf.dW)]
        for name, gm, gn, gk, A, B, eA, eB, C in gemms:
            gws = torch.empty(max(256, fxp.workspace_bytes(fxp.OP_GEMM, gm, gn, gk)), dtype=torch.uint8, device=dev)
            dt = timed(lambda: lib.fxp_gemm_unmap(0, 1, gm, gn, gk, p(A), gk, p(B), gk, p(eA), args.bits, p(eB), args.bits, p(C), gn,
                                                  p(gws), gws.numel(), st))
            ops, nbytes = 2.0 * gm * gn * gk, float(gm * gk + gn * gk + 4 * gm * gn)
            mfma_bound = ops / nbytes > RIDGE_OPS_PER_BYTE
            mhz = clock_during(lambda: lib.fxp_gemm_unmap(0, 1, gm, gn, gk, p(A), gk, p(B), gk, p(eA), args.bits, p(eB), args.bits,
                                                          p(C), gn, p(gws), gws.numel(), st), dt) if mfma_bound else None
            del gws
            t_roof = max(ops / (PEAK_INT8_TOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9))
            gemm_rows.append(dict(layer=layer.name, gemm=name, M=gm, N=gn, K=gk, us=round(dt * 1e6, 2),
                                  us_loop_min=round(timed.last_min * 1e6, 2),
                                  tops=round(ops / dt / 1e12, 1), gbs=round(nbytes / dt / 1e9, 1),
                                  bound="mfma" if mfma_bound else "hbm",
                                  frac_of_roofline=round(t_roof / dt, 3),
                                  core_clock_mhz=round(mhz, 0) if mhz else None))
            add("gemm_" + name, "k_gemm_nt*", dt, nbytes, ops)

    # ------------------------------------------------------------------ in-step durations
    # The same steps once more with the library's timeline on: HIP events on the launching stream at the entry of
    # each layer call and after each of its launches.  An interval is the duration of a launch where it really
    # runs - behind the kernel that precedes it in the step and with what that kernel left in the caches (the
    # reduction walks a tensor back to front so that the map, walking front to back, finds its head in the
    # Infinity Cache; a loop of map launches alone never sees that).  These are the durations the rows use.
    TL = {1: "scale", 2: "map", 3: "gemm_fwd", 4: "gemm_dW", 5: "gemm_dX", 6: "gemm_dW"}     # a stand-alone slice sum belongs to dW
    tl_steps = max(3, min(args.steps, 20))
    cap = tl_steps * len(layers) * 12 + 8
    us_buf, tag_buf, cnt = (ctypes.c_float * cap)(), (ctypes.c_int * cap)(), ctypes.c_int(0)
    step(args.warmup + args.steps)
    torch.cuda.synchronize()
    fxp._check(lib.fxp_timeline_begin(cap), "fxp_timeline_begin")
    for i in range(tl_steps):
        step(args.warmup + args.steps + 1 + i)
    fxp._check(lib.fxp_timeline_end(us_buf, tag_buf, cap, ctypes.byref(cnt)), "fxp_timeline_end")
    in_step = {}                 # (layer index, class) -> microseconds summed over tl_steps
    idle_us, entries = 0.0, 0    # the first interval starts at the first call's entry event: entries counts calls so far
    for k in range(cnt.value):
        tag, us = tag_buf[k], float(us_buf[k])
        if tag == 0:
            entries += 1
            idle_us += us
        else:
            li = (entries // 2) % len(layers)
            in_step[(li, TL[tag])] = in_step.get((li, TL[tag]), 0.0) + us
    launches = dict(scale=2, map=2, gemm_fwd=1, gemm_dW=1, gemm_dX=1)
    for row in rows:
        t = sum(v for (li, c), v in in_step.items() if c == row) / tl_steps * 1e-6
        rows[row]["t_loop"], rows[row]["t"] = rows[row]["t"], t
    for g, li in zip(gemm_rows, [i for i in range(len(layers)) for _ in range(3)]):
        t = in_step.get((li, "gemm_" + g["gemm"]), 0.0) / tl_steps
        ops, nbytes = 2.0 * g["M"] * g["N"] * g["K"], float(g["M"] * g["K"] + g["N"] * g["K"] + 4 * g["M"] * g["N"])
        g["us_loop"], g["us"] = g["us"], round(t, 2)
        g["tops"], g["gbs"] = round(ops / t / 1e6, 1), round(nbytes / t / 1e3, 1)
        g["frac_of_roofline"] = round(max(ops / (PEAK_INT8_TOPS * 1e6), nbytes / (PEAK_HBM_GBS * 1e3)) / t, 3)
    # core clock over whole steps (the probe runs beside about 5 ms of steps)
    n_probe = max(2, int(5.0 / max(ms_per_step, 1e-3)))
    for i in range(2):
        step(i)
    side.wait_stream(torch.cuda.current_stream())
    lib.fxp_clock_probe(p(probe_out), int(min(20000, max(1000, 0.8 * n_probe * ms_per_step * 1e3))), side.cuda_stream)
    for i in range(n_probe + 1):
        step(2 + i)
    torch.cuda.synchronize()
    ticks, cycles = probe_out.cpu().tolist()
    step_clock_mhz = 100.0 * cycles / ticks if ticks > 0 else None

    dominant = max(rows, key=lambda k: rows[k]["t"])
    c = rows[dominant]
    avg_launch = c["t"] / c["launches"]
    if c["ops"] and c["ops"] / c["bytes"] > RIDGE_OPS_PER_BYTE:
        achieved = c["ops"] / c["t"] / 1e12
        roofline = dict(bound="mfma", achieved=round(achieved, 2), peak=PEAK_INT8_TOPS, unit="TOP/s",
                        frac=round(achieved / PEAK_INT8_TOPS, 4))
    else:
        achieved = c["bytes"] / c["t"] / 1e9
        roofline = dict(bound="hbm", achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(achieved / PEAK_HBM_GBS, 4))
    meas_hbm, meas_mfma = measured_ceilings()
    ceiling = meas_mfma if roofline["bound"] == "mfma" else meas_hbm
    roofline["frac_of_measured_ceiling"] = round(achieved / ceiling, 4) if ceiling else None
    roofline["measured_ceiling"] = ceiling
    roofline.update(kernel=c["kernel"], row=dominant, launches_per_step=c["launches"],
                    avg_launch_us=round(avg_launch * 1e6, 2),
                    algorithmic_per_launch=(c["ops"] if roofline["bound"] == "mfma" else c["bytes"]) / c["launches"],
                    traffic=read_traffic(args.workload, dominant))
    kernels = {k: dict(kernel=v["kernel"], launches_per_step=v["launches"], us_per_step=round(v["t"] * 1e6, 2),
                       us_per_step_in_a_loop_of_its_own=round(v["t_loop"] * 1e6, 2),
                       gbs=round(v["bytes"] / v["t"] / 1e9, 1),
                       tops=(round(v["ops"] / v["t"] / 1e12, 1) if v["ops"] else None)) for k, v in rows.items()}

    # The rows the two targets are judged on: the MFMA-bound products against the published int8 peak (with the core
    # clock they ran at: the published peak is quoted at 2.4 GHz, and a compute-bound kernel on real operand bits
    # runs the board into its power limit), map and scale against the published HBM bandwidth.
    mfma_rows = [g for g in gemm_rows if g["bound"] == "mfma"]
    timing_note = ("in-step: HIP events between the launches of the layer calls (fxp_timeline_*), mean of "
                   f"{tl_steps} steps; core_clock_mhz: mean over the products' own back-to-back loops")
    targets = {
        "map_hbm": dict(gbs=kernels["map"]["gbs"], frac=round(kernels["map"]["gbs"] / PEAK_HBM_GBS, 4), target=0.70,
                        algorithmic_bytes_per_element=6, traffic=read_traffic(args.workload, "map")),
        "scale_hbm": dict(gbs=kernels["scale"]["gbs"], frac=round(kernels["scale"]["gbs"] / PEAK_HBM_GBS, 4), target=0.70,
                          algorithmic_bytes_per_element=4, traffic=read_traffic(args.workload, "scale")),
    }
    if mfma_rows:
        t_all = sum(g["us"] for g in mfma_rows) * 1e-6
        t_loop = sum(g["us_loop"] for g in mfma_rows) * 1e-6
        ops_all = sum(2.0 * g["M"] * g["N"] * g["K"] for g in mfma_rows)
        clocks = [g["core_clock_mhz"] for g in mfma_rows if g["core_clock_mhz"]]
        mhz = sum(clocks) / len(clocks) if clocks else None
        tops_all, tops_loop = ops_all / t_all / 1e12, ops_all / t_loop / 1e12
        targets["gemm_int8_mfma"] = dict(
            tops=round(tops_all, 1), frac=round(tops_all / PEAK_INT8_TOPS, 4), target=0.60, products=len(mfma_rows),
            # the products alone, launched back to back, and the core clock sampled beside that loop: the published
            # peak is 5.0 POP/s at 2.4 GHz, so the peak at the clock the board grants is 5.0 * clock / 2.4
            tops_in_a_loop_of_their_own=round(tops_loop, 1), core_clock_mhz=round(mhz, 0) if mhz else None,
            frac_at_measured_clock=round(tops_loop / (PEAK_INT8_TOPS * mhz / PEAK_CLOCK_MHZ), 4) if mhz else None)
    targets["timing"] = timing_note
    targets["core_clock_mhz_over_whole_steps"] = round(step_clock_mhz, 0) if step_clock_mhz else None
    targets["idle_us_per_step_between_layer_calls"] = round(idle_us / tl_steps, 2)

    if args.copy_calibration:
        copy_calibration(torch, dev)

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        X, W, dY = host_inputs[0]
        layer = layers[0]
        # a few rows first to size the sample to about --cpu-seconds of CPU work
        probe_rows = min(layer.M, 64)
        t = time.perf_counter()
        _, sv = oracle.linear_fwd(X[:probe_rows], W, seed=seed, step=0)
        oracle.linear_bwd(dY[:probe_rows], sv, seed=seed, step=0)
        per_row = (time.perf_counter() - t) / probe_rows
        rows = int(max(probe_rows, min(layer.M, args.cpu_seconds / max(per_row, 1e-9))))

        def run_once(r):
            t = time.perf_counter()
            _, sv = oracle.linear_fwd(X[:rows], W, seed=seed, step=r)
            oracle.linear_bwd(dY[:rows], sv, seed=seed, step=r)
            return time.perf_counter() - t

        # a layer the oracle finishes in well under the target time is simply repeated
        reps_cpu, dt = repeat_to_target(run_once, args.cpu_seconds) if rows == layer.M else (1, run_once(0))
        sample_ops = 3 * 2.0 * rows * layer.K * layer.N * reps_cpu
        cpu = dict(value=round(sample_ops / dt / 1e12, 6), unit="TOPS", cores=oracle.num_threads(), kind="oracle",
                   seconds=round(dt, 2),
                   sample=f"layer {layer.name}: first {rows} of {layer.M} rows of X and dY, full W; fwd+bwd"
                          + (f", {reps_cpu} times" if reps_cpu > 1 else ""))

    out = {
        "metric": "int8 fixed-point layer fwd+bwd TOPS",
        "value": round(tops, 3),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": config,
        "with_scale_guesses": {"ms_per_step": round(ms_guess, 4), "value": round(ops_per_step / (ms_guess * 1e-3) / 1e12, 3),
                               "note": "fxp_linear_fwd_guess / _bwd_guess, every guess right (same inputs every step): "
                                       "same outputs bit for bit, each large tensor read once for scale + map"},
        "targets": targets,
        "map_gbs": kernels["map"]["gbs"],
        "map_activation_weight_launch_gbs_rotating_inputs": round(map_rotating_gbs, 1) if map_rotating_gbs else None,
        "roofline": roofline,
        "kernels": kernels,
        "gemms": gemm_rows,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
