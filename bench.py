#!/usr/bin/env python3
"""Benchmark: one K-FAC step for all 54 conv/fc layers of ResNet-50 at per-GPU batch 32 on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic activations / output gradients
already resident in HBM: 108 Kronecker-factor builds (bf16 inputs, fp32 accumulate), 108 running-average
updates, 108 damped inverses (fp32) and 54 preconditioning products (fp32).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 32] [--no-cpu-baseline]
  python bench.py --config cfg4     batch 128, gamma 1e-4, 20 steps, inverses refreshed at steps 0 and 10: amortised ms
  python bench.py --only-steps      warm-up and timed steps only (one launch shape per kernel: for counter runs)
  python bench.py --peaks           the machine's matrix-core and streaming peaks as the library's probes measure them

One GPU only: the per-GPU share of the paper's data-parallel step is what is measured; --gpus N>1 exits.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_1811_12019_amd import binding as kb        # noqa: E402
from paper_1811_12019_amd import step as kstep        # noqa: E402
from paper_1811_12019_amd import synth                # noqa: E402

PEAK = {"mfma_bf16": 2500.0, "mfma_f32": 157.3, "alu_f32": 157.3, "hbm": 8000.0}   # TFLOP/s, TFLOP/s, TFLOP/s, GB/s
# fp32 products computed as sums of 16-bit MFMAs over split operands: 6 MFMAs per fp32 product with both operands
# split into three bf16 pieces (the sweep's panel product), 3 with both split into two fp16 pieces of scaled operands
# (the sweep's rank-128 updates, both preconditioning products); fp16 and bf16 MFMA peaks are equal
PEAK["mfma_bf16x3"] = round(PEAK["mfma_bf16"] / 6, 1)
PEAK["mfma_f16x2"] = round(PEAK["mfma_bf16"] / 3, 1)


def kernel_work(net: kstep.KfacNetworkStep):
    """Algorithmic work of each kernel over ONE step of the whole network: (bound, peak, unit, amount)."""
    shapes = [l.shape for l in net.layers]
    dims = [d for s in shapes for d in (s.d_A, s.d_G)]

    def is_plain(s):
        return s.kh == 1 and s.kw == 1 and s.stride == 1 and s.pad == 0

    mfma_ok = [s for s in shapes if s.C_in % 8 == 0]
    fac_conv = sum(kstep.factor_flops(s.R, s.d_A) for s in mfma_ok if not is_plain(s))
    fac_plain = (sum(kstep.factor_flops(s.R, s.d_A) for s in mfma_ok if is_plain(s)) +
                 sum(kstep.factor_flops(s.R, s.d_G) for s in shapes))
    w = {
        # all steps of all matrices in one kernel; a matrix's last step (short product, dense mirrored output) is a
        # small part of it; it also inverts the next step's pivot block (fp32 matrix cores) beside the update
        "inv_update_kernel": ("mfma", PEAK["mfma_f16x2"], "TFLOP/s",
                              sum(kstep.inverse_update_flops(d) + kstep.inverse_pivot_flops(d) - kstep.inverse_first_pivot_flops(d)
                                  for d in dims)),
        # latency-bound helpers of the sweep (one workgroup per matrix / per 128-row slab): first-block inverses of nb^3
        # flops (fp32 matrix cores), panel products of 2 d nb^2 (bf16 matrix cores, operands split three ways)
        "inv_pivot_kernel": ("mfma", PEAK["mfma_f32"], "TFLOP/s", sum(kstep.inverse_first_pivot_flops(d) for d in dims)),
        "inv_panel_kernel": ("mfma", PEAK["mfma_bf16x3"], "TFLOP/s", sum(kstep.inverse_panel_flops(d) for d in dims)),
        "gemm_nt_kernel": ("mfma", PEAK["mfma_f16x2"], "TFLOP/s", sum(kstep.precondition_flops(s.d_G, s.d_A) for s in shapes)),
        # the operands' piece planes: every element read (4 B) and written (2 x 2 B): the gradient by the preconditioning
        # call, the inverses by the inversion call (kfac_inverse_item.planes)
        "pre_split_kernel": ("hbm", PEAK["hbm"], "GB/s", sum(8.0 * s.d_G * s.d_A for s in shapes)),
        "inv_planes_kernel": ("hbm", PEAK["hbm"], "GB/s", sum(8.0 * d * d for d in dims)),
        "factor_generic_kernel": ("alu", PEAK["alu_f32"], "TFLOP/s",
                                  sum(kstep.factor_flops(s.R, s.d_A) for s in shapes if s.C_in % 8 != 0)),
        "factor_dma_kernel<conv>": ("mfma", PEAK["mfma_bf16"], "TFLOP/s", fac_conv),
        "factor_dma_kernel<plain>": ("mfma", PEAK["mfma_bf16"], "TFLOP/s", fac_plain),
        "kfac::ema_kernel": ("hbm", PEAK["hbm"], "GB/s", sum(12.0 * d * d for d in dims)),
        "kfac::ema_batched_kernel": ("hbm", PEAK["hbm"], "GB/s", sum(12.0 * d * d for d in dims)),
        "inv_init_kernel": ("hbm", PEAK["hbm"], "GB/s", sum(4.0 * d * (d + 1) for d in dims if d > kstep.INVERSE_BLOCK)),
    }
    return w


def factor_shape_roofline_ms(layers):
    """Ideal time of the factor stage: per factor the larger of its algorithmic flops at the bf16 matrix-core peak and
    its algorithmic bytes at the HBM peak (16-bit input tensor read once, not the unfolded matrix; the running average
    read and written, 8 bytes per element), summed over both factors of every layer."""
    total = 0.0
    for s in layers:
        for d, in_elems in ((s.d_A, s.N * s.C_in * s.H * s.W), (s.d_G, s.R * s.d_G)):
            t_mfma = kstep.factor_flops(s.R, d) / (PEAK["mfma_bf16"] * 1e12)
            t_hbm = (2.0 * in_elems + 8.0 * d * d) / (PEAK["hbm"] * 1e9)
            total += max(t_mfma, t_hbm)
    return total * 1e3


def measured_traffic(kernel: str, batch: int):
    """HBM bytes per launch of `kernel` as rocprofv3's FETCH_SIZE + WRITE_SIZE counters measured them on this
    workload (scaled by a copy kernel of known size); the figure is kept with the profile summaries.  None when no
    summary covers this kernel and batch size."""
    import re
    path = os.path.join(ROOT, "profiles", "hbm_traffic_resnet50_b32_step.md")
    if batch != 32 or not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\|\s*`?([^|`]+?)`?\s*\|.*\|\s*([0-9.]+)\s*\|\s*$", line)
        if m and m.group(1).strip() == kernel:
            return {"bytes_per_launch": float(m.group(2)), "source": "profiles/hbm_traffic_resnet50_b32_step.md"}
    return None


def timed_steps(net, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        net.step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def stage_times(net, reps=3):
    """Milliseconds per stage (HIP events on the launch stream), averaged over `reps` steps."""
    names = ["factors", "ema", "inverse", "precondition"]
    fns = [net.build_factors, net.update_running, net.invert, net.precondition]
    acc = dict.fromkeys(names, 0.0)
    for _ in range(reps):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(fns) + 1)]
        evs[0].record()
        for i, fn in enumerate(fns):
            fn()
            evs[i + 1].record()
        torch.cuda.synchronize()
        for i, n in enumerate(names):
            acc[n] += evs[i].elapsed_time(evs[i + 1]) / reps
    return acc


def packed_triangle_rates(net, reps=5):
    """Outside the step: the change rate of all 108 factors between two refreshes, packing them into upper triangles, and
    feeding the running averages from packed factors (the sender's and the owner's side of the symmetry-aware
    exchange), as HBM rates."""
    full = [t for l in net.layers for t in (l.A_new, l.G_new)]
    run = [t.clone() for l in net.layers for t in (l.A_run, l.G_run)]
    packed = [torch.empty(kb.packed_elems(t.shape[0]), device=t.device) for t in full]
    pack_batch, ema_batch = kb.PackBatch(full, packed), kb.PackBatch(run, packed)
    dims = [int(t.shape[0]) for t in full]
    diff_batch = kb.DiffBatch(full, run)
    w = [torch.randn_like(l.P) for l in net.layers]
    w_prev = [t.clone() for t in w]
    upd_batch = kb.UpdateBatch(w, w_prev, [l.P for l in net.layers])
    n_weights = sum(t.numel() for t in w)
    # Batch Normalization layers behind the 53 convolutions: normalised input and output gradient, bf16 NHWC
    bn_x, bn_g = [], []
    for l in net.layers:
        s = l.shape
        if s.kh * s.kw == 1 and s.H == 1:                # the fc layer has none
            continue
        x = torch.randn((s.N, s.H_out, s.W_out, s.C_out), device=l.P.device).to(torch.bfloat16)
        bn_x.append(x)
        bn_g.append((0.01 * torch.randn_like(x, dtype=torch.float32)).to(torch.bfloat16))
    bn_batch = kb.BnBatch(bn_x, bn_g, kb.KFAC_BF16, bn_x[0].device)

    res = {}
    for name, fn, nbytes in (
            ("bn_sample_grads_batched", lambda: kb.kfac_bn_sample_grads_batched(bn_batch), sum(4.0 * x.numel() for x in bn_x)),
            ("weight_update_batched", lambda: kb.kfac_weight_update_batched(upd_batch, 1e-3, 0.9), 28.0 * n_weights),
            ("factor_diff_batched", lambda: kb.kfac_factor_diff_batched(diff_batch), sum(8.0 * d * d for d in dims)),
            ("pack_upper_batched", lambda: kb.kfac_pack_upper_batched(pack_batch), sum(4.0 * d * (d + 1) for d in dims)),
            ("ema_packed_batched", lambda: kb.kfac_ema_packed_batched(ema_batch, 0.95),
             sum(4.0 * d * (d + 1) + 4.0 * d * d for d in dims))):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        rate = nbytes / (ms * 1e-3) / 1e9
        res[name] = {"ms": round(ms, 4), "bound": "hbm", "achieved": round(rate, 1), "peak": PEAK["hbm"], "unit": "GB/s",
                     "frac": round(rate / PEAK["hbm"], 4)}
    return res


def cpu_oracle_baseline(net):
    """The float64 oracle, as it stands, on the whole step once: all 54 layers, same inputs (copied back from the
    device), identity running averages.  Reported baseline only."""
    from oracle import kfac_oracle as ko
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    t_cpu = 0.0
    for l in net.layers:
        s = l.shape
        act = l.act.float().permute(0, 3, 1, 2).cpu().numpy()
        gout = l.gout.float().permute(0, 3, 1, 2).cpu().numpy()
        gw = l.gradW.cpu().numpy()
        t0 = time.perf_counter()
        ko.kfac_layer_step(act, gout, gw, np.eye(s.d_A), np.eye(s.d_G), kh=s.kh, kw=s.kw, stride=s.stride, pad=s.pad,
                           order=ko.ORDER_KH_KW_C, decay=net.decay, gamma=net.gamma)
        t_cpu += time.perf_counter() - t0
    return {"value": round(t_cpu * 1e3, 1), "unit": "ms/step", "cores": int(threads), "kind": "oracle",
            "sample": f"float64 numpy oracle, one whole step: all {len(net.layers)} layers of the same workload "
                      f"({t_cpu:.1f} s; host copies of the inputs not timed)"}


def peaks():
    """Matrix-core and streaming peaks of this GPU as the library's probes measure them (HIP events)."""
    out = torch.empty(2048 * 256, device="cuda")
    res = {}

    def timed(fn, reps=3):
        fn()
        best = 1e30
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record(); torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best

    iters = 20000
    for name, dt, flops in (("mfma_f32_32x32x2", kb.KFAC_F32, 4096), ("mfma_bf16_32x32x16", kb.KFAC_BF16, 32768),
                            ("mfma_f16_32x32x16", kb.KFAC_F16, 32768)):
        best = 0.0
        for wgs in (256, 512, 1024, 2048):
            ms = timed(lambda: kb.kfac_probe_mfma(dt, wgs, iters, out))
            best = max(best, wgs * 4.0 * iters * 4 * flops / ms / 1e9)
        res[name + "_tflops"] = round(best, 1)
    src = torch.ones(1 << 29, dtype=torch.float32, device="cuda")       # 2 GiB
    dst = torch.empty_like(src)
    sink = torch.zeros(1, device="cuda")
    nbytes = src.numel() * 4
    bc = br = 0.0
    for wgs in (1024, 4096, 16384):
        bc = max(bc, 2.0 * nbytes / timed(lambda: kb.kfac_probe_copy(src, dst, wgs)) / 1e6)
        br = max(br, 1.0 * nbytes / timed(lambda: kb.kfac_probe_read(src, sink, wgs)) / 1e6)
    res["copy_gbs_read_plus_write"] = round(bc, 1)
    res["read_gbs"] = round(br, 1)
    res["published"] = {"mfma_bf16_tflops": PEAK["mfma_bf16"], "mfma_f32_tflops": PEAK["mfma_f32"], "hbm_gbs": PEAK["hbm"]}
    return res


def run_cfg4(args):
    """configs[4]: batch 128, factors rebuilt and gradients preconditioned every step, inverses refreshed every 10th."""
    layers = synth.resnet50_layers(128)
    net = kstep.KfacNetworkStep(layers, dtype=kb.KFAC_BF16, order=kb.KFAC_ORDER_KH_KW_C, decay=0.95, gamma=1e-4, seed=0)
    for _ in range(max(1, args.warmup)):
        net.step(refresh_inverse=True)
    net.reset_running()
    torch.cuda.synchronize()
    steps, every = 20, 10
    t0 = time.perf_counter()
    for i in range(steps):
        net.step(refresh_inverse=(i % every == 0))
    torch.cuda.synchronize()
    total_ms = (time.perf_counter() - t0) * 1e3

    def avg(fn, reps):
        fn(); torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / reps

    fresh_ms = avg(lambda: net.step(refresh_inverse=True), 3)
    stale_ms = avg(lambda: net.step(refresh_inverse=False), 5)
    assert int(net.inverse_info().abs().max()) == 0
    fac_flops = sum(kstep.factor_flops(s.R, s.d_A) + kstep.factor_flops(s.R, s.d_G) for s in layers)
    print(json.dumps({
        "metric": "ResNet-50 K-FAC step ms/GPU @ batch 128, inverses every 10th step (amortised over 20 steps)",
        "value": round(total_ms / steps, 3), "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": round(total_ms / steps, 3), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": "resnet50_kfac_step_all54layers_batch128_inverse_every10", "per_gpu_batch": 128,
                   "layers": len(layers), "decay": 0.95, "gamma": 1e-4, "refresh_steps": [0, 10]},
        "step_with_refresh_ms": round(fresh_ms, 3), "stale_step_ms": round(stale_ms, 3),
        "factor_tflops_stale_step_bound": round(fac_flops / (stale_ms * 1e-3) / 1e12, 1)}))


# what each stage computes in (the whole path stores and accumulates in fp32)
DTYPE = ("bf16 factor inputs (exact products, f32 accumulate); f32 storage; inverse products on 16-bit matrix cores from "
         "f32 operands split into 3 bf16 (panel) / 2 scaled f16 (rank-128 updates) pieces; preconditioning products from "
         "2 f16 pieces of operands scaled per 128x128 block")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--config", default="cfg3", choices=["cfg3", "cfg4"])
    ap.add_argument("--only-steps", action="store_true")
    ap.add_argument("--peaks", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch three plain 1 GiB -> 1 GiB element-wise copies (torch.neg), for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the per-GPU K-FAC step on ONE GPU; this build has no multi-GPU path "
              f"(got --gpus {args.gpus}).", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists).", file=sys.stderr)
        sys.exit(3)
    kb.load_library()
    if args.peaks:
        print(json.dumps({"peaks": peaks()}))
        return
    if args.config == "cfg4":
        run_cfg4(args)
        return

    layers = synth.resnet50_layers(args.batch)
    net = kstep.KfacNetworkStep(layers, dtype=kb.KFAC_BF16, order=kb.KFAC_ORDER_KH_KW_C, decay=0.95, gamma=1e-3, seed=0)
    for _ in range(args.warmup):
        net.step()
    ms = timed_steps(net, args.steps)
    if args.only_steps:
        if args.calibrate_copy:
            src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
            dst = torch.empty_like(src)
            for _ in range(3):
                torch.neg(src, out=dst)
            torch.cuda.synchronize()
        print(json.dumps({"value": round(ms, 3), "unit": "ms", "steps": args.steps, "warmup": args.warmup,
                          "config": {"workload": f"resnet50_kfac_step_all54layers_batch{args.batch}"}}))
        return

    stages = stage_times(net)
    # per-kernel durations over `steps` more steps, HIP events around every launch on the launch stream
    # (the inversion groups run back to back here: kernels that share the GPU would stretch each other's events)
    net.overlap_inversions = False          # (also makes step() run stage after stage)
    kb.kfac_kernel_timing_enable(True)
    for _ in range(args.steps):
        net.step()
    torch.cuda.synchronize()
    report = kb.kfac_kernel_timing_report()
    kb.kfac_kernel_timing_enable(False)
    net.overlap_inversions = True
    infos = net.inverse_info().cpu()
    assert int(infos.abs().max()) == 0, "an inversion reported a non-positive-definite factor"

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.neg(src, out=dst)
        torch.cuda.synchronize()
        del src, dst

    work = kernel_work(net)
    per_kernel = {}
    for name, (tot_ms, n) in report.items():
        base = name if name in work else name.split("<")[0]
        e = {"ms_per_step": round(tot_ms / args.steps, 4), "launches_per_step": n / args.steps,
             "avg_launch_us": round(1e3 * tot_ms / n, 2)}
        if base in work:
            bound, peak, unit, amount = work[base]
            rate = amount / (tot_ms / args.steps * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9)
            e.update({"bound": bound, "achieved": round(rate, 2), "peak": peak, "unit": unit, "frac": round(rate / peak, 4)})
        per_kernel[name] = e
    dominant = max(report, key=lambda k: report[k][0])
    dom = per_kernel[dominant]
    traffic = measured_traffic(dominant, args.batch)
    traffic_bytes = traffic["bytes_per_launch"] if traffic else None
    roofline = {"kernel": dominant, "bound": dom.get("bound"), "achieved": dom.get("achieved"), "peak": dom.get("peak"),
                "unit": dom.get("unit"), "frac": dom.get("frac"), "traffic": traffic_bytes,
                "traffic_source": traffic["source"] if traffic else None,
                "avg_launch_us": dom["avg_launch_us"], "launches_per_step": dom["launches_per_step"]}

    fac_flops = sum(kstep.factor_flops(s.R, s.d_A) + kstep.factor_flops(s.R, s.d_G) for s in layers)
    fac_ideal_ms = factor_shape_roofline_ms(layers)
    out = {
        "metric": "ResNet-50 K-FAC step ms/GPU @ batch 32; factor TFLOP/s & % MFMA peak",
        "value": round(ms, 3), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 3), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": f"resnet50_kfac_step_all54layers_batch{args.batch}", "per_gpu_batch": args.batch,
                   "layers": len(layers), "decay": 0.95, "gamma": 1e-3, "inverse_every_step": True},
        # stages run one after the other for the whole network; the timed step() overlaps them (the long inversion
        # chains of the widest layers start first and everything else runs beside them), so value < their sum
        "stage_ms": {k: round(v, 3) for k, v in stages.items()},
        "schedule": f"{len(net.waves)} waves" if net.pipelined and net.waves else "stage by stage",
        "factor_tflops": round(fac_flops / (stages["factors"] * 1e-3) / 1e12, 2),
        "factor_frac_of_bf16_mfma_peak": round(fac_flops / (stages["factors"] * 1e-3) / 1e12 / PEAK["mfma_bf16"], 4),
        # many factors are bandwidth- rather than matrix-core-bound (narrow ones over many rows): the sum over all 108
        # of the larger of their two ideal times, against the stage
        "factor_shape_roofline_ms": round(fac_ideal_ms, 4),
        "factor_frac_of_shape_roofline": round(fac_ideal_ms / stages["factors"], 4),
        "roofline": roofline,
        "kernels": per_kernel,
    }
    out["next_rows"] = packed_triangle_rates(net)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_oracle_baseline(net)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
