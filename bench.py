#!/usr/bin/env python3
"""Benchmark of the BPDQ per-layer quantization pass on one MI355X.

One "step" = the whole hot path for one layer: zero H, accumulate the calibration Hessian
over all tokens, damp + factor (U = chol(H^-1)), and the group/column sweep with lazy block
updates.  Inputs (W and all activation chunks) are resident in HBM before the timed region.
Prints ONE JSON line (metric = Mparams quantized/s).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_F32_TFLOPS = 157.3    # MI355X dense fp32 matrix peak
PEAK_MFMA_16BIT_TFLOPS = 2500.0  # MI355X dense bf16 / fp16 matrix peak
# 16-bit products a split kernel issues per fp32-accurate product
SPLIT_PRODUCTS = {"f16x2": 3, "bf16x3": 6}
KERNEL_NAMES = {"f16x2": "hess_syrk_f16x2_kernel", "bf16x3": "hess_syrk_bf16x3_kernel",
                "f32": "hess_syrk_f32_kernel"}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2_qwen7b_attn")
    ap.add_argument("--tokens-per-call", type=int, default=0,
                    help="tokens per bpdq_hessian_accumulate call (0 = all tokens in one call)")
    ap.add_argument("--hessian", choices=["f16x2", "bf16x3", "f32"], default="f16x2",
                    help="Hessian kernel: two fp16 halves per value (default, bpdq_hessian_accumulate), "
                         "three bf16 pieces, or the fp32 matrix cores")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB -> 1 GiB elementwise kernel (scale for HBM counters)")
    ap.add_argument("--phases-only", default="", help="comma list of hessian,prepare,quantize (profiling)")
    ap.add_argument("--ceilings", action="store_true",
                    help="measure the chip's own ceilings instead (register-only matrix-core loops, "
                         "streaming copy) and print them as one JSON line")
    ap.add_argument("--block-update", action="store_true",
                    help="measure the lazy block-update GEMM by itself (bpdq_block_update) at the five "
                         "layer shapes and several depths K, and print one JSON line")
    return ap.parse_args()


def block_update_probe():
    """W'[:, K:] -= E_blk U[0:K, K:] for the first block of a layer of every workload shape: the
    largest update of the layer, at the block depth the sweep uses (128) and at deeper ones."""
    import torch
    from paper_2602_04163_amd import binding as bq
    bq.load()
    dev = torch.device("cuda:0")
    res = {"unit": "TFLOP/s", "fp32_mfma_peak": PEAK_MFMA_F32_TFLOPS, "hbm_peak_GBps": 8000.0, "cases": []}
    for d_out, d_in in ((3584, 3584), (18944, 3584), (3584, 18944), (8192, 8192), (8192, 29568)):
        lde = (d_out + 63) // 64 * 64
        U = torch.randn((d_in, d_in), device=dev).triu_() * 0.05
        Wp = torch.randn((d_out, d_in), device=dev) * 0.02
        for Kd in (128, 256, 512, 1024):
            Et = torch.randn((Kd, lde), device=dev) * 0.01
            for _ in range(2):
                bq.bpdq_block_update(Et, U, 0, Wp, Kd, d_in)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
            for a, b in ev:
                a.record()
                bq.bpdq_block_update(Et, U, 0, Wp, Kd, d_in)
                b.record()
            torch.cuda.synchronize()
            ms = sorted(a.elapsed_time(b) for a, b in ev)[2]
            flops = 2.0 * d_out * Kd * (d_in - Kd)
            # compulsory traffic: the tail of W' read and written once, E_blk and the rows of U once
            nbytes = 8.0 * d_out * (d_in - Kd) + 4.0 * Kd * (d_in - Kd) + 4.0 * Kd * d_out
            res["cases"].append({"d_out": d_out, "d_in": d_in, "K": Kd, "us": round(ms * 1e3, 1),
                                 "tflops": round(flops / ms / 1e9, 1),
                                 "frac_of_fp32_mfma_peak": round(flops / ms / 1e9 / PEAK_MFMA_F32_TFLOPS, 3),
                                 "GBps_compulsory": round(nbytes / ms / 1e6, 1)})
        del U, Wp
    print(json.dumps(res), flush=True)


def ceilings():
    """Register-only loops of the matrix-core instructions the pass uses, on zero / one / normally
    distributed operand values, one or two wavefronts per SIMD, and a 1 GiB streaming copy: what
    this GPU sustains, next to the published peaks."""
    import torch
    from paper_2602_04163_amd import binding as bq
    bq.load()
    dev = torch.device("cuda:0")
    out = torch.empty(256 * 512, device=dev)
    peaks = {"f32": 157.3, "bf16": 2500.0, "f16": 2500.0, "f64": 78.6, "i8": 5000.0}
    iters = {"f32": 32000, "bf16": 64000, "f16": 64000, "f64": 16000, "i8": 64000}
    res = {"unit": "TFLOP/s", "mfma": [], "peaks": peaks}

    def timed(fn, reps=10):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev[reps // 2:])      # the later half: settled clocks
        return ms[len(ms) // 2]

    for kind in ("f32", "bf16", "f16", "f64", "i8"):
        for data in ("zeros", "ones", "normal"):
            for waves in (1, 2):
                flops = [0.0]

                def run():
                    flops[0] = bq.bpdq_probe_mfma(kind, data, waves, 256, iters[kind] // waves, out)
                ms = timed(run)
                tf = flops[0] / (ms * 1e-3) / 1e12
                res["mfma"].append({"kind": kind, "data": data, "waves_per_simd": waves,
                                    "ms": round(ms, 3), "tflops": round(tf, 1),
                                    "frac_of_peak": round(tf / peaks[kind], 3)})
    n = 1 << 28
    src = torch.randn(n, device=dev)
    dst = torch.empty_like(src)
    ms = timed(lambda: bq.bpdq_probe_copy(src, dst))
    res["copy"] = {"bytes_read": 4 * n, "bytes_written": 4 * n, "ms": round(ms, 3),
                   "GBps_read_plus_write": round(8 * n / (ms * 1e-3) / 1e9, 1), "hbm_peak_GBps": 8000.0}
    print(json.dumps(res), flush=True)


def cpu_baseline(wl, W_cpu, scales_cpu, n_tok_sub=65536, rows_sub=1024):
    """The oracle, as it stands, on a bounded sample of the same workload; its time is scaled
    linearly to the full layer (tokens for the Hessian, rows for the sweep)."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info
    from oracle import bpdq_oracle as orc
    from paper_2602_04163_amd import workloads as wk

    sub = wl.scaled(n_tok=n_tok_sub, chunk=min(wl.chunk, n_tok_sub))
    H = np.zeros((wl.d_in, wl.d_in))
    # time only the oracle's own work: the chunks are generated beforehand
    chunks = [wk.make_activation_chunk(sub, c, scales_cpu).numpy() for c in range(wk.n_chunks(sub))]
    t0 = time.perf_counter()
    for Xc in chunks:
        orc.hessian_accumulate(Xc, H)
    t_h = time.perf_counter() - t0
    t0 = time.perf_counter()
    U, dead, info = orc.prepare(H, wl.damp)
    t_p = time.perf_counter() - t0
    rows = min(rows_sub, wl.d_out)
    t0 = time.perf_counter()
    orc.quantize_layer(W_cpu[:rows].numpy(), U, dead, wl.bits, wl.group, wl.block,
                       wl.refine_iters, alpha=wl.alpha)
    t_q = time.perf_counter() - t0
    t_full = t_h * (wl.n_tok / n_tok_sub) + t_p + t_q * (wl.d_out / rows)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [torch.get_num_threads()])
    return {
        "value": wl.params / t_full / 1e6, "unit": "Mparams/s", "cores": int(threads),
        "kind": "oracle",
        "sample": (f"numpy fp64 oracle: Hessian on {n_tok_sub} of {wl.n_tok} tokens ({t_h:.2f} s, "
                   f"scaled x{wl.n_tok / n_tok_sub:.0f}), prepare at full size ({t_p:.2f} s), sweep on "
                   f"{rows} of {wl.d_out} rows ({t_q:.2f} s, scaled x{wl.d_out / rows:.0f}); "
                   f"extrapolated full layer {t_full:.1f} s"),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_04163_amd import binding as bq
    from paper_2602_04163_amd import workloads as wk

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.ceilings:
        ceilings()
        return
    if args.block_update:
        block_update_probe()
        return
    bq.load()
    dev = torch.device("cuda:0")
    wl = wk.WORKLOADS[args.workload]
    d_out, d_in, n_tok = wl.d_out, wl.d_in, wl.n_tok

    # ---- inputs, resident in HBM --------------------------------------------------------
    W = wk.make_weight(wl, device=dev)
    scales = wk.channel_scales(wl, device=dev)
    X = torch.empty((n_tok, d_in), device=dev, dtype=torch.float32)
    for c in range(wk.n_chunks(wl)):
        wk.make_activation_chunk(wl, c, scales, device=dev, out=X[c * wl.chunk:(c + 1) * wl.chunk])
    per_call = args.tokens_per_call if args.tokens_per_call > 0 else n_tok
    calls = [(a, min(a + per_call, n_tok)) for a in range(0, n_tok, per_call)]

    # ---- outputs and workspaces, allocated once -----------------------------------------
    H = torch.zeros((d_in, d_in), device=dev)
    U = torch.empty((d_in, d_in), device=dev)
    p = bq.make_params(wl.bits, wl.group, wl.block, wl.refine_iters, wl.alpha)
    ws_h = torch.empty(max(256, max(bq.bpdq_hessian_workspace_bytes(b - a, d_in) for a, b in calls)),
                       dtype=torch.uint8, device=dev)
    ws_p = torch.empty(bq.bpdq_prepare_workspace_bytes(d_in), dtype=torch.uint8, device=dev)
    ws_q = torch.empty(bq.bpdq_quantize_workspace_bytes(d_out, d_in, p), dtype=torch.uint8, device=dev)
    out = None
    infos = []
    phases = [s for s in args.phases_only.split(",") if s] or ["hessian", "prepare", "quantize"]
    ev = {k: [] for k in ("hessian", "prepare", "quantize")}
    # events the library records right around the Hessian tile-product kernel (the dominant kernel
    # of the step), on the stream it is launched on
    kern_ev = []

    def hessian_call(Xc, Hm, scale, symmetrize, ws, record):
        if not record:
            return bq.bpdq_hessian_accumulate_timed(args.hessian, Xc, Hm, scale, symmetrize, ws)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        b.record()              # created now; the library records them again at the kernel
        kern_ev.append((a, b))
        return bq.bpdq_hessian_accumulate_timed(args.hessian, Xc, Hm, scale, symmetrize, ws, a, b)

    def step(record):
        nonlocal out
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if record else None
        if record:
            marks[0].record()
        if "hessian" in phases:
            H.zero_()
            for a, b in calls:
                hessian_call(X[a:b], H, 2.0, False, ws_h, record)
        if record:
            marks[1].record()
        dead = None
        if "prepare" in phases:
            _, dead, info = bq.bpdq_prepare(H, wl.damp, U=U, ws=ws_p)
            infos.append(info)
        if record:
            marks[2].record()
        if "quantize" in phases:
            out = bq.bpdq_quantize_layer(W, U, dead, p, want_w_hat=True, ws=ws_q, out=out)
        if record:
            marks[3].record()
            ev["hessian"].append((marks[0], marks[1]))
            ev["prepare"].append((marks[1], marks[2]))
            ev["quantize"].append((marks[2], marks[3]))

    if "prepare" not in phases or "hessian" not in phases:
        # profiling a single phase still needs valid inputs for it
        saved = phases
        phases = ["hessian", "prepare", "quantize"]
        step(False)
        phases = saved
    if args.calibrate_copy:
        src = X.view(-1)[: (1 << 28)]                 # 2^28 floats = 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            bq.bpdq_probe_copy(src, dst)              # bpdq::probe_copy_kernel: the scale for the HBM counters
        del dst
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    phase_ms = {k: sum(a.elapsed_time(b) for a, b in v) / max(len(v), 1) for k, v in ev.items()}
    # outside the timed region: the factorisation of the last steps succeeded
    if infos and any(int(i.item()) != 0 for i in infos[-2:]):
        print("bench.py: bpdq_prepare reported a non-positive pivot", file=sys.stderr)
        sys.exit(1)
    kernel_ms = (sum(a.elapsed_time(b) for a, b in kern_ev) / len(kern_ev)) if kern_ev else 0.0

    # ---- roofline of the dominant kernel: the Hessian tile product -----------------------------
    # algorithmic flops: the symmetric half, d(d+1) multiply-adds' worth per token; duration: the
    # library's own events around that kernel (one launch per call here), measured in the timed steps
    flops_per_launch = float(d_in) * (d_in + 1) * (n_tok / len(calls))
    achieved = flops_per_launch / (kernel_ms * 1e-3) / 1e12 if kernel_ms > 0 else 0.0
    traffic = None
    kernel = KERNEL_NAMES[args.hessian]
    tp = os.path.join(ROOT, "profiles", f"{kernel[:-7]}_{args.workload}_traffic.json")   # from rocprofv3 --pmc runs
    if os.path.exists(tp) and len(calls) == 1:
        traffic = json.load(open(tp)).get("hbm_bytes_per_launch")
    if args.hessian in SPLIT_PRODUCTS:
        # `achieved` counts the fp32-accurate products of the update; the kernel issues n 16-bit
        # products for each, so its ceiling on that pipe is 1/n of the pipe's peak
        n = SPLIT_PRODUCTS[args.hessian]
        peak = PEAK_MFMA_16BIT_TFLOPS / n
        roof_extra = {"issued": achieved * n, "issued_peak": PEAK_MFMA_16BIT_TFLOPS,
                      "vs_fp32_mfma_peak": achieved / PEAK_MFMA_F32_TFLOPS,
                      "note": f"one fp32-accurate product = {n} {'fp16' if n == 3 else 'bf16'} MFMA products; "
                              f"peak = dense 16-bit matrix peak / {n}; duration = the tile-product kernel alone "
                              "(events recorded by the library around it); the phase time also holds the "
                              "split pre-pass and the reduction"}
        cp = os.path.join(ROOT, "profiles", "ceilings_mi355x.json")
        if os.path.exists(cp):
            c = json.load(open(cp)).get("f16_normal_tflops" if n == 3 else "bf16_normal_tflops")
            if c:
                roof_extra["measured_pipe_ceiling"] = c
                roof_extra["frac_of_measured_ceiling"] = achieved * n / c
    else:
        peak, roof_extra = PEAK_MFMA_F32_TFLOPS, {}
    res = {
        "metric": "Mparams quantized/s per layer (full pass: Hessian + prepare + sweep)",
        "value": wl.params / (ms_per_step * 1e-3) / 1e6,
        "unit": "Mparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f16x2": "f32 (Hessian products as 2 x fp16 halves of the scaled values, fp32 accumulate)",
                  "bf16x3": "f32 (Hessian products as 3 x bf16 pieces, fp32 accumulate)", "f32": "f32"}[args.hessian],
        "data": "synthetic",
        "config": {"workload": wl.name, "d_out": d_out, "d_in": d_in, "tokens": n_tok,
                   "bits": wl.bits, "group": wl.group, "block": wl.block,
                   "refine_iters": wl.refine_iters, "hessian_calls_per_step": len(calls),
                   "hessian_kernel": args.hessian},
        "phase_ms": {k: round(v, 4) for k, v in phase_ms.items()},
        "hessian_kernel_ms": round(kernel_ms, 4),
        "quantize_only_mparams_per_s": (wl.params / (phase_ms["quantize"] * 1e-3) / 1e6
                                        if phase_ms["quantize"] > 0 else None),
        "roofline": {"kernel": kernel, "bound": "mfma", "achieved": achieved,
                     "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": traffic, **roof_extra},
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, W.cpu(), scales.cpu())
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
