#!/usr/bin/env python3
"""Benchmark of the RFSF-TS hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic batch that is already resident in
HBM: random Fourier features, time increments, CountSketch, FFT-domain level recursion
(rfsf_ts_features) and the linear Gram of the resulting features (rfsf_ts_gram). For the
workload with a second batch, the step also computes the second batch's features and the
Gram is the cross Gram. The metric is sequences x time points per second, (N [+ N2]) * L / t_step.

Prints ONE JSON line. Besides the required fields it carries
  "roofline"     for the kernel that takes most of the step (algorithmic bytes or flops per
                 launch / average launch duration measured with HIP events on the launch stream),
  "kernels"      the same figures for all three kernels,
  "cpu_baseline" the fp64 CPU oracle timed on this machine's host cores on a bounded sample,
  "parity"       block / Gram errors of the GPU result against that oracle sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MFMA_FP32_PEAK_TFLOPS = 157.3    # MI355X dense fp32 matrix, published

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix, published


VALU_FP32_PEAK_TFLOPS = 157.3     # MI355X fp32 vector, published: 256 CUs x 128 fused multiply-adds per clock at 2.4 GHz. A loop of
                                  # plain (unpacked) v_fma_f32 chains measures 118 TFLOP/s here (rfsf_ts_probe_peaks), so the
                                  # rate does not hinge on packed instructions, which this library is built without
COS_FLOPS = 20                   # argument (fma), reduction by pi (fma, sub, 2 fma), r^2, degree-5 polynomial in r^2 (5 fma)


def bench_dp1d(args, w, inp, dev, ls) -> int:
    """Sibling variant RFSF-DP-1D: one fused kernel (projection on the matrix cores, cosine, time
    difference, per-component recurrence) + the Gram of its features. ALU-bound: nothing but X, W and
    bias is read and only the features are written."""
    import numpy as np
    import torch

    import paper_2501_07145_amd as rfsf
    from paper_2501_07145_amd import workloads as wl

    bias_h = wl.make_bias(w, 0)
    bias = torch.from_numpy(bias_h).cuda()
    ncols = 1 + w.M * w.F
    out = torch.empty((w.N, (ncols + 3) // 4 * 4), dtype=torch.float32, device="cuda")[:, :ncols]
    K = torch.empty((w.N, w.N), dtype=torch.float32, device="cuda")

    def step():
        rfsf.rfsf_dp1d_features(dev["X"], dev["W"], bias, ls, out=out)
        rfsf.rfsf_ts_gram(out, K=K)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps
    rfsf.rfsf_ts_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = rfsf.rfsf_ts_profile_read(reset=True)
    rfsf.rfsf_ts_profile_enable(False)

    units = w.N * w.L
    # per (time point, component): the projection's 2d flops run on the matrix cores, the cosine and the
    # recurrence (difference + fused multiply-add: 3 flops) on the vector units; the kernel is bound by
    # whichever of the two pipes is busier for the shape (wide d: matrix cores), and the line names that one
    elements = units * w.M * w.F
    ms = prof["ms_dp1d"] / max(1, prof["launches_dp1d"])
    valu_tflops = elements * (COS_FLOPS + 3.0) / (ms * 1e-3) / 1e12
    mfma_tflops = elements * 2.0 * w.d / (ms * 1e-3) / 1e12
    valu_frac, mfma_frac = valu_tflops / VALU_FP32_PEAK_TFLOPS, mfma_tflops / MFMA_FP32_PEAK_TFLOPS
    gram_pairs = w.N * w.N if ((w.N + 63) // 64) * ((w.N + 63) // 64 + 1) // 2 < 512 else w.N * (w.N + 1) / 2
    gms = prof["ms_gram"] / max(1, prof["launches_gram"])
    by_mfma = mfma_frac > valu_frac
    kernels = {
        "dp1d": {"bound": "mfma" if by_mfma else "alu", "achieved": mfma_tflops if by_mfma else valu_tflops,
                 "peak": MFMA_FP32_PEAK_TFLOPS if by_mfma else VALU_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                 "frac": max(mfma_frac, valu_frac), "traffic": None, "avg_launch_ms": ms,
                 "ms_per_step": prof["ms_dp1d"] / args.steps,
                 "alu_frac": valu_frac, "alu_peak": VALU_FP32_PEAK_TFLOPS, "mfma_frac": mfma_frac,
                 "cosines_per_s": elements / (ms * 1e-3)},
        "gram": {"bound": "mfma", "achieved": 2.0 * gram_pairs * ncols / (gms * 1e-3) / 1e12,
                 "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                 "frac": 2.0 * gram_pairs * ncols / (gms * 1e-3) / 1e12 / MFMA_FP32_PEAK_TFLOPS, "traffic": None,
                 "avg_launch_ms": gms, "ms_per_step": prof["ms_gram"] / args.steps},
    }
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    roofline = {k: kernels[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
    roofline["kernel"] = dominant
    result = {
        "metric": "rfsf_dp1d_sequence_steps_per_s", "value": units / t_step, "unit": "sequences*steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "variant": "dp1d", "N": w.N, "L": w.L, "d": w.d, "M": w.M, "F": w.F,
                   "lengthscale": ls, "paths": w.kind, "step": "DP-1D features + Gram"},
        "roofline": roofline, "kernels": kernels,
    }
    if getattr(args, "measured_peaks", None):
        result["measured_peaks"] = dict(args.measured_peaks)
    if not args.no_cpu_baseline:
        import oracle
        from tests.parity import block_errors
        rows = min(w.N, {"tiny": 16, "small": 1000, "medium": 64, "long": 32, "large": 64}[w.name]
                   if args.cpu_rows < 0 else args.cpu_rows)
        sel = np.linspace(0, w.N - 1, rows).round().astype(np.int64)
        t0 = time.perf_counter()
        want = oracle.dp1d_features(inp["X"][sel], inp["W"], bias_h, ls)
        t_feat = time.perf_counter() - t0
        err = block_errors(out.cpu().numpy()[sel], want, w.M, w.F)
        result["cpu_baseline"] = {"value": rows * w.L / t_feat, "unit": "sequences*steps/s", "cores": oracle.threads(),
                                  "kind": "oracle", "sample": f"{rows} of {w.N} sequences, features only, {t_feat:.2f} s, fp64"}
        result["parity"] = {"rows": int(rows), "max_block_err_per_level": [float(e) for e in err]}
    print(json.dumps(result))
    return 0


def bench_trp(args, w, inp, dev, ls) -> int:
    """Sibling variant RFSF-TRP with Q = D projections per level: projection kernel (as in the main path),
    one fp32 MFMA GEMM per level [N*L, 2F] x [2F, Q], a streaming scan over time, then the Gram."""
    import numpy as np
    import torch

    import paper_2501_07145_amd as rfsf
    from paper_2501_07145_amd import workloads as wl

    Q = w.D
    Z_h = wl.make_projections(w, 0)
    Z = torch.from_numpy(Z_h).cuda()
    ncols = 1 + w.M * Q
    rec, _ = rfsf.rfsf_trp_workspace_bytes(w.N, w.L, w.d, w.M, w.F, Q, w.rff_bf16)
    workspace = torch.empty(rec, dtype=torch.uint8, device="cuda")
    out = torch.empty((w.N, (ncols + 3) // 4 * 4), dtype=torch.float32, device="cuda")[:, :ncols]
    K = torch.empty((w.N, w.N), dtype=torch.float32, device="cuda")

    def step():
        rfsf.rfsf_trp_features(dev["X"], dev["W"], Z, ls, out=out, workspace=workspace, rff_bf16=w.rff_bf16)
        rfsf.rfsf_ts_gram(out, K=K)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps
    rfsf.rfsf_ts_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = rfsf.rfsf_ts_profile_read(reset=True)
    rfsf.rfsf_ts_profile_enable(False)

    units = w.N * w.L
    kernels = {}

    def entry(name, bound, work_per_step, unit, peak):
        n = prof[f"launches_{name}"]
        if n == 0:
            return
        avg_ms = prof[f"ms_{name}"] / n
        achieved = work_per_step * args.steps / n / (avg_ms * 1e-3) / (1e9 if unit == "GB/s" else 1e12)
        kernels[name] = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak,
                         "traffic": None, "avg_launch_ms": avg_ms, "launches_per_step": n / args.steps,
                         "ms_per_step": prof[f"ms_{name}"] / args.steps}

    entry("rff_increments", "hbm", units * (4.0 * w.d + 4.0 * w.M * 2 * w.F), "GB/s", HBM_PEAK_GBS)
    entry("trp_project", "mfma", 2.0 * units * w.M * 2 * w.F * Q, "TFLOP/s", MFMA_FP32_PEAK_TFLOPS)   # M GEMMs per scope
    entry("trp_scan", "hbm", 4.0 * units * w.M * Q + 4.0 * w.N * ncols, "GB/s", HBM_PEAK_GBS)
    gram_pairs = w.N * w.N if ((w.N + 63) // 64) * ((w.N + 63) // 64 + 1) // 2 < 512 else w.N * (w.N + 1) / 2
    entry("gram", "mfma", 2.0 * gram_pairs * ncols, "TFLOP/s", MFMA_FP32_PEAK_TFLOPS)
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    roofline = {k: kernels[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")}
    roofline["kernel"] = dominant
    result = {
        "metric": "rfsf_trp_sequence_steps_per_s", "value": units / t_step, "unit": "sequences*steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": t_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16+f32" if w.rff_bf16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "variant": "trp", "N": w.N, "L": w.L, "d": w.d, "M": w.M, "F": w.F, "Q": Q,
                   "lengthscale": ls, "paths": w.kind, "step": "TRP features + Gram", "workspace_bytes": rec},
        "roofline": roofline, "kernels": kernels,
    }
    if getattr(args, "measured_peaks", None):
        result["measured_peaks"] = dict(args.measured_peaks)
    if not args.no_cpu_baseline:
        import oracle
        from tests.parity import block_errors
        rows = min(w.N, {"tiny": 16, "small": 200, "medium": 16, "long": 8, "large": 8}[w.name]
                   if args.cpu_rows < 0 else args.cpu_rows)
        sel = np.linspace(0, w.N - 1, rows).round().astype(np.int64)
        Wo = wl.round_to_bf16(inp["W"]) if w.rff_bf16 else inp["W"]
        t0 = time.perf_counter()
        want = oracle.trp_features(inp["X"][sel], Wo, Z_h, ls)
        t_feat = time.perf_counter() - t0
        err = block_errors(out.cpu().numpy()[sel], want, w.M, Q)
        result["cpu_baseline"] = {"value": rows * w.L / t_feat, "unit": "sequences*steps/s", "cores": oracle.threads(),
                                  "kind": "oracle", "sample": f"{rows} of {w.N} sequences, features only, {t_feat:.2f} s, fp64"}
        result["parity"] = {"rows": int(rows), "max_block_err_per_level": [float(e) for e in err]}
    print(json.dumps(result))
    return 0


def _kernel_source_digest() -> str:
    """Digest of the kernel sources the loaded library was built from; ties a stored rocprofv3 traffic figure to
    the code it was measured on."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2501_07145_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h", ".inc")):
            h.update(name.encode())
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def _measured_traffic(workload: str) -> dict:
    """HBM bytes per kernel launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary of this workload
    (profiles/hbm_traffic_<workload>.txt, lines `traffic_bytes_per_launch <kernel> <bytes>`), or {} when there
    is none or when it was measured on other kernel sources than the ones in this tree."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return {}
    digest, out = None, {}
    with open(path) as f:
        for line in f:
            t = line.split()
            if len(t) == 2 and t[0] == "kernel_sources_sha256":
                digest = t[1]
            elif len(t) == 3 and t[0] == "traffic_bytes_per_launch":
                out[t[1]] = float(t[2])
    return out if digest == _kernel_source_digest() else {}


def bench_ts(args, name: str, steps: int, warmup: int, cpu_baseline: bool) -> dict:
    """One workload through the tensor-sketch path: features (+ second batch) + Gram; returns the result dict."""
    import numpy as np
    import torch

    import paper_2501_07145_amd as rfsf
    from paper_2501_07145_amd import workloads as wl

    w = wl.WORKLOADS[name]
    inp = wl.make_inputs(w, 0)
    dev = {k: torch.from_numpy(v).cuda() for k, v in inp.items() if isinstance(v, np.ndarray)}
    ls = inp["lengthscale"]
    X2 = torch.from_numpy(wl.make_paths(w.scaled(N=w.N2), 1)).cuda() if w.N2 else None

    rec_bytes, _ = rfsf.rfsf_ts_workspace_bytes(w.N, w.L, w.d, w.M, w.F, w.D, w.rff_bf16)
    if args.workspace_mib > 0:
        rec_bytes = args.workspace_mib << 20
    workspace = torch.empty(rec_bytes, dtype=torch.uint8, device="cuda")
    ld = rfsf.feature_row_stride(w.M, w.D)
    out = torch.empty((w.N, ld), dtype=torch.float32, device="cuda")[:, :w.ncols]
    out2 = torch.empty((w.N2, ld), dtype=torch.float32, device="cuda")[:, :w.ncols] if w.N2 else None
    K = torch.empty((w.N, w.N2 if w.N2 else w.N), dtype=torch.float32, device="cuda")

    def step():
        rfsf.rfsf_ts_features(dev["X"], dev["W"], dev["hash"], dev["sign"], ls, w.D, out=out,
                              workspace=workspace, rff_bf16=w.rff_bf16)
        if args.normalize:
            rfsf.rfsf_ts_normalize_features(out, w.M, w.D)
        if X2 is not None:
            rfsf.rfsf_ts_features(X2, dev["W"], dev["hash"], dev["sign"], ls, w.D, out=out2,
                                  workspace=workspace, rff_bf16=w.rff_bf16)
            if args.normalize:
                rfsf.rfsf_ts_normalize_features(out2, w.M, w.D)
            rfsf.rfsf_ts_gram(out, out2, K=K)
        else:
            rfsf.rfsf_ts_gram(out, K=K)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / steps

    # same K steps again with per-kernel HIP events on the launch stream
    rfsf.rfsf_ts_profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    prof = rfsf.rfsf_ts_profile_read(reset=True)
    rfsf.rfsf_ts_profile_enable(False)

    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib * (1 << 18), dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    n_seq = w.N + w.N2
    units = n_seq * w.L                              # the metric's unit: sequences x time points
    incr_units = n_seq * (w.L - 1)                   # increments: what the kernels between X and out move
    incr_bytes = 4.0 * w.M * 2 * w.F                 # fp32 increments of one time step, all levels
    traffic = _measured_traffic(w.name)
    kernels = {}

    def entry(kname, bound, work_per_step, unit, peak, **extra):
        n = prof[f"launches_{kname}"]
        if n == 0:
            return
        avg_ms = prof[f"ms_{kname}"] / n
        per_launch = work_per_step * steps / n
        achieved = per_launch / (avg_ms * 1e-3) / (1e9 if unit == "GB/s" else 1e12)
        kernels[kname] = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                          "frac": achieved / peak, "traffic": traffic.get(kname),
                          "algorithmic_per_launch": per_launch, "avg_launch_ms": avg_ms,
                          "launches_per_step": n / steps, "ms_per_step": prof[f"ms_{kname}"] / steps}
        t_s = prof[f"ms_{kname}"] / steps * 1e-3
        for k, v in extra.items():
            kernels[kname][k] = v / t_s

    # projection kernel: binding resources are the HBM write of the increments and the sin/cos arithmetic
    # (K = d is tiny), so it is entered against the HBM roofline; the matrix-core share and the sin/cos rate
    # are reported beside it
    mfma_peak = MFMA_BF16_PEAK_TFLOPS if w.rff_bf16 else MFMA_FP32_PEAK_TFLOPS
    proj_flops = (2.0 if w.rff_bf16 else 1.0) * 2.0 * w.d * w.M * w.F    # bf16: X enters as two bf16 terms
    entry("rff_increments", "hbm", n_seq * 4.0 * w.L * w.d + incr_units * incr_bytes, "GB/s", HBM_PEAK_GBS,
          mfma_tflops=units * proj_flops / 1e12, sincos_pairs_per_s=float(units * w.M * w.F),
          write_gbs=incr_units * incr_bytes / 1e9)
    if "rff_increments" in kernels:
        kernels["rff_increments"]["mfma_peak"] = mfma_peak
        kernels["rff_increments"]["mfma_frac"] = kernels["rff_increments"]["mfma_tflops"] / mfma_peak
    entry("sketch_fft_scan", "hbm", incr_units * incr_bytes + 4.0 * n_seq * w.M * w.D, "GB/s", HBM_PEAK_GBS)
    Ny = w.N2 if w.N2 else w.N
    # flops the kernel performs: the whole matrix for a cross Gram; for K = Phi Phi^T of 2048+ rows
    # only the tiles on or above the diagonal (counted here as N(N+1)/2 inner products)
    gram_pairs = w.N * Ny if (w.N2 or ((w.N + 63) // 64) * ((w.N + 63) // 64 + 1) // 2 < 512) else w.N * (w.N + 1) / 2
    entry("gram", "mfma", 2.0 * gram_pairs * w.ncols, "TFLOP/s", MFMA_FP32_PEAK_TFLOPS)
    entry("normalize", "hbm", 2.0 * 4.0 * n_seq * w.ncols, "GB/s", HBM_PEAK_GBS)
    # beside the published peaks: what the simplest kernels of the same kind reach on this GPU (streaming reads for
    # the kernel that reads the increments, non-temporal streaming writes for the one that writes them, an issue
    # loop of fp32 matrix instructions for the Gram)
    peaks = getattr(args, "measured_peaks", None)
    if peaks:
        for kname, key in (("rff_increments", "write_nt_gbs"), ("sketch_fft_scan", "read_gbs"), ("gram", "mfma_f32_tflops"),
                           ("normalize", "copy_gbs")):
            if kname in kernels:
                kernels[kname]["measured_peak"] = peaks[key]
                kernels[kname]["frac_of_measured"] = kernels[kname]["achieved"] / peaks[key]
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    roofline = {k: kernels[dominant][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic",
                                                   "measured_peak", "frac_of_measured") if k in kernels[dominant]}
    roofline["kernel"] = dominant

    result = {
        "metric": "rfsf_ts_sequence_steps_per_s",
        "value": units / t_step,
        "unit": "sequences*steps/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": t_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16+f32" if w.rff_bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "N": w.N, "N2": w.N2, "L": w.L, "d": w.d, "M": w.M, "F": w.F, "D": w.D,
                   "lengthscale": ls, "paths": w.kind, "rff_bf16": w.rff_bf16,
                   "step": "features + normalisation + Gram" if args.normalize else "features + Gram",
                   "workspace_bytes": rec_bytes},
        "roofline": roofline,
        "kernels": kernels,
    }

    if cpu_baseline:
        import oracle
        from tests.parity import block_errors, gram_error
        default_rows = {"tiny": 16, "small": 1000, "medium": 512, "long": 128, "large": 256, "paper": 100, "paper_long": 2}[w.name]
        rows = min(w.N, default_rows if args.cpu_rows < 0 else args.cpu_rows)
        sel = np.linspace(0, w.N - 1, rows).round().astype(np.int64)
        Xs = inp["X"][sel]
        Wo = wl.round_to_bf16(inp["W"]) if w.rff_bf16 else inp["W"]   # the rounding the bf16 variant applies
        t0 = time.perf_counter()
        want = oracle.features(Xs, Wo, inp["hash"], inp["sign"], ls, w.D)
        if args.normalize:
            want = oracle.normalize(want, w.M, w.D)
        t_feat = time.perf_counter() - t0
        t0 = time.perf_counter()
        Kw = oracle.gram(want)
        t_gram = time.perf_counter() - t0
        got = out.cpu().numpy()[sel]
        err = block_errors(got, want, w.M, w.D, level0=(1.0 / (w.M + 1) ** 0.5) if args.normalize else 1.0)
        Ksel = (rfsf.rfsf_ts_gram(out[torch.from_numpy(sel).cuda()].contiguous()) if X2 is not None
                else K[torch.from_numpy(sel).cuda()][:, torch.from_numpy(sel).cuda()])
        torch.cuda.synchronize()
        result["cpu_baseline"] = {
            "value": rows * w.L / (t_feat + t_gram), "unit": "sequences*steps/s", "cores": oracle.threads(),
            "kind": "oracle",
            "sample": f"{rows} of {w.N} sequences (evenly spaced rows), features {t_feat:.2f} s + "
                      f"{rows}x{rows} Gram {t_gram:.2f} s, fp64, direct O(D^2) convolution",
        }
        result["parity"] = {"rows": int(rows), "max_block_err_per_level": [float(e) for e in err],
                            "gram_err": gram_error(Ksel.cpu().numpy(), Kw)}
    del workspace, out, out2, K, dev, X2
    torch.cuda.empty_cache()
    return result


DEFAULT_STEPS = {"tiny": (300, 50), "small": (300, 50), "medium": (20, 3), "long": (20, 3), "large": (5, 1),
                 "paper": (20, 3), "paper_long": (20, 3)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: 300 for tiny/small, 20 for medium/long, 5 for large)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps (default: 50 / 3 / 1)")
    ap.add_argument("--workload", default="medium", choices=["tiny", "small", "medium", "long", "large", "paper", "paper_long"],
                    help="medium (default) is the largest configuration that runs in fp32 throughout")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the probe of what plain streaming kernels and issue loops reach on this GPU")
    ap.add_argument("--also", default=None,
                    help="comma-separated further workloads measured after the headline one with their own default "
                         "step counts and reported under 'other_workloads' (default: small,long,large,paper,paper_long when the "
                         "headline is the default medium run, none otherwise; 'none' switches it off)")
    ap.add_argument("--cpu-rows", type=int, default=-1, help="oracle sample size (-1: per-workload default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variant", default="ts", choices=["ts", "dp1d", "trp"],
                    help="ts: the tensor-sketch path (default, the headline metric); dp1d: the sibling RFSF-DP-1D "
                         "variant (one fused kernel, features [N, 1+M*F]) plus its Gram; trp: the sibling RFSF-TRP variant "
                         "(Q = D Gaussian projections per level) plus its Gram")
    ap.add_argument("--normalize", action="store_true",
                    help="add the level-wise normalisation of the features to the step (not part of the default path)")
    ap.add_argument("--workspace-mib", type=int, default=0,
                    help="workspace size instead of the recommended one (sets the number of sequences per launch)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="after the timed steps run one plain device copy of this many MiB (calibrates the "
                         "FETCH_SIZE / WRITE_SIZE counters under rocprofv3)")
    args = ap.parse_args()
    default_run = args.workload == "medium" and args.variant == "ts" and not args.normalize and \
        args.workspace_mib == 0 and args.copy_probe_mib == 0
    if args.also is None:
        args.also = "small,long,large,paper,paper_long" if default_run else "none"
    if args.steps is None:
        args.steps = DEFAULT_STEPS[args.workload][0]
    if args.warmup is None:
        args.warmup = DEFAULT_STEPS[args.workload][1]
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (sequences are independent; sharding N over "
              "GPUs is design-only). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2501_07145_amd import workloads as wl

    torch.cuda.set_device(0)
    if not args.no_measured_peaks:
        import paper_2501_07145_amd as rfsf
        scratch = torch.empty(4 << 30, dtype=torch.uint8, device="cuda")      # 16 times the last-level cache
        args.measured_peaks = rfsf.rfsf_ts_probe_peaks(scratch)
        del scratch
        torch.cuda.empty_cache()
    if args.variant != "ts":
        w = wl.WORKLOADS[args.workload]
        inp = wl.make_inputs(w, 0)
        dev = {k: torch.from_numpy(v).cuda() for k, v in inp.items() if isinstance(v, np.ndarray)}
        if args.variant == "dp1d":
            return bench_dp1d(args, w, inp, dev, inp["lengthscale"])
        return bench_trp(args, w, inp, dev, inp["lengthscale"])

    result = bench_ts(args, args.workload, args.steps, args.warmup, not args.no_cpu_baseline)
    if getattr(args, "measured_peaks", None):
        result["measured_peaks"] = dict(args.measured_peaks, note="plain streaming kernels over 4 GiB and fp32 issue loops, "
                                        "measured at the start of this run (rfsf_ts_probe_peaks)")
    others = [n for n in args.also.split(",") if n and n != "none" and n != args.workload]
    if others:
        # the other configurations, each at its own default step count, without the oracle leg: context for the
        # headline line above, which stays the one the metric is quoted on
        result["other_workloads"] = {}
        for name in others:
            if name not in wl.WORKLOADS:
                print(f"bench.py: unknown workload {name!r} in --also", file=sys.stderr)
                return 2
            r = bench_ts(args, name, *DEFAULT_STEPS[name], False)
            result["other_workloads"][name] = {
                "value": r["value"], "ms_per_step": r["ms_per_step"], "steps": r["steps"], "dtype": r["dtype"],
                "config": r["config"],
                "kernels": {k: {f: v[f] for f in ("bound", "frac", "achieved", "unit", "avg_launch_ms",
                                                   "launches_per_step", "frac_of_measured") if f in v}
                            for k, v in r["kernels"].items()}}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
