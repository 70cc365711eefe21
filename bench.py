#!/usr/bin/env python3
"""Bench of the BDR/MX hot path on one MI355X.

Workload ("bandwidth" configuration): a 268,435,456-element FP32 tensor (1 GiB), 0.02 x
Student-t(3), seed 1, already resident in HBM.  One step is one pass of the row-wise hot path
over it for each of MX9, MX6 and MX4: quantize to the packed planes, then dequantize back to
FP32 (six kernels).  The headline value is the algorithmic traffic of a step divided by its
wall time: 2 * n * (4 + bits/8) bytes per format.

Prints ONE JSON line.  Besides the contract keys it carries
  roofline      HBM roofline of the dominant kernel of the step -- the one with the largest
                share of the timed region, found from device events around every launch inside
                that region (it is the MX9 dequantize) -- and, under `kernels`, the same figures
                for all six, with `frac_min` the lowest of them;
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload, on all host
                threads it may use and on one;
  other         separately timed legs: fused round trip, QSNR sweep, column-wise quantize,
                mx_gemm (whatever the library implements), not part of `value`.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published peak
N_ELEMS = 1 << 28
COLS = 4096
FORMATS = ("MX9", "MX6", "MX4")


def alg_bytes(n, bits, elem_bytes=4):
    """Algorithmic bytes of one direction: the tensor once plus its packed image once."""
    return n * (elem_bytes + bits / 8.0)


def cpu_baseline(sample_elems, threads, single_sample_elems):
    """The oracle as it stands, on the first `sample_elems` of the same tensor recipe, the same
    step (quantize + dequantize for MX9, MX6, MX4), rows split over `threads` host threads; then
    the same on one thread over a smaller prefix."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle as O
    import synth_inputs as S

    x = S.bandwidth(sample_elems, COLS, device="cpu").numpy()
    fmts = (O.MX9, O.MX6, O.MX4)

    def work(p):
        for f in fmts:
            planes = O.quantize(f, p)
            O.dequantize(f, *planes, *p.shape)

    def run(xs, nthreads):
        rows = xs.shape[0]
        parts = [xs[i * rows // nthreads:(i + 1) * rows // nthreads] for i in range(nthreads)]
        parts = [np.ascontiguousarray(p) for p in parts if p.shape[0]]
        t0 = time.perf_counter()
        if len(parts) == 1:
            work(parts[0])
        else:
            with ThreadPoolExecutor(max_workers=len(parts)) as ex:
                list(ex.map(work, parts))
        dt = time.perf_counter() - t0
        nbytes = sum(2 * alg_bytes(xs.size, b) for b in (9, 6, 4))
        return nbytes / dt / 1e9, dt, len(parts)

    O.lib()
    v, dt, used = run(x, threads)
    v1, dt1, _ = run(x[:single_sample_elems // COLS], 1)
    return {
        "value": round(v, 3), "unit": "GB/s", "cores": used, "kind": "oracle",
        "sample": "first %d elements of the same tensor recipe, same step (MX9+MX6+MX4 quantize"
                  " and dequantize), %.1f s wall on %d threads" % (sample_elems, dt, used),
        "host_cores": os.cpu_count(),
        "single_thread": {"value": round(v1, 3), "unit": "GB/s", "cores": 1,
                          "sample": "first %d elements, %.1f s wall" % (single_sample_elems, dt1)},
    }


def median(v):
    v = sorted(v)
    n = len(v)
    return v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other", action="store_true", help="skip the separately timed legs")
    ap.add_argument("--cpu-sample", type=int, default=1 << 27)
    ap.add_argument("--cpu-single-sample", type=int, default=1 << 24)
    ap.add_argument("--pmc-probe", action="store_true",
                    help="run a 1 GiB tensor copy and one launch of each row-wise MX kernel, "
                         "three times, and exit (for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--aux-probe", action="store_true",
                    help="run a 1 GiB tensor copy, then the column-wise and row-wise BF16 kernels "
                         "(8192 x 12288, MX9), the gather kernel and general-format kernels, three "
                         "times, and exit (for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--other-probe", action="store_true",
                    help="run mx_gemm (both forms, 8192^3, MX6, MX9 and MX4), the 64-format sweep and the "
                         "dot-product pipeline model a few times and exit (for rocprofv3 --kernel-trace "
                         "and --pmc MfmaUtil VALUBusy)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (blocks are independent, so the path "
                 "shards by rows with no exchange and one GPU shows all of it); run with --gpus 1")

    import torch

    import paper_2302_08007_amd as B
    import synth_inputs as S

    torch.cuda.set_device(0)
    if args.aux_probe:
        return aux_probe(B, S, torch)
    x = S.bandwidth(N_ELEMS, COLS, device="cuda")
    rows, cols = x.shape
    y = torch.empty_like(x)
    planes = {n: B.alloc_planes(getattr(B, n), rows, cols) for n in FORMATS}
    fm = {n: getattr(B, n) for n in FORMATS}
    bits = {"MX9": 9, "MX6": 6, "MX4": 4}
    marks = []  # per timed step: 7 events bracketing the six kernels

    def step(record):
        # all three quantizes, then all three dequantizes: alternating a read-heavy and a
        # write-heavy kernel makes each wait for the other's write-back
        ev = []

        def mark():
            if record:
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                ev.append(e)
        mark()
        for n in FORMATS:
            B.bdr_quantize(fm[n], x, out=planes[n])
            mark()
        for n in FORMATS:
            B.bdr_dequantize(fm[n], planes[n], rows, cols, out=y)
            mark()
        if record:
            marks.append(ev)

    if args.other_probe:
        del x, y, planes
        M = N = K = 8192
        A, Bm = S.gemm_operands(M, N, K, device="cuda")
        pa, pb = B.bdr_quantize(B.MX6, A), B.bdr_quantize(B.MX6, Bm)
        C = torch.empty(M, N, device="cuda")
        ws = torch.empty(B.mx_gemm_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
        for i in range(45):  # the first 40 settle the matrix-core clock, the last 5 are the sample
            B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K, out=C, workspace=ws)
        for i in range(5):
            B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K, out=C)
        pa, pb = B.bdr_quantize(B.MX9, A), B.bdr_quantize(B.MX9, Bm)
        for i in range(10):  # MX9: the BF16 product kernel
            B.mx_gemm(B.MX9, B.MX9, pa, pb, M, N, K, out=C, workspace=ws)
        pa, pb = B.bdr_quantize(B.MX4, A), B.bdr_quantize(B.MX4, Bm)
        for i in range(10):  # MX4 x MX4: the FP4 product kernel
            B.mx_gemm(B.MX4, B.MX4, pa, pb, M, N, K, out=C, workspace=ws)
        xs = S.sweep(device="cuda")
        fmts = [B.fmt(k1, k1 if k2 == 0 else k2, d2, m) for k1 in (8, 16, 32, 64)
                for k2 in (1, 2, 4, 0) for d2 in (0, 1) for m in (2, 4)]
        wsw = torch.empty(B.lib.bdr_qsnr_sweep_workspace_bytes(len(fmts)), dtype=torch.uint8, device="cuda")
        for i in range(5):
            B.bdr_qsnr_sweep(fmts, xs, workspace=wsw)
        pa, pb = B.bdr_quantize(B.MX6, A), B.bdr_quantize(B.MX6, Bm)
        for i in range(5):
            B.mx_dot_pipeline(B.MX6, B.MX6, pa, pb, M, N, K, r=K, out=C, workspace=ws)
        for i in range(5):
            B.mx_dot_pipeline(B.MX6, B.MX6, pa, pb, M, N, K, r=64, out=C, workspace=ws)
        torch.cuda.synchronize()
        print(json.dumps({"other_probe": "45 x two-pass MX6 mx_gemm, 5 x single-kernel MX6 mx_gemm, "
                                         "10 x two-pass MX9 mx_gemm, 10 x two-pass MX4 mx_gemm, "
                                         "5 x 64-format sweep, 5 + 5 x MX6 "
                                         "mx_dot_pipeline (one pass, r = 64), all at 8192^3"}))
        return

    if args.pmc_probe:
        # the copy reads 1 GiB and writes 1 GiB: it calibrates the counters' units
        for _ in range(3):
            y.copy_(x)
            for n in ("MX6", "MX9", "MX4"):
                B.bdr_quantize(fm[n], x, out=planes[n])
                B.bdr_dequantize(fm[n], planes[n], rows, cols, out=y)
                B.bdr_quantize_dequantize(fm[n], x, out=y)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": "3 x (copy, then quantize, dequantize, fused for MX6, MX9, MX4)"}))
        return

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    step_bytes = sum(2 * alg_bytes(N_ELEMS, bits[n]) for n in FORMATS)
    value = step_bytes / (ms_per_step * 1e-3) / 1e9

    labels = ["quantize_" + n for n in FORMATS] + ["dequantize_" + n for n in FORMATS]
    kern = {}
    for n in FORMATS:
        mb = {"MX9": 7, "MX6": 4, "MX4": 2}[n]
        kern["quantize_" + n] = "mx_quantize_row_kernel<%d, float>" % mb
        kern["dequantize_" + n] = "mx_dequantize_row_kernel<%d, float>" % mb
    in_loop_us, kernels = {}, {}
    for k, lab in enumerate(labels):
        ts = [ev[k].elapsed_time(ev[k + 1]) * 1e3 for ev in marks]      # one per timed step
        in_loop_us[lab] = median(ts)
        mean_us = sum(ts) / len(ts)
        ab = alg_bytes(N_ELEMS, bits[lab.split("_")[1]])
        # `achieved` follows the average launch duration (what rocprofv3 --stats reports as
        # AverageNs, so the two can be compared); the median is given next to it
        kernels[lab] = {"kernel": kern[lab], "avg_launch_us": round(mean_us, 2),
                        "median_launch_us": round(in_loop_us[lab], 2), "launches": len(ts),
                        "algorithmic_bytes_per_launch": ab,
                        "achieved": round(ab / mean_us / 1e3, 1),
                        "frac": round(ab / mean_us / 1e3 / HBM_PEAK_GBS, 4),
                        "achieved_median": round(ab / in_loop_us[lab] / 1e3, 1),
                        "share_of_step": round(mean_us / (ms_per_step * 1e3), 4)}
    dom = max(labels, key=lambda l: kernels[l]["avg_launch_us"])     # largest share of the timed region
    traffic, traffic_commit = measured_traffic(dom)
    roofline = {
        "kernel": "%s (%s, fp32, 2^28 elements per launch)" % (kern[dom], dom.replace("_", " ")),
        "bound": "hbm", "achieved": kernels[dom]["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": kernels[dom]["frac"],
        "algorithmic_bytes_per_launch": kernels[dom]["algorithmic_bytes_per_launch"],
        "avg_launch_us": kernels[dom]["avg_launch_us"], "median_launch_us": kernels[dom]["median_launch_us"],
        "traffic": traffic, "traffic_profile_commit": traffic_commit,
        "frac_min": min(v["frac"] for v in kernels.values()),
        "kernels": kernels,
    }

    def timed(fn, reps=7, inner=3, warm=3):
        """Median, over `reps` samples, of the device time of one call.  A sample is `inner` calls
        enqueued between one pair of events (so the host's launch overhead overlaps with the
        previous call's execution) divided by `inner`; reps * inner >= 20 launches in every leg."""
        assert reps * inner >= 20
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(inner):
                fn()
            b.record()
            b.synchronize()
            ts.append(a.elapsed_time(b) / inner)
        return median(ts)

    other = {}
    if not args.no_other:
        # per-kernel figures from the timed loop itself (steady state, planes cold); the fused
        # round trip is timed on its own (2 GiB of traffic per call, nothing fits a cache)
        per = {}
        for n in FORMATS:
            ab = alg_bytes(N_ELEMS, bits[n])
            tq, td = in_loop_us["quantize_" + n] * 1e-3, in_loop_us["dequantize_" + n] * 1e-3
            tf = timed(lambda: B.bdr_quantize_dequantize(fm[n], x, out=y))
            per[n] = {
                "quantize_us": round(tq * 1e3, 1), "quantize_GBps": round(ab / tq / 1e6, 1),
                "quantize_frac": round(ab / tq / 1e6 / HBM_PEAK_GBS, 4),
                "dequantize_us": round(td * 1e3, 1), "dequantize_GBps": round(ab / td / 1e6, 1),
                "dequantize_frac": round(ab / td / 1e6 / HBM_PEAK_GBS, 4),
                "fused_roundtrip_us": round(tf * 1e3, 1),
                "fused_roundtrip_GBps": round(8.0 * N_ELEMS / tf / 1e6, 1),
                "fused_roundtrip_frac": round(8.0 * N_ELEMS / tf / 1e6 / HBM_PEAK_GBS, 4),
                "quantize_Gelem_s": round(N_ELEMS / tq / 1e6, 1),
            }
        other["rowwise_fp32_1GiB"] = per
        del y
        other.update(other_legs(B, S, torch, timed))

    cpu = None
    if not args.no_cpu_baseline:
        threads = min(16, os.cpu_count() or 1)
        cpu = cpu_baseline(args.cpu_sample, threads, args.cpu_single_sample)

    print(json.dumps({
        "metric": "MX9/MX6/MX4 quantize+dequantize algorithmic GB/s (fp32, row-wise)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "bandwidth: 268,435,456 fp32 (1 GiB), 0.02*Student-t(3), seed 1; "
                               "step = quantize+dequantize for MX9, MX6, MX4",
                   "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4)},
        "roofline": roofline, "cpu_baseline": cpu, "other": other,
        "profile_commit": {"unit_utilisation": profile_commit(UTIL_PROFILE)},
    }))


def aux_probe(B, S, torch):
    """One launch each, three times over, of the kernels outside the headline step whose HBM
    traffic is worth counting, after a copy of known size that calibrates the counters."""
    x = S.bandwidth(N_ELEMS, COLS, device="cuda")
    y = torch.empty_like(x)
    rows, cols = x.shape
    xa = S.activation(device="cuda")
    ra, ca = xa.shape
    ya = torch.empty_like(xa)
    prow = B.alloc_planes(B.MX9, ra, ca, B.AXIS_ROW)
    pcol = B.alloc_planes(B.MX9, ra, ca, B.AXIS_COL)
    fh, fr = B.fmt(32, 2, 1, 4), B.fmt(32, 4, 2, 4)
    ph, pr = B.alloc_planes(fh, rows, cols), B.alloc_planes(fr, rows, cols)
    rows_t, cols_t, n_look = 1 << 20, 128, 1 << 20
    g = torch.Generator(device="cuda").manual_seed(7)
    tab = torch.randn(rows_t, cols_t, generator=g, device="cuda") * 0.05
    pt = B.bdr_quantize(B.MX6, tab)
    del tab
    idx = torch.randint(0, rows_t, (n_look,), generator=g, device="cuda", dtype=torch.int64)
    yo = torch.empty(n_look, cols_t, device="cuda")
    tb = B.bdr_table_pack(B.MX6, pt, rows_t, cols_t)
    img = torch.empty(B.mx_operand_bytes(B.MX6, ra, ca), dtype=torch.uint8, device="cuda")
    img9 = torch.empty(B.mx_operand_bytes(B.MX9, ra, ca, B.OPERAND_BF16), dtype=torch.uint8, device="cuda")
    img4 = torch.empty(B.mx_operand_bytes(B.MX4, ra, ca, B.OPERAND_FP4), dtype=torch.uint8, device="cuda")
    img4t = torch.empty(B.mx_operand_bytes(B.MX4, ca, ra, B.OPERAND_FP4), dtype=torch.uint8, device="cuda")
    # a decoding step's product: 16 rows against the image of an [8192 x 8192] weight (a slice of the
    # activation tensor: any values do)
    wsrc = xa[:, :8192].float()                            # [8192 x 8192] as a weight [N x K] (FP32 source:
    #                                                        these set-up launches are not the probed kernels)
    wimg6 = B.bdr_quantize_operand(B.MX6, wsrc, image=B.OPERAND_FP6, b_operand=True)
    wimg4 = B.bdr_quantize_operand(B.MX4, wsrc, image=B.OPERAND_FP4, b_operand=True)
    a16 = wsrc[:16].contiguous()
    aimg6 = B.bdr_quantize_operand(B.MX6, a16, image=B.OPERAND_FP6)
    aimg4 = B.bdr_quantize_operand(B.MX4, a16, image=B.OPERAND_FP4)
    c16 = torch.empty(16, 8192, device="cuda")
    wpl9 = B.bdr_quantize(B.MX9, wsrc)                     # the same weight as MX9 planes
    apl9 = B.bdr_quantize(B.MX9, a16)
    gws9 = torch.empty(B.mx_gemm_workspace_bytes(16, 8192, 8192), dtype=torch.uint8, device="cuda")
    xc = x.view(-1)[:8192 * 8192].view(8192, 8192)   # a square slice for the column-wise general kernel
    yc = y.view(-1)[:8192 * 8192].view(8192, 8192)
    pc = B.alloc_planes(fh, 8192, 8192, B.AXIS_COL)
    for _ in range(3):
        y.copy_(x)
        B.bdr_quantize(B.MX9, xa, axis=B.AXIS_COL, out=pcol)
        B.bdr_dequantize(B.MX9, pcol, ra, ca, axis=B.AXIS_COL, out=ya)
        B.bdr_quantize_dequantize(B.MX9, xa, axis=B.AXIS_COL, out=ya)
        B.bdr_quantize(B.MX9, xa, axis=B.AXIS_ROW, out=prow)
        B.bdr_dequantize(B.MX9, prow, ra, ca, axis=B.AXIS_ROW, out=ya)
        B.bdr_gather_dequantize(B.MX6, pt, rows_t, cols_t, idx, out=yo)
        B.bdr_table_gather_dequantize(B.MX6, tb, rows_t, cols_t, idx, out=yo)
        B.bdr_quantize_operand(B.MX6, xa, axis=B.AXIS_ROW, out=img)
        B.bdr_quantize_operand(B.MX6, xa, axis=B.AXIS_COL, out=img)
        B.bdr_quantize_operand(B.MX9, xa, axis=B.AXIS_ROW, image=B.OPERAND_BF16, out=img9)
        B.bdr_quantize_operand(B.MX9, xa, axis=B.AXIS_COL, image=B.OPERAND_BF16, out=img9)
        B.bdr_quantize_operand(B.MX4, xa, axis=B.AXIS_ROW, image=B.OPERAND_FP4, out=img4)
        B.bdr_quantize_operand(B.MX4, xa, axis=B.AXIS_COL, image=B.OPERAND_FP4, out=img4t)
        B.mx_gemm_operands(B.MX6, B.MX6, aimg6, wimg6, 16, 8192, 8192, image=B.OPERAND_FP6, out=c16)
        B.mx_gemm_operands(B.MX4, B.MX4, aimg4, wimg4, 16, 8192, 8192, image=B.OPERAND_FP4, out=c16)
        B.mx_gemm(B.MX9, B.MX9, apl9, wpl9, 16, 8192, 8192, out=c16, workspace=gws9)   # B streamed from its planes
        B.bdr_quantize(fh, x, out=ph)
        B.bdr_dequantize(fh, ph, rows, cols, out=y)
        B.bdr_quantize(fr, x, out=pr)
        B.bdr_dequantize(fr, pr, rows, cols, out=y)
        B.bdr_quantize(fh, xc, axis=B.AXIS_COL, out=pc)
        B.bdr_dequantize(fh, pc, 8192, 8192, axis=B.AXIS_COL, out=yc)
    torch.cuda.synchronize()
    print(json.dumps({"aux_probe": "3 x (1 GiB copy; MX9 bf16 8192x12288 column quantize, dequantize, fused, "
                                   "row quantize, dequantize; MX6 gather 2^20 x 128 from planes and from the table image; the same "
                                   "bf16 tensor to the MX6 (FP6), MX9 (BF16) and MX4 (FP4) operand images, row and column blocks; the product of 16 rows with an 8192 x 8192 MX6 (FP6) and MX4 (FP4) image and with MX9 planes; k1 32 k2 2 d2 1 m 4 and "
                                   "k1 32 k2 4 d2 2 m 4 quantize, dequantize on 1 GiB fp32; k1 32 k2 2 d2 1 m 4 "
                                   "column quantize, dequantize on 8192 x 8192 fp32)"}))


def profile_commit(path):
    """The commit a summary under profiles/ says it was taken at (a line `commit: <hash>`)."""
    try:
        for line in open(path):
            if line.startswith("commit:"):
                return line.split(":", 1)[1].split()[0]
    except OSError:
        pass
    return None


UTIL_PROFILE = os.path.join(ROOT, "profiles", "mx_gemm_and_sweep_unit_utilisation.txt")


def profiled_util(kernel_prefix, column):
    """MfmaUtil (column -2) or VALUBusy (column -1), in percent, of a kernel from the committed
    rocprofv3 summary (not measured in this run; `profile_commit` says when it was), or None."""
    try:
        with open(UTIL_PROFILE) as fh:
            for line in fh:
                if line.startswith(kernel_prefix):
                    return float(line.split()[column])
    except (OSError, ValueError, IndexError):
        pass
    return None


def profiled_mfma_util(kernel_prefix):
    return profiled_util(kernel_prefix, -2)


def measured_traffic(label):
    """(HBM bytes per launch, commit) of one of the six kernels of the step, e.g.
    "dequantize_MX9", from the committed rocprofv3 --pmc summary (profiles/), else (None, None)."""
    path = os.path.join(ROOT, "profiles", "mx_rowwise_f32_1GiB_traffic.txt")
    op, fm = label.split("_")
    key = "traffic_bytes_per_launch[%s_%s]" % (fm.lower(), op)
    try:
        for line in open(path):
            if line.startswith(key):
                return float(line.split("=")[1]), profile_commit(path)
    except OSError:
        pass
    return None, None


def other_legs(B, S, torch, timed):
    """QSNR sweep (configs/s), activation-shaped bf16 row/column quantize, mx_gemm (TFLOP/s)."""
    out = {}
    try:
        xs = S.sweep(device="cuda")
        fmts = [B.fmt(k1, k1 if k2 == 0 else k2, d2, m) for k1 in (8, 16, 32, 64)
                for k2 in (1, 2, 4, 0) for d2 in (0, 1) for m in (2, 4)]
        ws = torch.empty(B.lib.bdr_qsnr_sweep_workspace_bytes(len(fmts)), dtype=torch.uint8, device="cuda")
        res = (torch.empty(64, dtype=torch.float64, device="cuda"),
               torch.empty(65, dtype=torch.float64, device="cuda"))
        t = timed(lambda: B.bdr_qsnr_sweep(fmts, xs, workspace=ws, out=res))
        out["qsnr_sweep_64fmt_16Mi"] = {
            "ms": round(t, 4), "configs_per_s": round(64 / (t * 1e-3), 1),
            "Gelem_configs_per_s": round(64 * xs.numel() / (t * 1e-3) / 1e9, 1),
            "distinct_quantizers": 32,
            "valu_busy_pct_rocprofv3": profiled_util("sweep_kernel<float,true>", -1),
            # QSNR (dB) per format, in the order k1 (8, 16, 32, 64) x k2 (1, 2, 4, k1) x d2 (0, 1) x m (2, 4)
            "qsnr_db": [round(v, 3) for v in res[0].cpu().tolist()]}
        del xs
        # a sweep of the size of the paper's design-space exploration ("800+ configurations",
        # Sec. IV) on its workload (Gaussian vectors of varying variance, 16384 x 256)
        xd = S.design_space(device="cuda")
        big = [B.fmt(k1, k2, d2, m) for k1 in (8, 16, 32, 64, 128, 256) for k2 in (1, 2, 4, 8, 16)
               if k2 <= k1 for d2 in (0, 1, 2, 3) for m in range(2, 9)]
        wsb = torch.empty(B.lib.bdr_qsnr_sweep_workspace_bytes(len(big)), dtype=torch.uint8, device="cuda")
        resb = (torch.empty(len(big), dtype=torch.float64, device="cuda"),
                torch.empty(len(big) + 1, dtype=torch.float64, device="cuda"))
        t = timed(lambda: B.bdr_qsnr_sweep(big, xd, workspace=wsb, out=resb), reps=7, inner=3)
        qs = resb[0].cpu()
        out["qsnr_sweep_%dfmt_design_space_4Mi" % len(big)] = {
            "ms": round(t, 4), "configs_per_s": round(len(big) / (t * 1e-3), 1),
            "Gelem_configs_per_s": round(len(big) * xd.numel() / (t * 1e-3) / 1e9, 1),
            "qsnr_db_min": round(qs.min().item(), 3), "qsnr_db_max": round(qs.max().item(), 3)}
        del xd
    except B.BdrError as e:
        out["qsnr_sweep_64fmt_16Mi"] = {"error": str(e)}
    try:
        # formats of the design-space sweep other than Table II's, as storage formats (Sec. IV):
        # 1 GiB fp32, quantize then dequantize in a loop, an event after every launch (so each
        # kernel runs against cold planes, as in the headline step)
        xg = S.bandwidth(N_ELEMS, COLS, device="cuda")
        yg = torch.empty_like(xg)
        r, c = xg.shape
        leg = {}
        for label, f in (("k1_32_k2_2_d2_1_m4", B.fmt(32, 2, 1, 4)), ("k1_64_k2_4_d2_1_m2", B.fmt(64, 4, 1, 2)),
                         ("k1_8_k2_1_d2_1_m4", B.fmt(8, 1, 1, 4)), ("bfp_k1_16_m4", B.fmt(16, 16, 0, 4)),
                         ("run_time_tuple_k1_32_k2_4_d2_2_m4", B.fmt(32, 4, 2, 4))):
            pl = B.alloc_planes(f, r, c)
            fbits = (f.m + 1) + 8.0 / f.k1 + float(f.d2) / f.k2
            ab = alg_bytes(N_ELEMS, fbits)
            tq, td = [], []
            for it in range(23):
                e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
                e[0].record()
                B.bdr_quantize(f, xg, out=pl)
                e[1].record()
                B.bdr_dequantize(f, pl, r, c, out=yg)
                e[2].record()
                e[2].synchronize()
                if it >= 3:
                    tq.append(e[0].elapsed_time(e[1]))
                    td.append(e[1].elapsed_time(e[2]))
            tq, td = median(tq), median(td)
            leg[label] = {"bits_per_element": fbits,
                          "quantize_us": round(tq * 1e3, 1), "quantize_frac": round(ab / tq / 1e6 / HBM_PEAK_GBS, 4),
                          "dequantize_us": round(td * 1e3, 1), "dequantize_frac": round(ab / td / 1e6 / HBM_PEAK_GBS, 4)}
            del pl
        out["general_formats_fp32_1GiB_rowwise"] = leg
        del xg, yg
    except B.BdrError as e:
        out["general_formats_fp32_1GiB_rowwise"] = {"error": str(e)}
    try:
        # the same kind of format blocked down the columns (the tiled general kernel): fp32
        # 8192 x 8192, two inputs in rotation, quantize and dequantize timed separately
        xc = [S.gemm_operands(8192, 8, 8192, device="cuda", seed=40 + i)[0] for i in range(2)]
        r, c = xc[0].shape
        yc = torch.empty_like(xc[0])
        leg = {}
        for label, f, fbits in (("k1_32_k2_2_d2_1_m_4", B.fmt(32, 2, 1, 4), 5 + 8 / 32 + 1 / 2),
                                ("bfp_k1_16_m_4", B.fmt(16, 16, 0, 4), 5 + 8 / 16)):
            ab = alg_bytes(r * c, fbits, 4)
            pl = B.alloc_planes(f, r, c, B.AXIS_COL)
            k = [0]

            def runq():
                B.bdr_quantize(f, xc[k[0] % 2], axis=B.AXIS_COL, out=pl)
                k[0] += 1
            tq = timed(runq, reps=7, inner=3)
            td = timed(lambda: B.bdr_dequantize(f, pl, r, c, axis=B.AXIS_COL, out=yc), reps=7, inner=3)
            leg[label] = {"quantize_us": round(tq * 1e3, 1), "quantize_frac": round(ab / tq / 1e6 / HBM_PEAK_GBS, 4),
                          "dequantize_us": round(td * 1e3, 1), "dequantize_frac": round(ab / td / 1e6 / HBM_PEAK_GBS, 4)}
            del pl
        out["general_formats_fp32_8192x8192_colwise"] = leg
        del xc, yc
    except B.BdrError as e:
        out["general_formats_fp32_8192x8192_colwise"] = {"error": str(e)}
    try:
        # three buffers in rotation so the 192 MiB input is not served from the 256 MB cache
        xa = [S.activation(device="cuda", seed=3 + i) for i in range(3)]
        r, c = xa[0].shape
        ab = alg_bytes(r * c, 9, 2)
        leg = {}
        for axis, name in ((B.AXIS_ROW, "row"), (B.AXIS_COL, "col")):
            pl = B.alloc_planes(B.MX9, r, c, axis)
            k = [0]

            def run():
                B.bdr_quantize(B.MX9, xa[k[0] % 3], axis=axis, out=pl)
                k[0] += 1
            t = timed(run, reps=7, inner=6, warm=40)   # (the first launches after a change of kernel run at the clock the previous leg left)
            leg[name] = {"us": round(t * 1e3, 1), "GBps": round(ab / t / 1e6, 1),
                         "frac": round(ab / t / 1e6 / HBM_PEAK_GBS, 4)}
        out["activation_bf16_8192x12288_MX9"] = leg
        # the same tensor quantized straight into an operand image of the product kernels: MX6 into
        # the FP6 image (2 bytes read, 1 written per element), MX9 into the BF16 image (2 and 2),
        # blocks along rows / down columns
        # MX4 into the FP4 image (2 read, 1/2 + 1/16 written)
        for fmt, image, nbytes, key in ((B.MX6, B.OPERAND_FP6, 3, "activation_bf16_8192x12288_MX6_operand_image"),
                                        (B.MX9, B.OPERAND_BF16, 4, "activation_bf16_8192x12288_MX9_operand_image"),
                                        (B.MX4, B.OPERAND_FP4, 2.5625, "activation_bf16_8192x12288_MX4_operand_image_fp4")):
            legi = {}
            abi = r * c * nbytes
            for axis, name in ((B.AXIS_ROW, "row"), (B.AXIS_COL, "col")):
                rows_i, k_i = (r, c) if axis == B.AXIS_ROW else (c, r)
                img = torch.empty(B.mx_operand_bytes(fmt, rows_i, k_i, image), dtype=torch.uint8, device="cuda")
                k = [0]

                def runo():
                    B.bdr_quantize_operand(fmt, xa[k[0] % 3], axis=axis, image=image, out=img)
                    k[0] += 1
                t = timed(runo, reps=7, inner=6)
                legi[name] = {"us": round(t * 1e3, 1), "GBps": round(abi / t / 1e6, 1),
                              "frac": round(abi / t / 1e6 / HBM_PEAK_GBS, 4)}
            out[key] = legi
        del xa
    except B.BdrError as e:
        out["activation_bf16_8192x12288_MX9"] = {"error": str(e)}
    try:
        M = N = K = 8192
        A, Bm = S.gemm_operands(M, N, K, device="cuda")
        pa, pb = B.bdr_quantize(B.MX6, A), B.bdr_quantize(B.MX6, Bm)
        C = torch.empty(M, N, device="cuda")
        ws = torch.empty(B.mx_gemm_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
        leg = {}
        # two-pass form (MX6: operands rewritten once as block-scaled FP6, FP6 matrix instructions
        # with one block of 16 per 32-wide hardware block, so at most half of the FP6 peak) and
        # single-kernel form (BF16 in LDS, BF16 matrix instructions)
        for name, w, peak, key in (("two_pass", ws, 10100.0, "frac_of_fp6_mfma_peak_10100"),
                                   ("single_kernel", None, 2500.0, "frac_of_bf16_mfma_peak_2500")):
            # matrix-core clocks take about 30 ms of load to settle: 40 untimed calls first
            t = timed(lambda: B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K, out=C, workspace=w),
                      reps=5, inner=4, warm=40)
            tf = 2.0 * M * N * K / (t * 1e-3) / 1e12
            leg[name] = {"ms": round(t, 3), "TFLOPs": round(tf, 1), key: round(tf / peak, 4)}
        leg["two_pass"]["matrix_instruction"] = "fp6 block-scaled, 16 of 32 K positions used"
        # k1 = 16 against a hardware scale group of 32: half of each instruction multiplies zeros
        leg["two_pass"]["frac_of_usable_half_of_fp6_peak"] = round(leg["two_pass"]["TFLOPs"] / 5050.0, 4)
        leg["single_kernel"]["matrix_instruction"] = "bf16"
        leg["two_pass"]["mfma_util_pct_rocprofv3"] = profiled_mfma_util("gemm_ring_kernel<2,4,4,2,FP6>")
        leg["single_kernel"]["mfma_util_pct_rocprofv3"] = profiled_mfma_util("mx_gemm_kernel<4,4,2,4,4,2>")
        # fidelity of C against the product of the unquantized operands (library FP32 GEMM)
        B.mx_gemm(B.MX6, B.MX6, pa, pb, M, N, K, out=C, workspace=ws)
        Cfp = A @ Bm.t()
        leg["qsnr_db_vs_fp32_gemm"] = round(
            (10 * torch.log10(Cfp.double().square().sum() / (C.double() - Cfp.double()).square().sum())).item(), 3)
        out["mx_gemm_8192_MX6"] = leg
        # MX9 needs 8 significant bits: the two-pass form expands to BF16
        p9a, p9b = B.bdr_quantize(B.MX9, A), B.bdr_quantize(B.MX9, Bm)
        t = timed(lambda: B.mx_gemm(B.MX9, B.MX9, p9a, p9b, M, N, K, out=C, workspace=ws),
                  reps=5, inner=4, warm=40)
        tf = 2.0 * M * N * K / (t * 1e-3) / 1e12
        q9 = (10 * torch.log10(Cfp.double().square().sum() / (C.double() - Cfp.double()).square().sum())).item()
        out["mx_gemm_8192_MX9"] = {"two_pass": {"ms": round(t, 3), "TFLOPs": round(tf, 1),
                                                "frac_of_bf16_mfma_peak_2500": round(tf / 2500.0, 4),
                                                "matrix_instruction": "bf16",
                                                "mfma_util_pct_rocprofv3": profiled_mfma_util("gemm_ring_kernel<2,4,4,2,BF16>")},
                                   "qsnr_db_vs_fp32_gemm": round(q9, 3)}
        del p9a, p9b
        # context only, not part of the path: the library's own BF16 product of the same
        # (unquantized) operands on this machine, C in BF16 -- what the chip grants a BF16 GEMM today
        Ah, Bh = A.to(torch.bfloat16), Bm.to(torch.bfloat16)
        Ch = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
        tl = timed(lambda: torch.matmul(Ah, Bh.t(), out=Ch), reps=5, inner=4, warm=40)
        out["mx_gemm_8192_MX9"]["library_bf16_gemm_for_context"] = {
            "ms": round(tl, 3), "TFLOPs": round(2.0 * M * N * K / (tl * 1e-3) / 1e12, 1)}
        del Ah, Bh, Ch
        # MX4 x MX4: the two-pass form uses block-scaled FP4 images (half the operand bytes)
        p4a, p4b = B.bdr_quantize(B.MX4, A), B.bdr_quantize(B.MX4, Bm)
        t = timed(lambda: B.mx_gemm(B.MX4, B.MX4, p4a, p4b, M, N, K, out=C, workspace=ws),
                  reps=5, inner=4, warm=40)
        tf = 2.0 * M * N * K / (t * 1e-3) / 1e12
        q4 = (10 * torch.log10(Cfp.double().square().sum() / (C.double() - Cfp.double()).square().sum())).item()
        out["mx_gemm_8192_MX4"] = {"two_pass": {"ms": round(t, 3), "TFLOPs": round(tf, 1),
                                                "frac_of_fp4_mfma_peak_10100": round(tf / 10100.0, 4),
                                                "frac_of_usable_half_of_fp4_peak": round(tf / 5050.0, 4),
                                                "matrix_instruction": "fp4 block-scaled, 16 of 32 K positions used",
                                                "mfma_util_pct_rocprofv3": profiled_mfma_util("gemm_ring_kernel<2,4,4,2,FP4>")},
                                   "qsnr_db_vs_fp32_gemm": round(q4, 3)}
        del p4a, p4b, Cfp
    except B.BdrError as e:
        out["mx_gemm_8192_MX6"] = {"error": str(e)}
    try:
        # the paper's own dot-product pipeline (Sec. IV-B), modelled bit for bit: how far is the
        # FP32-accumulating matrix-core path from it?  Both add the same exact products; the
        # reference is the FP64 product of the dequantized operands.
        M = N = K = 8192
        A, Bm = S.gemm_operands(M, N, K, device="cuda")
        C = torch.empty(M, N, device="cuda")
        ws = torch.empty(B.mx_gemm_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
        leg = {}
        for name, f in (("MX6", B.MX6), ("MX9", B.MX9)):
            pa, pb = B.bdr_quantize(f, A), B.bdr_quantize(f, Bm)
            ref = B.bdr_dequantize(f, pa, M, K).double() @ B.bdr_dequantize(f, pb, N, K).double().t()
            sig = ref.square().sum()

            def acc_qsnr(c):
                err = (c.double() - ref).square().sum().item()
                # no error at all (every sum exactly representable): reported as the string "exact"
                return round(10 * math.log10(sig.item() / err), 2) if err > 0 else "exact"
            ent = {}
            for r in (64, K):
                t = timed(lambda: B.mx_dot_pipeline(f, f, pa, pb, M, N, K, r=r, f_bits=25, out=C, workspace=ws),
                          reps=5, inner=4, warm=2)
                ent["r_%d" % r] = {"ms": round(t, 3), "TFLOPs_equivalent": round(2.0 * M * N * K / (t * 1e-3) / 1e12, 1),
                                   "qsnr_db_vs_fp64_product": acc_qsnr(C)}
            B.mx_gemm(f, f, pa, pb, M, N, K, out=C, workspace=ws)
            ent["mx_gemm_two_pass_qsnr_db_vs_fp64_product"] = acc_qsnr(C)
            B.mx_gemm(f, f, pa, pb, M, N, K, out=C)
            ent["mx_gemm_single_kernel_qsnr_db_vs_fp64_product"] = acc_qsnr(C)
            leg[name] = ent
            del pa, pb, ref
        leg["f_bits"] = 25
        # ALU-bound: about 6.1 vector-ALU lane-ops per entry of C and block of K (counted in the
        # kernel's code: 392 wave instructions per K step of 4 blocks and 16 entries per lane)
        # against 256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-ops/s
        lane_ops = 6.1 * M * N * (K // 16)
        roof_ms = lane_ops / 39.3e12 * 1e3
        leg["roofline"] = {"bound": "alu", "unit": "T lane-op/s", "peak": 39.3,
                           "lane_ops_per_entry_and_block": 6.1, "time_at_peak_ms": round(roof_ms, 3),
                           "achieved": round(lane_ops / (leg["MX6"]["r_%d" % K]["ms"] * 1e-3) / 1e12, 2),
                           "frac": round(roof_ms / leg["MX6"]["r_%d" % K]["ms"], 4),
                           "of": "MX6, one pass (r = K)"}
        out["mx_dot_pipeline_8192"] = leg
        del A, Bm, C, ws
    except B.BdrError as e:
        out["mx_dot_pipeline_8192"] = {"error": str(e)}
    try:
        # embedding-table lookups from MX6 storage (Sec. V): 2^20 rows x 128, 2^20 random rows
        rows_t, cols_t, n_look = 1 << 20, 128, 1 << 20
        g = torch.Generator(device="cuda").manual_seed(7)
        tab = torch.randn(rows_t, cols_t, generator=g, device="cuda") * 0.05
        pt = B.bdr_quantize(B.MX6, tab)
        del tab
        idx = torch.randint(0, rows_t, (n_look,), generator=g, device="cuda", dtype=torch.int64)
        yo = torch.empty(n_look, cols_t, device="cuda")
        t = timed(lambda: B.bdr_gather_dequantize(B.MX6, pt, rows_t, cols_t, idx, out=yo), reps=5, inner=5)
        ab = n_look * (cols_t * 6 // 8 + 8 + cols_t * 4)
        out["gather_dequantize_MX6_1Mi_rows_x128_fp32"] = {
            "us": round(t * 1e3, 1), "GBps": round(ab / t / 1e6, 1),
            "frac": round(ab / t / 1e6 / HBM_PEAK_GBS, 4), "lookups_per_s": round(n_look / (t * 1e-3), 1)}
        # the same lookups from the table image that keeps a row's 96 bytes together
        tb = B.bdr_table_pack(B.MX6, pt, rows_t, cols_t)
        t = timed(lambda: B.bdr_table_gather_dequantize(B.MX6, tb, rows_t, cols_t, idx, out=yo), reps=5, inner=5)
        out["gather_dequantize_MX6_1Mi_rows_x128_fp32"]["rows_kept_together"] = {
            "us": round(t * 1e3, 1), "GBps": round(ab / t / 1e6, 1),
            "frac": round(ab / t / 1e6 / HBM_PEAK_GBS, 4), "lookups_per_s": round(n_look / (t * 1e-3), 1)}
        del pt, idx, yo, tb
    except B.BdrError as e:
        out["gather_dequantize_MX6_1Mi_rows_x128_fp32"] = {"error": str(e)}
    try:
        # the three products of one training iteration of a GPT3-width linear layer (Sec. V):
        # 6 quantizations (row- and column-wise) and 3 mx_gemm calls on BF16 tensors
        from paper_2302_08007_amd.training import mx_linear
        T, I, Osz = 8192, 12288, 12288
        g = torch.Generator(device="cuda").manual_seed(6)
        x = torch.randn(T, I, generator=g, device="cuda").to(torch.bfloat16).requires_grad_()
        w = (torch.randn(Osz, I, generator=g, device="cuda") / I ** 0.5).to(torch.bfloat16).requires_grad_()
        gy = torch.randn(T, Osz, generator=g, device="cuda").to(torch.bfloat16)

        for name, f, peak, key in (("MX9", B.MX9, 2500.0, "frac_of_bf16_mfma_peak_2500"),
                                   ("MX6", B.MX6, 10100.0, "frac_of_fp6_mfma_peak_10100"),
                                   ("MX4", B.MX4, 10100.0, "frac_of_fp4_mfma_peak_10100")):
            def step_fn():
                x.grad = None
                w.grad = None
                mx_linear(x, w, f).backward(gy)
            t = timed(step_fn, reps=10, inner=2, warm=8)
            tf = 3 * 2.0 * T * I * Osz / (t * 1e-3) / 1e12
            out["mx_linear_fwd_bwd_8192x12288x12288_%s_bf16" % name] = {
                "ms": round(t, 3), "TFLOPs": round(tf, 1), key: round(tf / peak, 4)}
        # direct-cast inference (Sec. V, "Inferencing"): the weight's operand image is made once,
        # a call quantizes the 8192 x 12288 BF16 activations into theirs and multiplies
        from paper_2302_08007_amd.training import MXWeight, mx_linear_inference
        leg = {}
        for an, wn in (("MX9", "MX9"), ("MX6", "MX6"), ("MX6", "MX4"), ("MX4", "MX4")):
            wq = MXWeight(w.detach(), getattr(B, wn))
            fa = getattr(B, an)
            with torch.no_grad():
                t = timed(lambda: mx_linear_inference(x, wq, fa), reps=10, inner=2, warm=12)
            leg["act_%s_weight_%s" % (an, wn)] = {"ms": round(t, 3), "TFLOPs": round(2.0 * T * I * Osz / (t * 1e-3) / 1e12, 1)}
            del wq
        out["mx_linear_inference_8192x12288x12288_bf16"] = leg
        # a decoding step: 16 tokens against the same weight (its image made once); the product is a
        # stream over the weight image, so its bytes set the time -- BF16 image 2 bytes per element,
        # FP6 1, FP4 9/16; the library's BF16 product of the unquantized tensors for context
        leg = {}
        x16 = x.detach()[:16].contiguous()
        y16 = torch.empty(16, Osz, device="cuda", dtype=torch.bfloat16)
        with torch.no_grad():
            for an, wn in (("MX9", "MX9"), ("MX6", "MX6"), ("MX4", "MX4")):
                wq = MXWeight(w.detach(), getattr(B, wn))
                fa = getattr(B, an)
                t = timed(lambda: mx_linear_inference(x16, wq, fa), reps=7, inner=10, warm=20)
                img_bytes = sum(v.numel() for v in wq._images.values())
                leg["act_%s_weight_%s" % (an, wn)] = {"us": round(t * 1e3, 1), "weight_image_MB": round(img_bytes / 1e6, 1),
                                                      "weight_image_GBps": round(img_bytes / t / 1e6, 1)}
                del wq
            # MX9 weights kept as they are stored (three planes, 9 bits per element): the step quantizes
            # the tokens to planes and mx_gemm streams the weight planes, expanding them in registers
            wp = B.bdr_quantize(B.MX9, w.detach())
            gws = torch.empty(B.mx_gemm_workspace_bytes(16, Osz, I), dtype=torch.uint8, device="cuda")
            c16 = torch.empty(16, Osz, device="cuda", dtype=torch.bfloat16)

            def from_planes():
                B.mx_gemm(B.MX9, B.MX9, B.bdr_quantize(B.MX9, x16), wp, 16, Osz, I, out=c16, workspace=gws)
            t = timed(from_planes, reps=7, inner=10, warm=20)
            pbytes = sum(p.numel() for p in wp)
            leg["act_MX9_weight_MX9_from_planes"] = {"us": round(t * 1e3, 1), "weight_planes_MB": round(pbytes / 1e6, 1),
                                                     "weight_planes_GBps": round(pbytes / t / 1e6, 1)}
            del wp, gws, c16
            wd = w.detach()
            t = timed(lambda: torch.matmul(x16, wd.t(), out=y16), reps=7, inner=10, warm=20)
            leg["library_bf16_gemm_for_context"] = {"us": round(t * 1e3, 1), "weight_MB": round(wd.numel() * 2 / 1e6, 1)}
        out["mx_linear_decode_16_tokens_12288x12288_bf16"] = leg
    except B.BdrError as e:
        out["mx_linear_fwd_bwd_8192x12288x12288_MX9_bf16"] = {"error": str(e)}
    return out


if __name__ == "__main__":
    main()
