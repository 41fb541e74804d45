#!/usr/bin/env python3
"""Benchmark of the weight-stationary recurrence matmul on one MI355X.

A step is one pass of the whole hot path (load the stationary A, stream B, run the k chains,
emit C) over one synthetic workload, i.e. one call of the C ABI.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu] [--no-extra]
                  [--copy-calibration]

NAME is one of the five matmul workloads (default c3_bf16_8192), k1_bf16_tallk (few output blocks, long k: the
k-in-space kernel variant), t1_trsm_8192 (the tiled triangular solve), h1_chol_8192 (the tiled Cholesky
factorisation) or f1_attn_4096 (the attention tile recurrence).  Whatever the headline, the others are measured
after it and reported under "workloads" (--no-extra: none of them; --matmul-only: only the five).

The headline workload is the 8192^3 bf16 case (compute bound, MFMA roofline); the int8 8192^3
and the batched narrow-stream cases are measured after it and reported under "workloads".
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

# published MI355X peaks used for the roofline fractions
PEAK = {"bf16": (2500.0, "TFLOP/s"), "i8": (5000.0, "TOP/s")}
HBM_PEAK_GBS = 8000.0
ROTATE = 3     # distinct (A, B, C) sets cycled through, so operands are not served from cache
# HBM-side bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what the same
# counter reads for a 1 GiB device copy (fetch x2.000, write x1.000); measured with the command lines
# recorded in profiles/bench_all_workloads.md.  None where not measured.
TRAFFIC_BYTES = {"c3_bf16_8192": 1926994252, "c4_i8_8192": 1119826627, "c5_bf16_narrow": 4386214339,
                 "c2_bf16_512": 4332367, "c1_i8_64": 52670}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3_bf16_8192")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-extra", action="store_true", help="measure only the headline workload")
    ap.add_argument("--matmul-only", action="store_true",
                    help="beside the headline, measure only the other matmul workloads (no triangular solve, Cholesky, attention)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one 1 GiB device copy (reference point for HBM traffic counters)")
    return ap.parse_args()


def measure(lib, torch, w, steps, warmup, sets):
    """Time `steps` launches; returns (wall ms per step, mean kernel ms by events, kernel name)."""
    from datagen import ws_inputs
    dev = "cuda:0"
    data = []
    for r in range(sets):
        wr = ws_inputs.Workload(w.name, w.dtype, w.batch, w.M, w.K, w.N, w.dist, w.param, w.seed + 1000 * r)
        A, B = ws_inputs.make_inputs(wr, dev)
        cshape = (w.batch, w.M, w.N) if w.batch > 1 else (w.M, w.N)
        C = torch.empty(cshape, dtype=torch.int32 if w.dtype == "i8" else torch.float32, device=dev)
        data.append((A, B, C))
    A, B, C = data[0]
    dt = lib.CYC_I8_I32 if w.dtype == "i8" else lib.CYC_BF16_F32
    kname = lib.cyc_kernel_name(A.data_ptr(), B.data_ptr(), C.data_ptr(), w.batch, w.M, w.K, w.N,
                                w.M * w.K, w.K * w.N, w.M * w.N, dt)
    stream = torch.cuda.current_stream()

    def step(i):
        a, b, c = data[i % sets]
        st = lib.cyc_recurrence_matmul_batched(a.data_ptr(), b.data_ptr(), c.data_ptr(), w.batch, w.M, w.K, w.N,
                                               w.M * w.K, w.K * w.N, w.M * w.N, dt, stream.cuda_stream)
        if st != 0:
            raise RuntimeError(lib.cyc_status_string(st))

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # the library is launched on torch's current stream, so torch events bracket its kernels
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for i, (e0, e1) in enumerate(evs):
        e0.record(stream)
        step(i)
        e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    kern_ms = sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps
    del data
    torch.cuda.empty_cache()
    return wall_ms, kern_ms, kname


def measure_trsm(lib, torch, w, steps, warmup, sets):
    """Time `steps` tiled triangular solves (each a sequence of kernels); returns (wall ms, event ms)."""
    from datagen import ws_inputs
    dev = "cuda:0"
    data = []
    for r in range(sets):
        wr = ws_inputs.TriWorkload(w.name, w.n, w.nrhs, w.nb, w.seed + 1000 * r)
        L, B = ws_inputs.make_tri_inputs(wr, dev)
        X = torch.empty((w.n, w.nrhs), dtype=torch.float32, device=dev)
        Xh = torch.empty((w.n, w.nrhs), dtype=torch.bfloat16, device=dev)
        data.append((L, B, X, Xh))
    stream = torch.cuda.current_stream()

    def step(i):
        L, B, X, Xh = data[i % sets]
        st = lib.cyc_recurrence_trsm(L.data_ptr(), B.data_ptr(), X.data_ptr(), Xh.data_ptr(), w.n, w.nrhs, w.nb,
                                     stream.cuda_stream)
        if st != 0:
            raise RuntimeError(lib.cyc_status_string(st))

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for i, (e0, e1) in enumerate(evs):
        e0.record(stream)
        step(i)
        e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ev_ms = sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps
    del data
    torch.cuda.empty_cache()
    return wall_ms, ev_ms


def measure_chol(lib, torch, w, steps, warmup, sets):
    """Time `steps` tiled Cholesky factorisations (each a sequence of kernels); returns (wall ms, event ms)."""
    from datagen import ws_inputs
    dev = "cuda:0"
    data = []
    for r in range(sets):
        A = ws_inputs.spd_f32(w.n, w.seed + 1000 * r, 0, dev)
        data.append((A, torch.empty((w.n, w.n), dtype=torch.float32, device=dev),
                     torch.empty((w.n, w.n), dtype=torch.bfloat16, device=dev)))
    stream = torch.cuda.current_stream()

    def step(i):
        A, L, Lh = data[i % sets]
        st = lib.cyc_recurrence_cholesky(A.data_ptr(), L.data_ptr(), Lh.data_ptr(), w.n, w.nb, stream.cuda_stream)
        if st != 0:
            raise RuntimeError(lib.cyc_status_string(st))

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for i, (e0, e1) in enumerate(evs):
        e0.record(stream)
        step(i)
        e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ev_ms = sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps
    del data
    torch.cuda.empty_cache()
    return wall_ms, ev_ms


def measure_attn(lib, torch, w, steps, warmup, sets):
    """Time `steps` attention calls (one kernel each); returns (wall ms, event ms)."""
    from datagen import ws_inputs
    dev = "cuda:0"
    data = []
    for r in range(sets):
        wr = ws_inputs.AttnWorkload(w.name, w.batch, w.N, w.M, w.d, w.seed + 1000 * r)
        Q, K, V = ws_inputs.make_attn_inputs(wr, dev)
        data.append((Q, K, V, torch.empty((w.batch, w.N, w.d), dtype=torch.float32, device=dev)))
    stream = torch.cuda.current_stream()

    def step(i):
        Q, K, V, O = data[i % sets]
        st = lib.cyc_recurrence_attention(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), w.batch, w.N, w.M, w.d,
                                          stream.cuda_stream)
        if st != 0:
            raise RuntimeError(lib.cyc_status_string(st))

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for i, (e0, e1) in enumerate(evs):
        e0.record(stream)
        step(i)
        e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ev_ms = sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps
    del data
    torch.cuda.empty_cache()
    return wall_ms, ev_ms


def attn_entry(w, wall_ms, ev_ms):
    ach = w.ops / (ev_ms * 1e-3) / 1e12
    return {"kernel": "attention", "batch": w.batch, "N": w.N, "M": w.M, "d": w.d, "ms_per_step": round(wall_ms, 5),
            "kernel_ms": round(ev_ms, 5), "achieved": round(ach, 1), "unit": "TFLOP/s", "bound": "mfma",
            "frac": round(ach / PEAK["bf16"][0], 4)}


def bench_attn(lib, torch, w, args):
    """The attention recurrence as the headline workload: one step = one call = one kernel."""
    wall_ms, ev_ms = measure_attn(lib, torch, w, args.steps, args.warmup, ROTATE)
    e = attn_entry(w, wall_ms, ev_ms)
    out = {
        "metric": "recurrence matmul TFLOP/s (TOP/s int8) and % of MI355X MFMA/HBM roofline",
        "value": round(w.ops / 1e12 / (wall_ms * 1e-3), 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "N": w.N, "M": w.M, "d": w.d, "kernel": "attention",
                   "accumulate": "fp32", "seed": w.seed, "operand_sets_rotated": ROTATE},
        "roofline": {"bound": "mfma", "achieved": e["achieved"], "peak": PEAK["bf16"][0], "unit": "TFLOP/s",
                     "frac": e["frac"], "traffic": None, "kernel": "attention", "kernel_ms": e["kernel_ms"]},
    }
    if not args.no_cpu:
        import numpy as np
        from datagen import ws_inputs
        from oracle import attn_oracle, ws_oracle
        elems = min(w.batch, 48)
        wr = ws_inputs.AttnWorkload(w.name, elems, w.N, w.M, w.d, w.seed)
        Q, K, V = ws_inputs.make_attn_inputs(wr, "cpu")
        w64 = lambda t: ws_oracle.bits_to_f64(ws_oracle.bf16_bits(t))
        t0 = time.perf_counter()
        for b in range(elems):
            attn_oracle.attention(w64(Q[b]), w64(K[b]), w64(V[b]))
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(4.0 * elems * w.N * w.M * w.d / dt / 1e12, 6), "unit": "TFLOP/s",
                               "cores": ws_oracle.threads(), "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"attention oracle (fp64 softmax definition) on the first {elems} of the {w.batch} "
                                         f"batch elements of {w.name} (elements are independent), same seed and distribution"}
    return out


def roofline(w, kern_ms):
    # which roofline bounds the workload: its operations per algorithmic byte (A and B read once, C written once)
    # against the chip's ridge, peak operations per second over peak HBM bytes per second
    if w.ops / w.algorithmic_bytes < PEAK[w.dtype][0] * 1e12 / (HBM_PEAK_GBS * 1e9):
        ach = w.algorithmic_bytes / (kern_ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": TRAFFIC_BYTES.get(w.name)}
    peak, unit = PEAK[w.dtype]
    ach = w.ops / (kern_ms * 1e-3) / 1e12
    return {"bound": "mfma", "achieved": round(ach, 1), "peak": peak, "unit": unit,
            "frac": round(ach / peak, 4), "traffic": TRAFFIC_BYTES.get(w.name)}


def cpu_baseline(w, budget_s=15.0):
    """The oracle's row-chain form, as it stands, on a bounded block of the same workload."""
    import numpy as np
    import torch
    from datagen import ws_inputs
    from oracle import ws_oracle
    mode = "i8" if w.dtype == "i8" else "bf16"

    def block(rows, cols):
        wr = ws_inputs.Workload(w.name, w.dtype, 1, rows, w.K, cols, w.dist, w.param, w.seed)
        A, B = ws_inputs.make_inputs(wr, "cpu")
        if mode == "bf16":
            return ws_oracle.bf16_bits(A), ws_oracle.bf16_bits(B)
        return A.numpy(), B.numpy()

    cols = min(w.N, 1024)
    A, B = block(64, cols)
    t0 = time.perf_counter()
    ws_oracle.ws_rowchain(A, B, mode)
    rate = 64 * w.K * cols / max(time.perf_counter() - t0, 1e-6)        # cell-steps per second
    rows = int(min(max(64, rate * budget_s / (w.K * cols)), 8192, max(w.M, 16))) // 16 * 16      # never more rows than A has
    # a batched workload whose single element is over in a fraction of a second: take several elements
    elems = min(w.batch, 8) if rows >= min(w.M, 8192) // 16 * 16 and w.batch > 1 else 1
    blocks = []
    for b in range(elems):
        wr = ws_inputs.Workload(w.name, w.dtype, 1, rows, w.K, cols, w.dist, w.param, w.seed + 1000 * b)
        A, B = ws_inputs.make_inputs(wr, "cpu")
        blocks.append((ws_oracle.bf16_bits(A), ws_oracle.bf16_bits(B)) if mode == "bf16" else (A.numpy(), B.numpy()))
    t0 = time.perf_counter()
    for A, B in blocks:
        ws_oracle.ws_rowchain(A, B, mode)
    dt = time.perf_counter() - t0
    unit = "TOP/s" if mode == "i8" else "TFLOP/s"
    what = (f"a {rows} x {w.K} x {cols} block (first rows of A, first columns of B)" if elems == 1 else
            f"{elems} batch elements of {rows} x {w.K} x {cols} (seeds {w.seed}, {w.seed + 1000}, ...)")
    return {"value": round(2.0 * elems * rows * w.K * cols / dt / 1e12, 6), "unit": unit, "cores": ws_oracle.threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"row-chain oracle on {what} of {w.name}, same distribution"}


def trsm_entry(wt, wall_ms, ev_ms):
    ach = wt.ops / (ev_ms * 1e-3) / 1e12
    return {"kernel": "trsm", "n": wt.n, "nrhs": wt.nrhs, "nb": wt.nb, "ms_per_step": round(wall_ms, 5),
            "kernel_ms": round(ev_ms, 5), "achieved": round(ach, 1), "unit": "TFLOP/s", "bound": "mfma",
            "frac": round(ach / PEAK["bf16"][0], 4)}


def chol_entry(w, wall_ms, ev_ms):
    ach = w.ops / (ev_ms * 1e-3) / 1e12
    return {"kernel": "cholesky", "n": w.n, "nb": w.nb, "ms_per_step": round(wall_ms, 5), "kernel_ms": round(ev_ms, 5),
            "achieved": round(ach, 1), "unit": "TFLOP/s", "bound": "mfma", "frac": round(ach / PEAK["bf16"][0], 4)}


def bench_chol(lib, torch, w, args):
    """The tiled Cholesky factorisation as the headline workload: one step = one factorisation (a sequence of kernels)."""
    wall_ms, ev_ms = measure_chol(lib, torch, w, args.steps, args.warmup, ROTATE)
    e = chol_entry(w, wall_ms, ev_ms)
    out = {
        "metric": "recurrence matmul TFLOP/s (TOP/s int8) and % of MI355X MFMA/HBM roofline",
        "value": round(w.ops / 1e12 / (wall_ms * 1e-3), 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "nb": w.nb, "kernel": "cholesky", "accumulate": "fp32", "seed": w.seed,
                   "operand_sets_rotated": ROTATE},
        # a step is three launches per panel; the figure is the whole step (n^3/3 flops) against the MFMA peak
        "roofline": {"bound": "mfma", "achieved": e["achieved"], "peak": PEAK["bf16"][0], "unit": "TFLOP/s",
                     "frac": e["frac"], "traffic": None, "kernel": "cholesky (all kernels of a step)",
                     "kernel_ms": e["kernel_ms"]},
    }
    if not args.no_cpu:
        from datagen import ws_inputs
        from oracle import chol_oracle, ws_oracle
        reps = 6
        mats = [ws_inputs.spd_f32(w.n, w.seed + 1000 * r, 0, "cpu").numpy() for r in range(reps)]
        t0 = time.perf_counter()
        for A in mats:
            chol_oracle.chol_tiled(A, w.nb)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(reps * w.ops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": ws_oracle.threads(),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"tiled Cholesky oracle on {reps} whole matrices of {w.name} (seeds {w.seed}, "
                                         f"{w.seed + 1000}, ...), same distribution"}
    return out


def bench_trsm(lib, torch, wt, args):
    """The tiled triangular solve as the headline workload: one step = one solve (a sequence of kernels)."""
    wall_ms, ev_ms = measure_trsm(lib, torch, wt, args.steps, args.warmup, ROTATE)
    e = trsm_entry(wt, wall_ms, ev_ms)
    out = {
        "metric": "recurrence matmul TFLOP/s (TOP/s int8) and % of MI355X MFMA/HBM roofline",
        "value": round(wt.ops / 1e12 / (wall_ms * 1e-3), 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wt.name, "n": wt.n, "nrhs": wt.nrhs, "nb": wt.nb, "kernel": "trsm",
                   "accumulate": "fp32", "seed": wt.seed, "operand_sets_rotated": ROTATE},
        # a step is ~255 launches; the figure is the whole step against the MFMA peak, not one kernel's
        "roofline": {"bound": "mfma", "achieved": e["achieved"], "peak": PEAK["bf16"][0], "unit": "TFLOP/s",
                     "frac": e["frac"], "traffic": None, "kernel": "trsm (all kernels of a step)",
                     "kernel_ms": e["kernel_ms"]},
    }
    if not args.no_cpu:
        import numpy as np
        from datagen import ws_inputs
        from oracle import tri_oracle, ws_oracle
        L, B = ws_inputs.make_tri_inputs(wt, "cpu")
        cols = 4096
        Bs = np.ascontiguousarray(B[:, :cols].numpy())
        t0 = time.perf_counter()
        tri_oracle.tri_tiled(ws_oracle.bf16_bits(L), Bs, wt.nb)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(wt.n * (wt.n + 1) * cols / dt / 1e12, 6), "unit": "TFLOP/s",
                               "cores": ws_oracle.threads(), "kind": "oracle", "seconds": round(dt, 2),
                               "sample": f"tiled triangular-solve oracle on the first {cols} right-hand sides of "
                                         f"{wt.name} (columns are independent), same seed and distribution"}
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on exactly one GPU (no collectives, no sharding); got --gpus {args.gpus}",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2511_09987_amd as lib
    from datagen import ws_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(2)
    matmuls = dict(ws_inputs.WORKLOADS, **ws_inputs.KSPACE_WORKLOADS)
    known = (sorted(matmuls) + sorted(ws_inputs.TRI_WORKLOADS) + sorted(ws_inputs.ATTN_WORKLOADS) +
             sorted(ws_inputs.CHOL_WORKLOADS))
    if args.workload not in known:
        print(f"bench.py: unknown workload {args.workload}; choose from {known}", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.workload in ws_inputs.TRI_WORKLOADS:
        print(json.dumps(bench_trsm(lib, torch, ws_inputs.TRI_WORKLOADS[args.workload], args)))
        return
    if args.workload in ws_inputs.ATTN_WORKLOADS:
        print(json.dumps(bench_attn(lib, torch, ws_inputs.ATTN_WORKLOADS[args.workload], args)))
        return
    if args.workload in ws_inputs.CHOL_WORKLOADS:
        print(json.dumps(bench_chol(lib, torch, ws_inputs.CHOL_WORKLOADS[args.workload], args)))
        return

    w = matmuls[args.workload]
    torch.cuda.synchronize()
    wall_ms, kern_ms, kname = measure(lib, torch, w, args.steps, args.warmup, ROTATE)
    unit = "GB/s" if w.N <= 16 else PEAK[w.dtype][1]
    value = (w.algorithmic_bytes / 1e9 if w.N <= 16 else w.ops / 1e12) / (wall_ms * 1e-3)

    out = {
        "metric": "recurrence matmul TFLOP/s (TOP/s int8) and % of MI355X MFMA/HBM roofline",
        "value": round(value, 2), "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "int8", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "M": w.M, "K": w.K, "N": w.N, "kernel": kname,
                   "accumulate": "fp32" if w.dtype == "bf16" else "int32", "seed": w.seed,
                   "operand_sets_rotated": ROTATE},
        "roofline": dict(roofline(w, kern_ms), kernel=kname, kernel_ms=round(kern_ms, 5)),
    }

    if not args.no_extra:
        extra = {}
        names = ("c3_bf16_8192", "c4_i8_8192", "c5_bf16_narrow", "c2_bf16_512", "c1_i8_64")
        for name in names if args.matmul_only else names + tuple(ws_inputs.KSPACE_WORKLOADS):
            if name == w.name:
                continue
            wx = matmuls[name]
            sets = ROTATE if wx.algorithmic_bytes * ROTATE < 40e9 else 1
            wms, kms, kn = measure(lib, torch, wx, args.steps, args.warmup, sets)
            rf = roofline(wx, kms)
            extra[name] = {"kernel": kn, "ms_per_step": round(wms, 5), "kernel_ms": round(kms, 5),
                           "achieved": rf["achieved"], "unit": rf["unit"], "bound": rf["bound"], "frac": rf["frac"]}
        # the tiled triangular solve (a sequence of kernels per step: diagonal-space solves and tri-space GEMMs)
        for name, wt in ({} if args.matmul_only else ws_inputs.TRI_WORKLOADS).items():
            wms, ems = measure_trsm(lib, torch, wt, max(3, args.steps // 5), max(1, args.warmup // 5), ROTATE)
            extra[name] = trsm_entry(wt, wms, ems)
        # the tiled Cholesky factorisation (three launches per panel)
        for name, wc in ({} if args.matmul_only else ws_inputs.CHOL_WORKLOADS).items():
            wms, ems = measure_chol(lib, torch, wc, max(2, args.steps // 4), 1, 2)
            extra[name] = chol_entry(wc, wms, ems)
        # the attention tile recurrence (one kernel per step)
        for name, wa in ({} if args.matmul_only else ws_inputs.ATTN_WORKLOADS).items():
            wms, ems = measure_attn(lib, torch, wa, max(3, args.steps // 2), max(1, args.warmup // 2), ROTATE)
            extra[name] = attn_entry(wa, wms, ems)
        out["workloads"] = extra

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes"] = {"read": src.numel() * 4, "written": src.numel() * 4}
        del src, dst

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
