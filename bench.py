#!/usr/bin/env python3
"""Benchmark of the weight-stationary recurrence matmul on one MI355X.

A step is one pass of the whole hot path (load the stationary A, stream B, run the k chains,
emit C) over one synthetic workload, i.e. one call of the C ABI.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu] [--no-extra]
                  [--matmul-only] [--copy-calibration] [--ceiling-all]

NAME is one of the five matmul workloads of the benchmark definition (default c3_bf16_8192, the one
the metric is quoted on), k1_bf16_tallk (few output blocks, long k: k in space), m1_bf16_narrowm (few
rows of A over a large B: (j,k) in space), t1_trsm_8192 (tiled triangular solve: 32 launches per
step), h1_chol_8192 (tiled Cholesky factorisation) or f1_attn_4096 (attention tile recurrence).
Whatever the headline, the others are measured after it and reported under "workloads"
(--no-extra: none of them; --matmul-only: only the matmul ones).

Every workload rotates three operand sets so that no operand is served from the last-level cache.
For every workload a second, untimed pass runs the same steps beside a one-wave clock probe
(cyc_diag_clock on another stream), which gives the engine clock sustained under that load:
`clock_ghz`, and for the MFMA-bound ones `frac_sustained` = achieved / (peak * clock_ghz / 2.4).
`mfma_ceiling` is what back-to-back MFMAs from registers reach on this machine in this run
(cyc_diag_mfma_ceiling).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "recurrence matmul TFLOP/s (TOP/s int8) and % of MI355X MFMA/HBM roofline"
# published MI355X peaks used for the roofline fractions; the MFMA peaks assume the 2.4 GHz engine clock
PEAK = {"bf16": (2500.0, "TFLOP/s"), "i8": (5000.0, "TOP/s")}
PEAK_CLOCK_GHZ = 2.4
HBM_PEAK_GBS = 8000.0
ROTATE = 3     # distinct operand sets cycled through
TRAFFIC_PROFILE = os.path.join("profiles", "bench_all_workloads.md")
DEV = "cuda:0"


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
    ap.add_argument("--constant-data", action="store_true",
                    help="diagnostic: matmul operands are all ones instead of the workload's random values (shows how much of "
                         "the time is the chip's power management reacting to the data); never a valid measurement")
    ap.add_argument("--ceiling-all", action="store_true",
                    help="measure the register-only MFMA rate for both instruction shapes and both element types")
    ap.add_argument("--issue-mix", action="store_true",
                    help="also measure what a SIMD issues beside its MFMAs (cyc_diag_issue_mix): rounds of 256 matrix-pipe "
                         "cycles with 0 .. 96 other instructions between the MFMAs, both MFMA shapes, one and two waves per SIMD")
    return ap.parse_args()


def traffic_table():
    """HBM-side bytes per launch from the committed rocprofv3 summary (FETCH_SIZE / WRITE_SIZE, each scaled by what
    the same counter reads for a 1 GiB copy): {workload: bytes}, and where they come from."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    out, stamp = {}, ""
    try:
        text = open(path).read()
    except OSError:
        return out, None
    m = re.search(r"measured (\d{4}-\d{2}-\d{2})", text)
    stamp = m.group(1) if m else "undated"
    sec = text.split("## HBM-side traffic per launch", 1)
    if len(sec) == 2:
        for line in sec[1].split("\n## ", 1)[0].splitlines():
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) >= 6 and re.match(r"^[a-z]\d_", cells[0]):
                try:
                    out[cells[0]] = int((float(cells[3]) + float(cells[5])) * (1 << 20))
                except ValueError:
                    pass
    return out, f"{TRAFFIC_PROFILE} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, calibrated against a 1 GiB copy; {stamp})"


# ---------------------------------------------------------------------------------------------- workloads
def all_workloads():
    from datagen import ws_inputs
    table = {}
    for group, kind in ((ws_inputs.WORKLOADS, "matmul"), (ws_inputs.KSPACE_WORKLOADS, "matmul"),
                        (ws_inputs.NARROWM_WORKLOADS, "matmul"), (ws_inputs.TRI_WORKLOADS, "trsm"),
                        (ws_inputs.CHOL_WORKLOADS, "chol"), (ws_inputs.ATTN_WORKLOADS, "attn")):
        for name, w in group.items():
            table[name] = (kind, w)
    return table


CONSTANT_DATA = False     # set by --constant-data


def make_step(lib, torch, kind, w, sets):
    """Operand sets resident on the GPU and step(i): one call of the C ABI on set i % sets.  Returns (step, info)."""
    from datagen import ws_inputs
    stream = torch.cuda.current_stream()
    data = []
    info = {}
    if kind == "matmul":
        dt = lib.CYC_I8_I32 if w.dtype == "i8" else lib.CYC_BF16_F32
        for r in range(sets):
            wr = ws_inputs.Workload(w.name, w.dtype, w.batch, w.M, w.K, w.N, w.dist, w.param, w.seed + 1000 * r)
            A, B = ws_inputs.make_inputs(wr, DEV)
            if CONSTANT_DATA:
                A.fill_(1)
                B.fill_(1)
            cshape = (w.batch, w.M, w.N) if w.batch > 1 else (w.M, w.N)
            data.append((A, B, torch.empty(cshape, dtype=torch.int32 if w.dtype == "i8" else torch.float32, device=DEV)))
        A, B, C = data[0]
        info["kernel"] = lib.cyc_kernel_name(A.data_ptr(), B.data_ptr(), C.data_ptr(), w.batch, w.M, w.K, w.N,
                                             w.M * w.K, w.K * w.N, w.M * w.N, dt)

        def call(a, b, c):
            return lib.cyc_recurrence_matmul_batched(a.data_ptr(), b.data_ptr(), c.data_ptr(), w.batch, w.M, w.K, w.N,
                                                     w.M * w.K, w.K * w.N, w.M * w.N, dt, stream.cuda_stream)
    elif kind == "trsm":
        for r in range(sets):
            L, B = ws_inputs.make_tri_inputs(ws_inputs.TriWorkload(w.name, w.n, w.nrhs, w.nb, w.seed + 1000 * r), DEV)
            data.append((L, B, torch.empty((w.n, w.nrhs), dtype=torch.float32, device=DEV),
                         torch.empty((w.n, w.nrhs), dtype=torch.bfloat16, device=DEV)))
        info["kernel"] = "trsm"

        def call(L, B, X, Xh):
            return lib.cyc_recurrence_trsm(L.data_ptr(), B.data_ptr(), X.data_ptr(), Xh.data_ptr(), w.n, w.nrhs, w.nb,
                                           stream.cuda_stream)
    elif kind == "chol":
        for r in range(sets):
            data.append((ws_inputs.spd_f32(w.n, w.seed + 1000 * r, 0, DEV),
                         torch.empty((w.n, w.n), dtype=torch.float32, device=DEV),
                         torch.empty((w.n, w.n), dtype=torch.bfloat16, device=DEV)))
        info["kernel"] = "cholesky"

        def call(A, L, Lh):
            return lib.cyc_recurrence_cholesky(A.data_ptr(), L.data_ptr(), Lh.data_ptr(), w.n, w.nb, stream.cuda_stream)
    else:
        for r in range(sets):
            Q, K, V = ws_inputs.make_attn_inputs(ws_inputs.AttnWorkload(w.name, w.batch, w.N, w.M, w.d, w.seed + 1000 * r), DEV)
            data.append((Q, K, V, torch.empty((w.batch, w.N, w.d), dtype=torch.float32, device=DEV)))
        info["kernel"] = "attention"

        def call(Q, K, V, O):
            return lib.cyc_recurrence_attention(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), w.batch, w.N, w.M,
                                                w.d, stream.cuda_stream)

    def step(i):
        st = call(*data[i % sets])
        if st != 0:
            raise RuntimeError(lib.cyc_status_string(st))

    return step, info


def time_steps(torch, step, steps, warmup):
    """`warmup` untimed steps, then exactly `steps` timed ones: (wall ms per step, mean ms per step by events on the
    stream the library launches on, which is torch's current stream)."""
    stream = torch.cuda.current_stream()
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
    return wall_ms, sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps


def sustained_clock(lib, torch, step, ev_ms, window_ms=25.0):
    """Engine clock (GHz) while the steps run: a one-wave probe on a second stream counts shader cycles against the
    constant 100 MHz counter for `window_ms` while the main stream is kept busy with steps.  Untimed."""
    side = torch.cuda.Stream()
    out = torch.zeros(2, dtype=torch.int64, device=DEV)
    n = int(window_ms / max(ev_ms, 1e-3)) + 4
    for i in range(3):
        step(i)                                    # the chip is already under load when the probe starts
    st = lib.cyc_diag_clock(out.data_ptr(), int(window_ms * 1000), side.cuda_stream)
    if st != 0:
        raise RuntimeError(lib.cyc_status_string(st))
    for i in range(n):
        step(i)
    torch.cuda.synchronize()
    cycles, ticks = (int(v) for v in out.cpu())
    return cycles / ticks / 10.0 if ticks > 0 else None


def mfma_ceiling(lib, torch, dtype_name, shape=16, launches=8, iters=8000):
    """Rate of back-to-back MFMAs from registers (no memory traffic) and the clock it ran at."""
    dt = lib.CYC_I8_I32 if dtype_name == "i8" else lib.CYC_BF16_F32
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    stream = torch.cuda.current_stream()
    ops = [0.0]

    def step(i):
        st, o = lib.cyc_diag_mfma_ceiling(dt, shape, iters, sink.data_ptr(), stream.cuda_stream)
        if st != 0:
            raise RuntimeError(lib.cyc_status_string(st))
        ops[0] = o

    _, ev_ms = time_steps(torch, step, launches, 3)
    clock = sustained_clock(lib, torch, step, ev_ms)
    rate = ops[0] / (ev_ms * 1e-3) / 1e12
    return {"rate": round(rate, 1), "unit": PEAK[dtype_name][1], "frac_of_peak": round(rate / PEAK[dtype_name][0], 4),
            "clock_ghz": round(clock, 3) if clock else None, "mfma": f"{shape}x{shape}", "ms_per_launch": round(ev_ms, 4)}


def issue_mix_table(lib, torch, iters=4000):
    """Cycles a SIMD needs per round of 256 matrix-pipe cycles when other instructions are issued between the MFMAs
    (constant operands, nothing but registers and a few LDS words: the issue port is all that is measured)."""
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    stream = torch.cuda.current_stream()
    rows = []
    for shape in (16, 32):
        for waves in (1, 2):
            for kind, kname in ((0, "v_fma_f32"), (1, "v_exp_f32"), (2, "ds_read_b128")):
                for per_round in (0, 16, 32, 48, 64, 96):
                    if per_round == 0 and kind != 0:
                        continue
                    ops = [0.0]

                    def step(i):
                        st, o = lib.cyc_diag_issue_mix(shape, kind, per_round, waves, iters, sink.data_ptr(), stream.cuda_stream)
                        if st != 0:
                            raise RuntimeError(lib.cyc_status_string(st))
                        ops[0] = o

                    _, ev_ms = time_steps(torch, step, 4, 2)
                    clock = sustained_clock(lib, torch, step, ev_ms)
                    rows.append({"mfma": f"{shape}x{shape}", "waves_per_simd": waves, "other": kname if per_round else "-",
                                 "others_per_round": per_round, "ms_per_launch": round(ev_ms, 4),
                                 "tflops_in_mfmas": round(ops[0] / (ev_ms * 1e-3) / 1e12, 1), "clock_ghz": round(clock, 3) if clock else None,
                                 "cycles_per_round": round(ev_ms * 1e-3 * clock * 1e9 / (iters * waves), 1) if clock else None})
    return rows


# ---------------------------------------------------------------------------------------------- rooflines
def roofline_of(kind, w, ev_ms, clock, traffic):
    """Which roofline bounds the workload and how close the measured launch comes.  Matmul workloads: operations per
    algorithmic byte (A and B read once, C written once) against the chip's ridge; the tiny parity cases c1 and c2
    are latency bound and get no fraction.  The other recurrences are priced against the bf16 MFMA peak."""
    name = w.name
    dtype = getattr(w, "dtype", "bf16")
    peak, unit = PEAK[dtype]
    out = {}
    if kind == "matmul" and w.ops < 1e9:
        out = {"bound": "latency", "achieved": round(w.ops / (ev_ms * 1e-3) / 1e12, 3), "peak": None, "unit": unit, "frac": None}
    elif kind == "matmul" and w.ops / w.algorithmic_bytes < peak * 1e12 / (HBM_PEAK_GBS * 1e9):
        ach = w.algorithmic_bytes / (ev_ms * 1e-3) / 1e9
        out = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4)}
    else:
        ach = w.ops / (ev_ms * 1e-3) / 1e12
        out = {"bound": "mfma", "achieved": round(ach, 1), "peak": peak, "unit": unit, "frac": round(ach / peak, 4)}
        if clock:
            out["frac_sustained"] = round(ach / (peak * clock / PEAK_CLOCK_GHZ), 4)
    out["clock_ghz"] = round(clock, 3) if clock else None
    out["traffic"] = traffic[0].get(name)
    out["traffic_source"] = traffic[1] if out["traffic"] is not None else None
    return out


def headline_value(kind, w, wall_ms):
    """BASELINE metric: TFLOP/s (TOP/s) for the compute-bound workloads, GB/s for the HBM-bound ones."""
    if kind == "matmul" and w.ops >= 1e9 and w.ops / w.algorithmic_bytes < PEAK[w.dtype][0] * 1e12 / (HBM_PEAK_GBS * 1e9):
        return w.algorithmic_bytes / 1e9 / (wall_ms * 1e-3), "GB/s"
    return w.ops / 1e12 / (wall_ms * 1e-3), PEAK[getattr(w, "dtype", "bf16")][1]


def config_of(kind, w, kernel):
    if kind == "matmul":
        return {"workload": w.name, "batch": w.batch, "M": w.M, "K": w.K, "N": w.N, "kernel": kernel,
                "accumulate": "fp32" if w.dtype == "bf16" else "int32", "seed": w.seed, "operand_sets_rotated": ROTATE}
    if kind == "trsm":
        return {"workload": w.name, "n": w.n, "nrhs": w.nrhs, "nb": w.nb, "kernel": kernel, "accumulate": "fp32", "seed": w.seed,
                "operand_sets_rotated": ROTATE}
    if kind == "chol":
        return {"workload": w.name, "n": w.n, "nb": w.nb, "kernel": kernel, "accumulate": "fp32", "seed": w.seed,
                "operand_sets_rotated": ROTATE}
    return {"workload": w.name, "batch": w.batch, "N": w.N, "M": w.M, "d": w.d, "kernel": kernel, "accumulate": "fp32",
            "seed": w.seed, "operand_sets_rotated": ROTATE}


def run_workload(lib, torch, kind, w, steps, warmup, traffic):
    step, info = make_step(lib, torch, kind, w, ROTATE)
    wall_ms, ev_ms = time_steps(torch, step, steps, warmup)
    clock = sustained_clock(lib, torch, step, ev_ms)
    rf = roofline_of(kind, w, ev_ms, clock, traffic)
    rf["kernel"] = info["kernel"] if kind in ("matmul", "attn") else info["kernel"] + " (all kernels of a step)"
    rf["kernel_ms"] = round(ev_ms, 5)
    del step
    torch.cuda.empty_cache()
    return wall_ms, ev_ms, info["kernel"], rf


# ---------------------------------------------------------------------------------------------- CPU baselines
def cpu_baseline_matmul(w, budget_s=15.0):
    """The oracle's row-chain form, as it stands, on a bounded block of the same workload."""
    from datagen import ws_inputs
    from oracle import ws_oracle
    mode = "i8" if w.dtype == "i8" else "bf16"
    host = (lambda A, B: (ws_oracle.bf16_bits(A), ws_oracle.bf16_bits(B))) if mode == "bf16" else (lambda A, B: (A.numpy(), B.numpy()))
    cols = min(w.N, 1024)
    probe_rows = min(w.M, 64)
    A, B = host(*ws_inputs.make_inputs(ws_inputs.Workload(w.name, w.dtype, 1, probe_rows, w.K, cols, w.dist, w.param, w.seed), "cpu"))
    t0 = time.perf_counter()
    ws_oracle.ws_rowchain(A, B, mode)
    rate = probe_rows * w.K * cols / max(time.perf_counter() - t0, 1e-6)        # cell-steps per second
    rows = int(min(max(64, rate * budget_s / (w.K * cols)), 8192, max(w.M, 16)))
    rows = min(w.M, max(16, rows // 16 * 16))                                   # never more rows than A has
    # a batched workload whose single element is over in a fraction of a second: take several elements
    elems = min(w.batch, 8) if rows >= min(w.M, 8192) // 16 * 16 and w.batch > 1 else 1
    blocks = []
    for b in range(elems):
        wr = ws_inputs.Workload(w.name, w.dtype, 1, rows, w.K, cols, w.dist, w.param, w.seed + 1000 * b)
        blocks.append(host(*ws_inputs.make_inputs(wr, "cpu")))
    t0 = time.perf_counter()
    for A, B in blocks:
        ws_oracle.ws_rowchain(A, B, mode)
    dt = time.perf_counter() - t0
    what = (f"a {rows} x {w.K} x {cols} block (first rows of A, first columns of B)" if elems == 1 else
            f"{elems} batch elements of {rows} x {w.K} x {cols} (seeds {w.seed}, {w.seed + 1000}, ...)")
    return {"value": round(2.0 * elems * rows * w.K * cols / dt / 1e12, 6), "unit": "TOP/s" if mode == "i8" else "TFLOP/s",
            "cores": ws_oracle.threads(), "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"row-chain oracle on {what} of {w.name}, same distribution"}


def cpu_baseline(kind, w):
    import numpy as np
    from datagen import ws_inputs
    from oracle import ws_oracle
    if kind == "matmul":
        return cpu_baseline_matmul(w)
    if kind == "trsm":
        from oracle import tri_oracle
        L, B = ws_inputs.make_tri_inputs(w, "cpu")
        cols = 4096
        Bs = np.ascontiguousarray(B[:, :cols].numpy())
        t0 = time.perf_counter()
        tri_oracle.tri_tiled(ws_oracle.bf16_bits(L), Bs, w.nb)
        dt = time.perf_counter() - t0
        return {"value": round(w.n * (w.n + 1) * cols / dt / 1e12, 6), "unit": "TFLOP/s", "cores": ws_oracle.threads(),
                "kind": "oracle", "seconds": round(dt, 2),
                "sample": f"tiled triangular-solve oracle on the first {cols} right-hand sides of {w.name} (columns are "
                          f"independent), same seed and distribution"}
    if kind == "chol":
        from oracle import chol_oracle
        reps = 6
        mats = [ws_inputs.spd_f32(w.n, w.seed + 1000 * r, 0, "cpu").numpy() for r in range(reps)]
        t0 = time.perf_counter()
        for A in mats:
            chol_oracle.chol_tiled(A, w.nb)
        dt = time.perf_counter() - t0
        return {"value": round(reps * w.ops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": ws_oracle.threads(), "kind": "oracle",
                "seconds": round(dt, 2),
                "sample": f"tiled Cholesky oracle on {reps} whole matrices of {w.name} (seeds {w.seed}, {w.seed + 1000}, ...), "
                          f"same distribution"}
    from oracle import attn_oracle
    elems = min(w.batch, 48)
    Q, K, V = ws_inputs.make_attn_inputs(ws_inputs.AttnWorkload(w.name, elems, w.N, w.M, w.d, w.seed), "cpu")
    w64 = lambda t: ws_oracle.bits_to_f64(ws_oracle.bf16_bits(t))
    t0 = time.perf_counter()
    for b in range(elems):
        attn_oracle.attention(w64(Q[b]), w64(K[b]), w64(V[b]))
    dt = time.perf_counter() - t0
    return {"value": round(4.0 * elems * w.N * w.M * w.d / dt / 1e12, 6), "unit": "TFLOP/s", "cores": ws_oracle.threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"attention oracle (fp64 softmax definition) on the first {elems} of the {w.batch} batch elements of "
                      f"{w.name} (elements are independent), same seed and distribution"}


# ---------------------------------------------------------------------------------------------- main
def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on exactly one GPU (no collectives, no sharding); got --gpus {args.gpus}",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2511_09987_amd as lib

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(2)
    table = all_workloads()
    if args.workload not in table:
        print(f"bench.py: unknown workload {args.workload}; choose from {sorted(table)}", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    traffic = traffic_table()
    global CONSTANT_DATA
    CONSTANT_DATA = args.constant_data

    kind, w = table[args.workload]
    wall_ms, ev_ms, kernel, rf = run_workload(lib, torch, kind, w, args.steps, args.warmup, traffic)
    value, unit = headline_value(kind, w, wall_ms)
    dtype = getattr(w, "dtype", "bf16")
    out = {
        "metric": METRIC, "value": round(value, 2), "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype == "bf16" else "int8",
        "data": "constant (diagnostic, not a valid measurement)" if args.constant_data else "synthetic",
        "config": config_of(kind, w, kernel), "roofline": rf,
    }

    if not args.no_extra:
        extra = {}
        order = ("c3_bf16_8192", "c4_i8_8192", "c5_bf16_narrow", "c2_bf16_512", "c1_i8_64", "k1_bf16_tallk", "m1_bf16_narrowm",
                 "t1_trsm_8192", "h1_chol_8192", "f1_attn_4096")
        for name in order:
            k2, w2 = table[name]
            if name == w.name or (args.matmul_only and k2 != "matmul"):
                continue
            # the multi-kernel recurrences take milliseconds per step: fewer steps keep the whole run short
            steps = args.steps if k2 == "matmul" else max(3, args.steps // (4 if k2 == "chol" else 2))
            warm = args.warmup if k2 == "matmul" else max(1, args.warmup // 4)
            wms, ems, kn, rf2 = run_workload(lib, torch, k2, w2, steps, warm, traffic)
            entry = {"kernel": kn, "ms_per_step": round(wms, 5), "kernel_ms": round(ems, 5)}
            entry.update({k: rf2[k] for k in ("achieved", "unit", "bound", "frac", "clock_ghz") if k in rf2})
            if "frac_sustained" in rf2:
                entry["frac_sustained"] = rf2["frac_sustained"]
            extra[name] = entry
        out["workloads"] = extra

    # what the matrix pipes alone sustain on this machine, in this run
    if args.ceiling_all:
        out["mfma_ceiling"] = {f"{d}_{s}x{s}": mfma_ceiling(lib, torch, d, s) for d in ("bf16", "i8") for s in (16, 32)}
    else:
        out["mfma_ceiling"] = {f"{d}_16x16": mfma_ceiling(lib, torch, d, 16) for d in ("bf16", "i8")}

    if args.issue_mix:
        out["issue_mix"] = issue_mix_table(lib, torch)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=DEV).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes"] = {"read": src.numel() * 4, "written": src.numel() * 4}
        del src, dst

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(kind, w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
