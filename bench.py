#!/usr/bin/env python3
"""Throughput of the whole SpGEMM hot path on one MI355X.

A step is one pass of the full path (row count, binning, symbolic per bin, scan, numeric per
bin, CSR write) over the R-MAT A*A workload: 2^20 x 2^20, fp32, 16 edges per vertex drawn,
power-law rows.  Operands and the output buffers are resident in HBM when timing starts.

Prints one JSON line:
  value      GFLOP/s, counting 2 flops per intermediate product
  roofline   the numeric dense-workspace kernel (the dominant one) against the 8 TB/s HBM peak,
             from algorithmic bytes and HIP-event durations taken inside the timed region
  roofline_other  the same for the symbolic dense kernel
  other_configs   ms per pass, GFLOP/s and stream-model fraction of the stencil, rectangular and tensor
                  configurations (same protocol, fewer steps; not part of `value`)
  cpu_baseline  the CPU checker (std::map Gustavson, all host cores) on a product-weighted sample of rows
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

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "k_num_dense_rmat20_hbm_traffic.txt")
KERNEL_SOURCES = ("common.hpp", "dense_kernels.hpp")   # what the dense kernels are compiled from


def kernel_source_hash() -> str:
    import hashlib
    hsh = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2404_04541_amd", "csrc", name), "rb") as f:
            hsh.update(f.read())
    return hsh.hexdigest()


def measured_traffic(key: str = "hbm_bytes_per_launch"):
    """HBM bytes per launch of a dense kernel from the committed rocprofv3 counter summary (FETCH_SIZE and WRITE_SIZE,
    each scaled by what the same counter reads for a plain 1 GiB copy; for kernels with many narrow requests the
    FETCH_SIZE scale is an upper bound); None when there is none or the kernels' sources changed since it was taken."""
    try:
        fields = dict(line.split(":", 1) for line in open(TRAFFIC_FILE) if ":" in line and not line.startswith("#"))
        if fields["source_sha256"].strip() != kernel_source_hash():
            return None
        return float(fields[key])
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(A, B, ip_rows: np.ndarray, budget_ip: float = 2.0e8) -> dict:
    """Time the CPU checker on rows drawn with probability proportional to their product counts (so that long
    rows, whose maps are large, weigh as they do in the whole product), about budget_ip products in all."""
    import oracle
    from paper_2404_04541_amd import workloads as W
    prefix = np.cumsum(ip_rows.astype(np.float64))
    u = W.rand_unit(0, 900, np.arange(4096, dtype=np.uint64)) * prefix[-1]
    draw = np.searchsorted(prefix, u, side="right")
    pick = draw[np.sort(np.unique(draw, return_index=True)[1])]
    n = int(np.searchsorted(np.cumsum(ip_rows[pick]), budget_ip)) + 1
    pick = np.ascontiguousarray(np.sort(pick[:n]))
    oracle.build()
    t0 = time.perf_counter()
    r = oracle.spgemm_rows(A.rowptr, A.colidx, A.values, B.rowptr, B.colidx, B.values, rows=pick)
    dt = time.perf_counter() - t0
    ip = int(r.ip.sum())
    return {"value": 2.0 * ip / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"{pick.size} rows of the same A*A drawn with probability proportional to their products ({ip} intermediate "
                      f"products, {int(r.cnt.sum())} output entries), {dt:.1f} s wall"}


def stream_bytes(ip_total, nnz_c, nnz_a, m, v):
    return ip_total * (8 + v) + nnz_c * (4 + v) + nnz_a * (60 + v) + m * 60


def time_config(sg, torch, A, B, steps, warmup):
    """ms per pass (symbolic + numeric, outputs preallocated) of one configuration, and its sizes."""
    h = sg.Handle()
    dA = sg.to_device(A)
    dB = dA if B is A else sg.to_device(B)
    rp = torch.empty(A.rows + 1, dtype=torch.int64, device="cuda")
    _, nnz_c, plan = sg.spgemm_symbolic(h, dA, dB, rp)
    col = torch.empty(nnz_c, dtype=torch.int32, device="cuda")
    val = torch.empty(nnz_c, dtype=dA.values.dtype, device="cuda")
    ip_total = plan.stats()["ip_total"]
    plan.destroy()
    for it in range(warmup + steps):
        if it == warmup:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        _, n, pl = sg.spgemm_symbolic(h, dA, dB, rp)
        sg.spgemm_numeric(h, pl, dA, dB, rp, col, val)
        torch.cuda.synchronize()
        pl.destroy()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    v = A.values.dtype.itemsize
    b = stream_bytes(ip_total, nnz_c, A.nnz, A.rows, v)
    return {"ms_per_step": ms, "GFLOP/s": 2.0 * ip_total / ms / 1e6, "intermediate_products": ip_total, "nnz_c": nnz_c,
            "effective_hbm_frac": b / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "dtype": "f32" if v == 4 else "f64"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--scale", type=int, default=20, help="R-MAT scale (20 = the benchmark configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the stencil / rectangular / tensor configurations")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (read 1 GiB, write 1 GiB): the reference for HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no multi-GPU path exists); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2404_04541_amd import workloads as W
    from paper_2404_04541_amd import binding as sg
    if not os.path.exists(sg.LIB_PATH):
        from paper_2404_04541_amd.build import build_library
        build_library()

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    A, B = W.config3(args.scale)
    h = sg.Handle()
    h.set_option(sg.OPT_TIMING, 1)
    dA = sg.to_device(A)
    dB = dA
    # first pass sizes the output; its buffers are reused by every step
    rp = torch.empty(A.rows + 1, dtype=torch.int64, device="cuda")
    _, nnz_c, plan = sg.spgemm_symbolic(h, dA, dB, rp)
    col = torch.empty(nnz_c, dtype=torch.int32, device="cuda")
    val = torch.empty(nnz_c, dtype=dA.values.dtype, device="cuda")
    sg.spgemm_numeric(h, plan, dA, dB, rp, col, val)
    st = plan.stats()
    plan.destroy()
    ip_total = st["ip_total"]

    def step():
        _, n, pl = sg.spgemm_symbolic(h, dA, dB, rp)
        assert n == nnz_c
        sg.spgemm_numeric(h, pl, dA, dB, rp, col, val)
        s = pl.stats()   # waits for this step's numeric kernels (event times)
        pl.destroy()
        return s

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    per_kernel = {}
    for _ in range(args.steps):
        s = step()
        for k, v in s["kernel_ms"].items():
            per_kernel[k] = per_kernel.get(k, 0.0) + v
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    gflops = 2.0 * ip_total * args.steps / dt / 1e9

    v = A.values.dtype.itemsize
    m, nnz_a = A.rows, A.nnz
    bytes_stream = stream_bytes(ip_total, nnz_c, nnz_a, m, v)
    eff_gbs = bytes_stream * args.steps / dt / 1e9
    # dominant kernel: numeric dense workspace.  Algorithmic bytes per launch = the gathered B
    # entries of its rows (column + value per intermediate product) + the C entries it writes.
    dense_ip = sum(st["num_bin_ip"][5:7])
    dense_nnz = sum(st["num_bin_nnz"][5:7])
    dense_bytes = dense_ip * (4 + v) + dense_nnz * (4 + v)
    dense_ms = per_kernel.get("num_dense", 0.0) / args.steps
    achieved = dense_bytes / (dense_ms * 1e-3) / 1e9 if dense_ms > 0 else 0.0
    # symbolic dense kernel: the gathered B columns of its rows (4 B per product); what it leaves in the plan
    # for the numeric phase is extra, not counted
    sym_ip = sum(st["sym_bin_ip"][4:7])
    sym_bytes = sym_ip * 4
    sym_ms = per_kernel.get("sym_dense", 0.0) / args.steps
    sym_achieved = sym_bytes / (sym_ms * 1e-3) / 1e9 if sym_ms > 0 else 0.0
    out = {
        "metric": "SpGEMM GFLOP/s (2 x intermediate products / s)", "value": gflops, "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64 (sums of products of f32 operands, rounded once to f32)", "data": "synthetic",
        "config": {"workload": f"C=A*A, A R-MAT scale {args.scale} (a=0.57,b=c=0.19,d=0.05), 16 edges/vertex drawn, "
                               f"duplicates merged, fp32 values U[0,1), seed 0",
                   "rows": m, "nnz_a": nnz_a, "intermediate_products": ip_total, "nnz_c": nnz_c},
        "effective_hbm": {"bytes_per_step": bytes_stream, "GB/s": eff_gbs, "frac_of_peak": eff_gbs / HBM_PEAK_GBS,
                          "model": "IP*(8+v) + nnzC*(4+v) + nnzA*(60+v) + rows*60, v = value bytes"},
        "kernel_ms_per_step": {k: per_kernel[k] / args.steps for k in per_kernel},
        "roofline": {"kernel": "k_num_dense<float>", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(),
                     "bytes_per_launch": dense_bytes, "ms_per_launch": dense_ms},
        "roofline_other": [{"kernel": "k_sym_dense", "bound": "hbm", "achieved": sym_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": sym_achieved / HBM_PEAK_GBS, "traffic": measured_traffic("k_sym_dense_hbm_bytes_per_launch"),
                            "bytes_per_launch": sym_bytes, "ms_per_launch": sym_ms}],
        "plan_bytes": st["plan_bytes"], "plan_list_bytes_used": st["plan_list_used"],
    }
    del col, val, rp, dA, dB
    if not args.no_other_configs:
        torch.cuda.empty_cache()
        other = {}
        for name, make in (("config2 stencil 128^3 A*A f64", W.config2), ("config4 rectangular A*B f64", W.config4),
                           ("config5 tensor mode-3 unfolding * M f64", W.config5)):
            A2, B2 = make()
            other[name] = time_config(sg, torch, A2, B2, steps=5, warmup=2)
            del A2, B2
            torch.cuda.empty_cache()
        out["other_configs"] = other
    if not args.no_cpu_baseline:
        run = np.concatenate([[0], np.cumsum(np.diff(B.rowptr)[A.colidx])])
        ip_rows = run[A.rowptr[1:]] - run[A.rowptr[:-1]]
        out["cpu_baseline"] = cpu_baseline(A, B, ip_rows)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
