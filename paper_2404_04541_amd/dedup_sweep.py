"""The paper's synthetic first-order sweep (section 7.2) on the GPU: row-wise SpGEMM B * rot(B^T) for K from
2500 to 40000, timed with the long rows routed through a dense accumulator indexed by column ("direct" tiles:
the dense workspace) and through accumulators that hold only the columns that exist ("ranked" tiles: the sparse
workspace), plus the library's own choice.

    python -m paper_2404_04541_amd.dedup_sweep [--steps 5]

Prints one JSON line per K: products, output entries, products per entry (the amount of deduplication) and
milliseconds of symbolic + numeric kernels per route.
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def time_route(sg, torch, h, dB, dC, steps):
    rp, nnz, plan = sg.spgemm_symbolic(h, dB, dC)
    col = torch.empty(nnz, dtype=torch.int32, device="cuda")
    val = torch.empty(nnz, dtype=dB.values.dtype, device="cuda")
    sg.spgemm_numeric(h, plan, dB, dC, rp, col, val)
    st = plan.stats()
    plan.destroy()
    sym = num = 0.0
    for _ in range(steps):
        _, _, plan = sg.spgemm_symbolic(h, dB, dC, rp)
        sg.spgemm_numeric(h, plan, dB, dC, rp, col, val)
        s = plan.stats()
        plan.destroy()
        km = s["kernel_ms"]
        num += sum(v for k, v in km.items() if k.startswith("num_"))
        sym += sum(v for k, v in km.items() if not k.startswith("num_"))
    return st, sym / steps, num / steps


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--ks", type=int, nargs="*", default=[2500, 5000, 10000, 20000, 40000])
    args = ap.parse_args()
    import torch
    from . import workloads as W
    from . import binding as sg
    for K in args.ks:
        B, C = W.dedup_sweep(K)
        dB, dC = sg.to_device(B), sg.to_device(C)
        out = {"K": K, "I": B.rows, "nnz_b": B.nnz}
        # route: (forced workspace, direct-tile threshold, products per entry up to which rows are searched tiles)
        routes = {"auto": (sg.WORKSPACE_AUTO, None, None),
                  "dense (direct tiles)": (sg.WORKSPACE_DENSE, 256, 0),
                  "sparse (ranked tiles)": (sg.WORKSPACE_DENSE, 1 << 20, 0)}
        for name, (force, direct_min, search_ratio) in routes.items():
            h = sg.Handle()
            h.set_option(sg.OPT_TIMING, 1)
            h.set_option(sg.OPT_FORCE_WORKSPACE, force)
            if direct_min is not None:
                h.set_option(sg.OPT_DIRECT_MIN, direct_min)
            if search_ratio is not None:
                h.set_option(sg.OPT_SEARCH_RATIO, search_ratio)
            st, sym, num = time_route(sg, torch, h, dB, dC, args.steps)
            out.setdefault("intermediate_products", st["ip_total"])
            out.setdefault("nnz_c", st["nnz_c"])
            out.setdefault("products_per_entry", round(st["ip_total"] / max(st["nnz_c"], 1), 2))
            out[name] = {"symbolic_ms": round(sym, 3), "numeric_ms": round(num, 3),
                         "tiles": st["dense_tiles"], "direct": st["dense_direct_tiles"], "searched": st["dense_search_tiles"]}
            h.close()
        print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
