"""Where the time of the two dense kernels goes, phase by phase (profiling aid).

Runs the R-MAT A*A benchmark product with the clock variant of the library (the same sources built with
-DSPG_PHASE_CLOCKS: thread 0 of every workgroup reads the shader clock at phase boundaries, nothing is
skipped) and prints each phase's share of the summed workgroup time, scaled to the kernel's HIP-event time.

    python -m paper_2404_04541_amd.phase_profile [--scale 20]
"""
from __future__ import annotations

import argparse
import ctypes as C
import os

import numpy as np

SYM = {0: "row fetch", 1: "clear flag list", 2: "piece set-up (A entries, B row bounds, scans)", 3: "stream products (wave 0's share)",
       4: "short pieces + wait for the slowest wave", 5: "entries per block / group", 6: "tile planning", 7: "allocation round trip",
       8: "records, flag words out, column decode", 9: "tail"}
NUM = {0: "run draw", 1: "run set-up (tile records, A entries)", 2: "wait for the previous tile + piece bounds",
       3: "ranked, columns: clear + piece list", 4: "ranked, columns: list -> flags, ranks, C.colidx", 5: "ranked: product pass",
       6: "ranked: C.values out", 7: "direct: set-up", 8: "direct: product pass", 9: "direct: compress + out",
       10: "searched: columns in, C.colidx out", 11: "searched: product pass", 12: "searched: C.values out",
       13: "ranked, no plan structure: mark pass, ranks, decode", 14: "tail", 15: "ranked, flag words: ranks, decode, C.colidx"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--scale", type=int, default=20)
    args = ap.parse_args()
    import torch
    from . import binding as sg, workloads as W
    from .build import LIB_CLOCKS, build_library
    if not os.path.exists(LIB_CLOCKS):
        build_library(phase_clocks=True)
    sg.LIB_PATH = LIB_CLOCKS
    lib = sg.load_library()
    lib.spgemm_debug_phase_clocks.argtypes = [C.c_void_p, C.c_void_p]
    a, _ = W.config3(args.scale)
    h = sg.Handle()
    h.set_option(sg.OPT_TIMING, 1)
    dA = sg.to_device(a)
    for it in range(3):
        rp, nnz, plan = sg.spgemm_symbolic(h, dA, dA)
        if it == 0:
            col = torch.empty(nnz, dtype=torch.int32, device="cuda")
            val = torch.empty(nnz, dtype=dA.values.dtype, device="cuda")
        sg.spgemm_numeric(h, plan, dA, dA, rp, col, val)
        st = plan.stats()
        buf = (C.c_ulonglong * 64)()
        assert lib.spgemm_debug_phase_clocks(plan.ptr, buf) == 0
        plan.destroy()
    clk = np.array(list(buf), dtype=np.float64).reshape(2, 32)
    print(f"R-MAT scale {args.scale} A*A: products {st['ip_total']}, nnz(C) {st['nnz_c']}; third pass of three")
    for name, tab, row, key in (("k_sym_dense", SYM, clk[0], "sym_dense"), ("k_num_dense", NUM, clk[1], "num_dense")):
        ms, tot = st["kernel_ms"][key], row[:16].sum()
        print(f"{name}: {ms:.2f} ms (HIP events)")
        for i in range(16):
            if row[i] > 0:
                print(f"  {tab.get(i, str(i)):58s} {100 * row[i] / tot:6.2f} %  {ms * row[i] / tot:7.2f} ms")
    print(f"dense tiles {st['dense_tiles']} (direct {st['dense_direct_tiles']}, searched {st['dense_search_tiles']}), runs {st['dense_runs']}")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
