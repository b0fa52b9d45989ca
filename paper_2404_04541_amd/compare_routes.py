"""Times of the library's other routes beside the row-wise single pass (a measuring aid).

    python -m paper_2404_04541_amd.compare_routes outer      outer-product route against spgemm() on configurations 1 and 4
    python -m paper_2404_04541_amd.compare_routes pipeline   row-block pipeline against spgemm() on the R-MAT product
"""
from __future__ import annotations

import argparse
import time


def timed(fn, torch, reps=3):
    fn()
    torch.cuda.synchronize()
    best = 1e30
    for _ in range(reps):
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        best = min(best, time.perf_counter() - t0)
    return best * 1e3


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["outer", "pipeline"])
    ap.add_argument("--scale", type=int, default=20, help="R-MAT scale of the pipeline comparison")
    ap.add_argument("--blocks", type=int, default=8)
    args = ap.parse_args()
    import torch
    from . import binding as sg, workloads as W
    h = sg.Handle()
    if args.what == "outer":
        print("route times, best of 3, results through the allocator (ms)")
        for name, (A, B) in (("config 1 (1000^2, 10 per row)", W.config1()), ("config 4 (4194304^2 x 4194304 x 65536)", W.config4())):
            dA, dB = sg.to_device(A), sg.to_device(B)
            t_row = timed(lambda: sg.spgemm(h, dA, dB), torch)
            t_conv = timed(lambda: (sg.dcsc_from_csr(h, dA), sg.dcsr_from_csr(h, dB)), torch)
            Ac, Br = sg.dcsc_from_csr(h, dA), sg.dcsr_from_csr(h, dB)
            t_outer = timed(lambda: sg.spgemm_outer(h, Ac, Br), torch)
            C = sg.spgemm_outer(h, Ac, Br)
            print(f"{name}: row-wise spgemm {t_row:.2f} ms; outer product {t_outer:.2f} ms (+ {t_conv:.2f} ms to build the doubly compressed operands); "
                  f"nnz(C) {C.nnz}")
    else:
        A, _ = W.config3(args.scale)
        dA = sg.to_device(A)
        t_single = timed(lambda: sg.spgemm(h, dA, dA), torch)
        t_pipe = timed(lambda: sg.spgemm_pipelined(h, dA, dA, args.blocks), torch)
        print(f"R-MAT scale {args.scale} A*A: single pass spgemm {t_single:.2f} ms; pipeline of {args.blocks} row blocks {t_pipe:.2f} ms "
              f"(both with result allocation)")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
