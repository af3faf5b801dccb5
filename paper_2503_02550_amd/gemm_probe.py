"""Times one bf16 GEMM shape through the C ABI (sif_k_gemm_bf16) and prints its rate; also the program to put behind
`rocprofv3 --pmc ... --` when the kernel's counters are wanted.

    python3 -m paper_2503_02550_amd.gemm_probe M N K [--tile 0|128|256] [--a-layout 0|1] [--b-layout 0|1]
                                                     [--epilogue E] [--iters I]
"""
import argparse

import torch

from . import binding as S


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("m", type=int)
    ap.add_argument("n", type=int)
    ap.add_argument("k", type=int)
    ap.add_argument("--tile", type=int, default=0)
    ap.add_argument("--a-layout", type=int, default=0, help="0: A stored [M][K], 1: [K][M]")
    ap.add_argument("--b-layout", type=int, default=0, help="0: B stored [N][K], 1: [K][N]")
    ap.add_argument("--epilogue", type=int, default=0, help="SIF_EPI_* bits (1 bias, 2 GELU)")
    ap.add_argument("--iters", type=int, default=10)
    a = ap.parse_args()
    dev = "cuda:0"
    A = torch.randn((a.m, a.k) if a.a_layout == 0 else (a.k, a.m), device=dev).to(torch.bfloat16)
    B = torch.randn((a.n, a.k) if a.b_layout == 0 else (a.k, a.n), device=dev).to(torch.bfloat16)
    Cm = torch.zeros((a.m, a.n), device=dev, dtype=torch.bfloat16)
    bias = torch.zeros(a.n, device=dev, dtype=torch.bfloat16)

    def run():
        S.sif_k_gemm_bf16(A, B, Cm, a.m, a.n, a.k, A.shape[1], B.shape[1], a.n, a_layout=a.a_layout, b_layout=a.b_layout,
                          epilogue=a.epilogue, bias=bias, tile=a.tile)

    for _ in range(3):
        run()
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(a.iters):
        run()
    t1.record()
    torch.cuda.synchronize()
    us = t0.elapsed_time(t1) * 1e3 / a.iters
    print(f"gemm {a.m} x {a.n} x {a.k} layouts {a.a_layout}{a.b_layout} tile {a.tile}: {us:.1f} us, {2.0 * a.m * a.n * a.k / us / 1e6:.1f} TFLOP/s")


if __name__ == "__main__":
    main()
