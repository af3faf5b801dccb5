"""Times the fused attention forward kernel for one shape through the C ABI (sif_k_attn_fwd) and prints its rate; also
the program to put behind `rocprofv3 --pmc ... --` when the kernel's counters are wanted.

    python3 -m paper_2503_02550_amd.attn_probe BATCH SEQ HEADS D_HEAD [--causal] [--iters I]
"""
import argparse

import torch

from . import binding as S


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("batch", type=int)
    ap.add_argument("seq", type=int)
    ap.add_argument("heads", type=int)
    ap.add_argument("d_head", type=int)
    ap.add_argument("--causal", action="store_true")
    ap.add_argument("--iters", type=int, default=10)
    a = ap.parse_args()
    dev = "cuda:0"
    da = a.heads * a.d_head
    qkv = torch.randn((a.batch * a.seq, 3 * da), device=dev).to(torch.bfloat16)
    o = torch.zeros((a.batch * a.seq, da), device=dev, dtype=torch.bfloat16)

    def run():
        S.sif_k_attn_fwd(qkv, o, a.batch, a.seq, a.heads, a.d_head, 3 * da, da, 1 if a.causal else 0)

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
    flops = 4.0 * a.batch * a.heads * a.seq * a.seq * a.d_head * (0.5 if a.causal else 1.0)
    nbytes = 8.0 * a.batch * a.seq * da
    print(f"attention forward {a.batch} x {a.seq} x {a.heads} heads x {a.d_head}{' causal' if a.causal else ''}: {us:.1f} us, "
          f"{flops / us / 1e6:.1f} TFLOP/s, {nbytes / us / 1e6:.2f} TB/s of q, k, v, o")


if __name__ == "__main__":
    main()
