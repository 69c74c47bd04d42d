#!/usr/bin/env python3
"""Times one fake-quantized linear layer (zo_linear_fakequant_mma) through both contractions -- bf16 matrix instructions on
de-quantized operands, and int8 matrix instructions on the integer codes with a per-group rescale -- at the linear shapes of
the Llama-2-7B-shaped workload (8 x 1024 tokens), W4A8, groups of 64 and 128 and per-channel steps (group 0: the integer
route then has no rescale inside its loop).  Whole-call times come from events on the
launch stream; per-kernel times and counters come from running this file under rocprofv3.

    python3 -m paper_2509_00031_amd.bench_linear_mma [--iters 10]
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

SHAPES = [(8192, 12288, 4096), (8192, 4096, 4096), (8192, 22016, 4096), (8192, 4096, 11008)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--groups", default="64,128,0")
    args = ap.parse_args()
    import torch
    from paper_2509_00031_amd import binding as zo
    torch.manual_seed(0)
    for (M, N, K) in SHAPES:
        X = torch.randn(M, K, device="cuda").to(torch.bfloat16)
        W = torch.randn(N, K, device="cuda") * 0.02
        for g in [int(v) for v in args.groups.split(",")]:
            for mma, name in ((zo.MMA_INT8, "int8"), (zo.MMA_BF16, "bf16")):
                run = lambda: zo.zo_linear_fakequant_mma(X, W, 4, g, 8, 1, 0, 1e-3, mma=mma)
                run()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(args.iters):
                    run()
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / args.iters
                print("M %5d N %5d K %5d group %3d %s: %.3f ms per call (both quantizers + GEMM), %.0f T(FL)OP/s of 2 M N K"
                      % (M, N, K, g, name, ms, 2.0 * M * N * K / ms / 1e9), flush=True)


if __name__ == "__main__":
    main()
