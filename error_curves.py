#!/usr/bin/env python3
"""Redraws the paper's two accuracy experiments on one MI355X, as tables.

  1. Error against k for A (16 x k) B (k x 16), uniform(-1, 1) inputs (the paper's first figure): the method in
     both modes, Markidis' method, the unscaled-residual variant, plain FP16 / BF16, and the naive FP32 product.
  2. Exponent-range types 1-4 of section "Effect of the exponent range of input matrices" (exp_rand inputs).

Every number is the relative residual of Eq. eval-matmul against the FP64 reference, averaged over --seeds seeds
(the paper uses 8).  GPU results come from ecgemm_sgemm; the FP32 and FP64 columns from the CPU oracle.
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seeds", type=int, default=8)
    ap.add_argument("--size", type=int, default=1024, help="M = N = K of the exponent-range experiment")
    args = ap.parse_args()
    import torch
    import paper_2203_03341_amd as ec
    import seeded_inputs as si
    from oracle import gemm

    modes = [("ours FP16", ec.MODE_FP16_SPLIT), ("ours BF16x3", ec.MODE_BF16_FULL), ("unscaled", ec.MODE_FP16_UNSCALED),
             ("Markidis", ec.MODE_FP16_MARKIDIS), ("ours FP16, outside acc. every k step", ec.MODE_FP16_OUTSIDE_ACC), ("every 4", ec.MODE_FP16_OUTSIDE_ACC_4), ("every 16", ec.MODE_FP16_OUTSIDE_ACC_16), ("plain FP16", ec.MODE_FP16_PLAIN), ("plain BF16", ec.MODE_BF16_PLAIN),
             ("FP32 on the matrix unit", ec.MODE_FP32_MFMA), ("automatic (arrangement chosen from the data)", ec.MODE_AUTO)]
    h = ec.Handle()
    h.set_stream(torch.cuda.current_stream().cuda_stream)

    def gpu(M, N, K, A, B, mode):
        dA = torch.from_numpy(np.ascontiguousarray(A.T)).cuda()
        dB = torch.from_numpy(np.ascontiguousarray(B.T)).cuda()
        dC = torch.empty((N, M), dtype=torch.float32, device="cuda")
        h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, mode)
        torch.cuda.synchronize()
        return dC.cpu().numpy().T

    def row(M, N, K, draw):
        acc = {name: [] for name, _ in modes}
        acc["FP32 naive"] = []
        for seed in range(args.seeds):
            A, B = draw(seed)
            c64 = gemm.sgemm_fp64_ref("N", "N", M, N, K, 1.0, A, B)
            acc["FP32 naive"].append(gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", M, N, K, 1.0, A, B)))
            for name, mode in modes:
                with np.errstate(all="ignore"):
                    acc[name].append(gemm.relative_residual(c64, gpu(M, N, K, A, B, mode)))
        return {k: float(np.mean(v)) for k, v in acc.items()}

    cols = ["FP32 naive"] + [name for name, _ in modes]
    print("## Error against k, A 16 x k, B k x 16, uniform(-1, 1), mean of %d seeds\n" % args.seeds)
    print("| k | " + " | ".join(cols) + " |\n|---|" + "---|" * len(cols))
    for p in range(4, 17, 2):
        k = 1 << p
        r = row(16, 16, k, lambda s: (si.urand(16, k, s, si.ID_A), si.urand(k, 16, s, si.ID_B)))
        print(f"| {k} | " + " | ".join(f"{r[c]:.2e}" for c in cols) + " |", flush=True)

    n = args.size
    types = [("Type 1: (-15,14) x (-15,14)", (-15, 14), (-15, 14)), ("Type 2: (-15,14) x (-100,-35)", (-15, 14), (-100, -35)),
             ("Type 3: (-35,-15) x (-35,-15)", (-35, -15), (-35, -15)), ("Type 4: (-100,-35) x (-100,-35)", (-100, -35), (-100, -35))]
    print("\n## Exponent ranges, exp_rand inputs, M = N = K = %d, mean of %d seeds\n" % (n, min(args.seeds, 3)))
    print("| inputs | " + " | ".join(cols) + " |\n|---|" + "---|" * len(cols))
    saved = args.seeds
    args.seeds = min(args.seeds, 3)
    for name, ra, rb in types:
        r = row(n, n, n, lambda s: (si.exp_rand(n, n, ra[0], ra[1], s, si.ID_A), si.exp_rand(n, n, rb[0], rb[1], s, si.ID_B)))
        print(f"| {name} | " + " | ".join(f"{r[c]:.2e}" for c in cols) + " |", flush=True)
    args.seeds = saved
    h.destroy()


if __name__ == "__main__":
    main()
