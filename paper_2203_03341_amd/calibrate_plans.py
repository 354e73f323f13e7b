"""Refits the constants of the plan cost estimate in csrc/ecgemm.hip (`estimated_us`) from timings on the GPU.

    python -m paper_2203_03341_amd.calibrate_plans build              # CPU: libecgemm_tuning.so, a build whose slice count
                                                                      #      can be forced through ECGEMM_FORCE_SLICES
    ECGEMM_LIB=paper_2203_03341_amd/libecgemm_tuning.so \
    python -m paper_2203_03341_amd.calibrate_plans sweep timings.jsonl   # GPU: both kernel shapes, every admissible slice
                                                                      #      count, about 170 problems in both modes
    python -m paper_2203_03341_amd.calibrate_plans fit timings.jsonl     # CPU: least squares on log time; prints the constants
                                                                      #      and how far the cheapest plan is from the best

The estimate itself is documented where it is used; `estimate_us` below is the same formula in Python and must be kept
in step with it.  Nothing here is needed to use the library.
"""
from __future__ import annotations

import collections
import json
import math
import os
import random
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
TUNING_LIB = os.path.join(HERE, "libecgemm_tuning.so")
UNITS = 256                                       # compute units the plans are made for
GEOMETRY = {1: (256, 128, UNITS), 2: (128, 128, 2 * UNITS)}   # shape -> tile rows, tile columns, workgroup slots
MODE_WORK = {0: 1.0, 1: 2.0}                      # matrix-pipe time per element relative to the three FP16 products
START = {"w4_unit": 22.0, "w4_work": 0.95, "x2_pair": 14.7, "x2_lone": 10.0, "x2_lone_per_depth": 0.28, "chip": 17.5,
         "fill_exponent": 0.9, "w4_round_us": 7.9, "x2_round_us": 4.7, "reduce_us": 1.0, "reduce_us_per_mb": 0.14}


def build_tuning_library() -> str:
    from . import build as b
    cmd = [b.HIPCC, *b.FLAGS, "-DECGEMM_TUNING", "-o", TUNING_LIB, *b.sources()]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    return TUNING_LIB


def problems(seed: int = 2):
    rng = random.Random(seed)
    out = [(n, n, n) for n in range(512, 5633, 512)]
    out += [(960, 2304, 18688), (3904, 640, 11808), (1920, 4800, 901), (6801, 2752, 608), (1536, 1536, 8192),
            (1024, 1024, 65536), (512, 512, 16384), (3000, 3000, 1100), (4095, 3001, 5003), (2048, 2048, 2048),
            (2304, 2304, 2304)]
    for _ in range(70):
        M, N, K = int(2 ** rng.uniform(9, 13.3)), int(2 ** rng.uniform(9, 13.3)), int(2 ** rng.uniform(8, 14.5))
        if M * N * K <= 6000 ** 3:
            out.append((M // 64 * 64 + rng.choice([0, 0, 0, 17]), N // 64 * 64 + rng.choice([0, 0, 3]),
                        K // 32 * 32 + rng.choice([0, 0, 5])))
    return out


def admissible_slices(M: int, N: int, K: int, shape: int):
    """Slice counts the planner may choose for the leftover tiles: at least 512 deep, none empty, at most 1024 in all."""
    bm, bn, slots = GEOMETRY[shape]
    tail = (-(-M // bm) * -(-N // bn)) % slots
    Kp = -(-K // 32) * 32
    stages = Kp // 32
    out = [1]
    if tail:
        out += [s for s in (2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32, 48, 64)
                if s <= Kp // 512 and s * tail <= 1024 and -(-stages // s) * (s - 1) < stages]
    return out


def sweep(path: str):
    import torch
    import paper_2203_03341_amd as ec
    from . import binding
    if os.path.abspath(binding.LIB_PATH) != TUNING_LIB:    # the binding picks its library when the package is imported
        raise SystemExit(f"build the tuning library and run with ECGEMM_LIB={TUNING_LIB}")
    h = ec.Handle()
    h.set_stream(torch.cuda.current_stream().cuda_stream)

    def timed(call, iters):
        call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            call()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters * 1e3

    with open(path, "w") as out:
        for mode in (ec.MODE_FP16_SPLIT, ec.MODE_BF16_FULL):
            for (M, N, K) in problems():
                A = torch.rand((K, M), device="cuda") * 2 - 1
                B = torch.rand((N, K), device="cuda") * 2 - 1
                C = torch.empty((N, M), device="cuda")
                iters = max(4, min(300, int(0.012 / (2 * M * N * K / 3e14 + 1e-5))))
                call = lambda: h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, A, M, B, K, 0.0, C, M, mode)
                for shape in (ec.SHAPE_256x128_W4, ec.SHAPE_128x128_X2):
                    h.set_shape(shape)
                    for slices in admissible_slices(M, N, K, shape):
                        os.environ["ECGEMM_FORCE_SLICES"] = str(slices)
                        us = sorted(timed(call, iters) for _ in range(3))[1]
                        h.set_timing(True)
                        for _ in range(4):
                            call()
                        torch.cuda.synchronize()
                        calls, split_ms, _ = h.get_timing()
                        h.set_timing(False)
                        out.write(json.dumps({"mode": mode, "M": M, "N": N, "K": K, "us": us, "split_us": split_ms / calls * 1e3,
                                              "plan": h.plan_info(M, N, K, mode)}) + "\n")
                        out.flush()
                print(mode, M, N, K, flush=True)


def rounds_us(items: int, depth: float, w4: bool, work: float, c: dict) -> float:
    """`items` equal items, each depth x 1024 deep, handed out in rounds of one (W4) or two (X2) per compute unit."""
    per_round = UNITS if w4 else 2 * UNITS
    us = 0.0
    while items > 0:
        n = min(items, per_round)
        if w4:
            unit = c["w4_unit"]
        else:
            unit = 2 * c["x2_pair"] if n > UNITS else c["x2_lone"] + c["x2_lone_per_depth"] * min(depth, 20.0)
        chip = 2.0 * (c["w4_work"] if w4 else 1.0) * (n / per_round) ** c["fill_exponent"] * c["chip"]
        us += depth * work * max(unit, chip) + (c["w4_round_us"] if w4 else c["x2_round_us"])
        items -= n
    return us


def estimate_us(row: dict, c: dict) -> float:
    p = row["plan"]
    w4 = p["tile_m"] == 256
    stage = 32 if w4 else 16
    Kp = -(-row["K"] // 32) * 32
    slices = p["slices"]
    sliced = p["sliced_tiles"] * slices if slices > 1 else 0
    slice_depth = -(-(Kp // stage) // slices) * stage / 1024.0 if slices > 1 else 0.0
    work = MODE_WORK[row["mode"]]
    us = rounds_us(p["whole_tiles"], Kp / 1024.0, w4, work, c) + rounds_us(sliced, slice_depth, w4, work, c)
    if sliced:
        us += c["reduce_us"] + c["reduce_us_per_mb"] * (slices + 1) * p["sliced_tiles"] * p["tile_m"] * p["tile_n"] * 4 / 1e6
    return us


def fit(path: str, steps: int = 12000, seed: int = 0):
    rows = [json.loads(line) for line in open(path)]
    groups = collections.defaultdict(list)
    for r in rows:
        groups[(r["mode"], r["M"], r["N"], r["K"])].append(r)

    def loss(c):  # mean squared log error of the whole call (the split pass is measured, not modelled)
        return sum(math.log((estimate_us(r, c) + r["split_us"]) / r["us"]) ** 2 for r in rows) / len(rows)

    def regret(c):  # how much slower the plan the estimate ranks first is than the best measured plan
        over = [min(g, key=lambda r: estimate_us(r, c))["us"] / min(r["us"] for r in g) - 1 for g in groups.values()]
        return sum(over) / len(over), sum(o > 0.05 for o in over), max(over)

    c, rng = dict(START), random.Random(seed)
    best = loss(c)
    for _ in range(steps):  # random coordinate search: ten smooth parameters, a few thousand rows
        k = rng.choice(list(c))
        old = c[k]
        c[k] = old * math.exp(rng.gauss(0, 0.04))
        now = loss(c)
        if now < best:
            best = now
        else:
            c[k] = old
    mean, over5, worst = regret(c)
    print("constants:", {k: round(v, 3) for k, v in c.items()})
    print(f"rms log error {math.sqrt(best):.3f}; cheapest plan is {100 * mean:.2f} % off the best on average, "
          f"{over5} of {len(groups)} problems more than 5 % (worst {100 * worst:.0f} %)")
    return c


if __name__ == "__main__":
    if len(sys.argv) >= 2 and sys.argv[1] == "build":
        print(build_tuning_library())
    elif len(sys.argv) == 3 and sys.argv[1] == "sweep":
        sweep(sys.argv[2])
    elif len(sys.argv) == 3 and sys.argv[1] == "fit":
        fit(sys.argv[2])
    else:
        raise SystemExit(__doc__)
