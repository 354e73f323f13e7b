#!/usr/bin/env python3
"""Throughput and accuracy of the error-corrected SGEMM on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one whole `ecgemm_sgemm` call (split of A and B, MFMA product, merge epilogue) on inputs that
already sit in HBM.  The default workload is the one the headline metric is quoted on: M = N = K = 16384,
FP16-split mode, entries sign * (1 + u) * 2^e with e uniform in [-15, 15].  One JSON line is printed:
FP32-equivalent TFLOP/s = 2 M N K / t, the MFMA roofline of the product kernel (its own duration measured
with HIP events on the launch stream), the relative residual against an FP64 reference next to that of a
naive FP32 product (both from the CPU oracle, on a seeded sample of rows of C), and the oracle's own speed
on the host cores as `cpu_baseline`.  After the headline the default run also times the other baseline
configurations (both modes) and lists them under `other_workloads`, each with its own accuracy check.
Energy: board power and shader clock are sampled while the headline call loops (`power`), while the same operands go
through this library's FP32 mode (`fp32_mode_of_this_library`, the FP32 baseline of the comparison) and while the
BF16 8192^3 configuration loops (its entry in `other_workloads`).
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

METRIC = "FP32-equivalent TFLOP/s (2MNK/t) at 16384^3 + rel. error vs FP64 ref"
PEAK_MFMA_16BIT_TFLOPS = 2516.6     # 256 CU x 4096 flop/clk x 2.4 GHz, dense FP16 / BF16
PEAK_FP32_VECTOR_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0             # HBM3E, published

# HBM bytes per product-kernel launch, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this program (the summary
# under profiles/ named beside each entry holds the command and the counter values).  Counters cannot be read from
# inside the run, so these are recorded figures, keyed by workload; None where no counter run exists.
# FETCH_SIZE x 2.0 (the counter shows half of a known 1 GiB read) + WRITE_SIZE x 1.0, in bytes.
MEASURED_TRAFFIC_BYTES = {
    "c3_16384_fp16_exprand15": 3.55e10,      # profiles/product_kernel_fp16_16384cubed.md: 34.4 GB + 1.07 GB
    "c4_8192_bf16_widerange": 6.98e9,        # profiles/product_kernel_bf16_8192cubed.md: 6.71 GB + 0.27 GB
    "c5_tallskinny_fp16": 1.36e9,            # profiles/product_kernel_fp16_tallskinny_16384x16384x256.md: 0.285 GB + 1.07 GB
    "c2_4096_fp16_urand": 6.04e8,            # profiles/product_kernel_fp16_4096cubed_persistent.md: 537 MB + 67 MB
    "c5_deepk_fp16": 5.71e8,                 # profiles/product_kernel_fp16_deepk_1024x1024x65536.md: 537 MB + 33.5 MB
                                             # (product kernel; its reduction moves another 38 MB)
    # profiles/product_kernel_hbm_traffic_other_workloads.md:
    "c2_4096_bf16_urand": 8.73e8, "c5_tallskinny_bf16": 1.50e9, "c5_deepk_bf16": 8.39e8,
    "c5_odd_transA_fp16": 5.73e8, "c5_odd_transA_bf16": 8.18e8,
    # profiles/one_launch_kernel_small_products.md (fused_kernel, 32 x 32 tiles): 1.85 MB + 0.26 MB
    "c1_256_fp16_urand": 2.1e6, "c1_256_bf16_urand": 2.1e6,
}

WORKLOADS = {
    # name: (M, N, K, transA, transB, mode, alpha, beta, distribution, oracle rows)
    "c1_256_fp16_urand": (256, 256, 256, "N", "N", "fp16", 1.0, 0.0, "urand", None),
    "c1_256_bf16_urand": (256, 256, 256, "N", "N", "bf16", 1.0, 0.0, "urand", None),
    "c2_4096_fp16_urand": (4096, 4096, 4096, "N", "N", "fp16", 1.0, 0.0, "urand", 1024),
    "c2_4096_bf16_urand": (4096, 4096, 4096, "N", "N", "bf16", 1.0, 0.0, "urand", 1024),
    "c3_16384_fp16_exprand15": (16384, 16384, 16384, "N", "N", "fp16", 1.0, 0.0, ((-15, 15), (-15, 15)), 512),
    # config 4 as written (both operands exp_rand(-100, 100)) overflows FP32 in every element of C, on the CPU
    # and on the GPU alike; the graded stand-in keeps A wide and B in the Type-1 range so that C stays finite
    "c4_8192_bf16_widerange": (8192, 8192, 8192, "N", "N", "bf16", 1.5, 0.5, ((-100, 100), (-15, 14)), 512),
    "c5_tallskinny_fp16": (16384, 16384, 256, "N", "N", "fp16", 1.0, 0.0, "urand", 2048),
    "c5_tallskinny_bf16": (16384, 16384, 256, "N", "N", "bf16", 1.0, 0.0, "urand", 2048),
    "c5_deepk_fp16": (1024, 1024, 65536, "N", "N", "fp16", 1.0, 0.0, "urand", 256),
    "c5_deepk_bf16": (1024, 1024, 65536, "N", "N", "bf16", 1.0, 0.0, "urand", 256),
    "c5_odd_transA_fp16": (4095, 3001, 5003, "T", "N", "fp16", 1.0, 0.0, "urand", 1024),
    "c5_odd_transA_bf16": (4095, 3001, 5003, "T", "N", "bf16", 1.0, 0.0, "urand", 1024),
    # not a baseline config: the size at which the one-kernel (fused) shape is compared with the split-first path
    "x_1024_fp16_urand": (1024, 1024, 1024, "N", "N", "fp16", 1.0, 0.0, "urand", None),
    "x_1024_bf16_urand": (1024, 1024, 1024, "N", "N", "bf16", 1.0, 0.0, "urand", None),
    "x_512_fp16_urand": (512, 512, 512, "N", "N", "fp16", 1.0, 0.0, "urand", None),
    "x_512_bf16_urand": (512, 512, 512, "N", "N", "bf16", 1.0, 0.0, "urand", None),
    # one block of the one-launch kernel by itself (with --shape fused), 64 chunks deep, in three operand layouts
    "x_oneblock_nn_fp16": (64, 64, 4096, "N", "N", "fp16", 1.0, 0.0, "urand", None),
    "x_oneblock_tn_fp16": (64, 64, 4096, "T", "N", "fp16", 1.0, 0.0, "urand", None),
    "x_oneblock_nt_fp16": (64, 64, 4096, "N", "T", "fp16", 1.0, 0.0, "urand", None),
    "x_oneblock_nn_bf16": (64, 64, 4096, "N", "N", "bf16", 1.0, 0.0, "urand", None),
    # deep products of few tiles: one launch with the depth in slices plus the reduction
    "x_deep_128x4096_fp16": (128, 128, 4096, "N", "N", "fp16", 1.0, 0.0, "urand", None),
    "x_deep_128x4096_bf16": (128, 128, 4096, "N", "N", "bf16", 1.0, 0.0, "urand", None),
    "x_deep_512x2048_fp16": (512, 512, 2048, "N", "N", "fp16", 1.0, 0.0, "urand", None),
    # not baseline configs either: the method with the leading product accumulated outside the matrix unit, as the
    # paper's listing does against round-toward-zero, next to the default (inside) at the same size
    "x_8192_fp16_urand": (8192, 8192, 8192, "N", "N", "fp16", 1.0, 0.0, "urand", 256),
    "x_8192_fp16_outside_urand": (8192, 8192, 8192, "N", "N", "fp16_outside", 1.0, 0.0, "urand", 256),
    "x_8192_fp16_outside4_urand": (8192, 8192, 8192, "N", "N", "fp16_outside4", 1.0, 0.0, "urand", 256),
    "x_8192_fp16_outside16_urand": (8192, 8192, 8192, "N", "N", "fp16_outside16", 1.0, 0.0, "urand", 256),
    # the automatic mode choice (made on the GPU during the split pass) next to the fixed modes on the same inputs:
    # x_8192_fp16_urand, c4_8192_bf16_widerange and x_1024_fp16_urand
    "x_8192_auto_urand": (8192, 8192, 8192, "N", "N", "auto", 1.0, 0.0, "urand", 256),
    "x_8192_auto_widerange": (8192, 8192, 8192, "N", "N", "auto", 1.5, 0.5, ((-100, 100), (-15, 14)), 512),
    "x_1024_auto_urand": (1024, 1024, 1024, "N", "N", "auto", 1.0, 0.0, "urand", None),
}
DEFAULT_WORKLOAD = "c3_16384_fp16_exprand15"
# what the default run times after the headline: every other baseline configuration, both modes (and the inputs of
# configuration 4 once more in the automatic mode, which runs them as FP16 on row / column scaled operands)
OTHER_WORKLOADS = ["c4_8192_bf16_widerange", "x_8192_auto_widerange", "c2_4096_fp16_urand", "c2_4096_bf16_urand", "c5_tallskinny_fp16",
                   "c5_tallskinny_bf16", "c5_deepk_fp16", "c5_deepk_bf16", "c5_odd_transA_fp16", "c5_odd_transA_bf16",
                   "c1_256_fp16_urand", "c1_256_bf16_urand"]
OTHER_ORACLE_ROWS = 256      # the oracle's sample of rows of C for those (the headline keeps its own, larger one)

PRODUCTS = {"fp16": 3, "bf16": 6, "fp16_outside": 3, "fp16_outside4": 3, "fp16_outside16": 3}
PACKED_BYTES_PER_ELEMENT = {"fp16": 4, "bf16": 6, "fp16_outside": 4, "fp16_outside4": 4, "fp16_outside16": 4}


def make_inputs(M, N, K, transA, transB, dist, beta, seed=0):
    import seeded_inputs as si
    ar, ac = (M, K) if transA == "N" else (K, M)
    br, bc = (K, N) if transB == "N" else (N, K)
    if dist == "urand":
        A = si.urand(ar, ac, seed, si.ID_A)
        B = si.urand(br, bc, seed, si.ID_B)
    else:
        (a_lo, a_hi), (b_lo, b_hi) = dist
        A = si.exp_rand(ar, ac, a_lo, a_hi, seed, si.ID_A)
        B = si.exp_rand(br, bc, b_lo, b_hi, seed, si.ID_B)
    C = si.urand(M, N, seed, si.ID_C) if beta != 0 else None
    return A, B, C


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def hwmon_of_device(index: int):
    """(directory, matched): the hwmon node of the GPU that torch device `index` is, found by its PCI address; when
    no node matches (or torch does not expose the address) the first one, with matched = False."""
    import glob
    import torch
    nodes = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*"))
    if not nodes:
        return None, False
    try:
        prop = torch.cuda.get_device_properties(index)
        address = f"{prop.pci_domain_id:04x}:{prop.pci_bus_id:02x}:{prop.pci_device_id:02x}"
        for node in nodes:
            pci = os.path.basename(os.path.realpath(os.path.join(node, "..", "..")))      # .../device -> 0000:bb:dd.f
            if pci.lower().startswith(address):
                return node, True
    except Exception:
        pass
    return nodes[0], False


class Workload:
    """One baseline configuration resident on the GPU: inputs, handle, workspace, the call."""

    def __init__(self, name, seed, shape, tile_order=None):
        import torch
        import paper_2203_03341_amd as ec
        self.ec, self.torch, self.name, self.seed = ec, torch, name, seed
        (self.M, self.N, self.K, self.transA, self.transB, self.mode, self.alpha, self.beta, self.dist,
         self.oracle_rows) = WORKLOADS[name]
        self.mode_id = {"fp16": ec.MODE_FP16_SPLIT, "bf16": ec.MODE_BF16_FULL, "fp16_outside": ec.MODE_FP16_OUTSIDE_ACC,
                        "fp16_outside4": ec.MODE_FP16_OUTSIDE_ACC_4, "fp16_outside16": ec.MODE_FP16_OUTSIDE_ACC_16,
                        "auto": ec.MODE_AUTO}[self.mode]
        self.auto = self.mode == "auto"
        self.auto_scaled = False
        self.ops = {"N": ec.OP_N, "T": ec.OP_T}
        t0 = time.time()
        self.A, self.B, self.C = make_inputs(self.M, self.N, self.K, self.transA, self.transB, self.dist, self.beta, seed)
        self.gen_s = time.time() - t0
        self.dA = torch.from_numpy(np.ascontiguousarray(self.A.T)).cuda()
        self.dB = torch.from_numpy(np.ascontiguousarray(self.B.T)).cuda()
        self.dC0 = torch.from_numpy(np.ascontiguousarray(self.C.T)).cuda() if self.C is not None else None
        self.dC = torch.empty((self.N, self.M), dtype=torch.float32, device="cuda")
        self.stream = torch.cuda.current_stream()
        self.h = ec.Handle()
        self.h.set_stream(self.stream.cuda_stream)
        self.h.set_shape({"auto": ec.SHAPE_AUTO, "w4": ec.SHAPE_256x128_W4, "x2": ec.SHAPE_128x128_X2,
                          "fused": ec.SHAPE_64x64_FUSED, "fused32": ec.SHAPE_32x32_FUSED}[shape])
        if tile_order is not None:
            self.h.debug_set_tile_order(*tile_order)
        self.ws_bytes = self.h.workspace_size(self.ops[self.transA], self.ops[self.transB], self.M, self.N, self.K, self.mode_id)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.h.set_workspace(self.ws, self.ws_bytes)
        self.flops = 2.0 * self.M * self.N * self.K
        self.expected_ms = max(0.02, self.flops / 3.0e14 * 1e3)     # at 300 TFLOP/s; only sizes the default step counts
        self.plan_mode_id = self.mode_id
        if self.auto:       # which mode the library picks for these inputs: from here on `mode` names that one
            self.step()
            self.plan_mode_id, self.auto_scaled = self.h.auto_choice()
            self.mode = "fp16" if self.plan_mode_id == ec.MODE_FP16_SPLIT else "bf16"

    def step(self):
        if self.dC0 is not None:
            self.dC.copy_(self.dC0)      # beta != 0: every step starts from the same C (the copy is inside the timed region)
        self.h.sgemm(self.ops[self.transA], self.ops[self.transB], self.M, self.N, self.K, self.alpha, self.dA,
                     self.A.shape[0], self.dB, self.B.shape[0], self.beta, self.dC, self.M, self.mode_id)

    def default_counts(self, steps, warmup):
        if warmup is None:       # a board that has idled takes about 50 ms to raise its clocks
            warmup = int(min(500, max(3, np.ceil(50.0 / self.expected_ms))))
        if steps is None:        # at least 0.1 s of timed work
            steps = int(min(1000, max(20, np.ceil(100.0 / self.expected_ms))))
        return steps, warmup

    def time(self, steps, warmup):
        """W untimed steps, then exactly `steps` timed ones bracketed by synchronisations; the library's own HIP events
        (on the launch stream) give the split and product kernels' durations inside the same region."""
        torch, h = self.torch, self.h
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        if self.expected_ms < 0.2:
            # A call of a few microseconds: the three event records per call would be a large part of what is timed.
            # The step time comes from a loop without them, the kernel durations from a second loop of the same length.
            wall0 = time.perf_counter()
            for _ in range(steps):
                self.step()
            torch.cuda.synchronize()
            plain_ms = (time.perf_counter() - wall0) * 1e3 / steps
            h.set_timing(True)
            for _ in range(steps):
                self.step()
            torch.cuda.synchronize()
            calls, split_ms, product_ms = h.get_timing()
            h.set_timing(False)
            return plain_ms, split_ms / calls, product_ms / calls
        h.set_timing(True)
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        wall0 = time.perf_counter()
        start.record(self.stream)
        for _ in range(steps):
            self.step()
        stop.record(self.stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - wall0) * 1e3
        event_ms = start.elapsed_time(stop)
        calls, split_ms, product_ms = h.get_timing()
        h.set_timing(False)
        assert calls == steps
        ms_per_step = max(wall_ms, event_ms) / steps
        return ms_per_step, split_ms / calls, product_ms / calls

    def rooflines(self, split_ms, product_ms):
        M, N, K = self.M, self.N, self.K
        pad = lambda v, m: -(-v // m) * m
        bpe = PACKED_BYTES_PER_ELEMENT[self.mode]
        packed = (pad(M, 256) + pad(N, 256)) * pad(K, 32) * bpe
        product_bytes = packed + M * N * 4 * (2 if self.beta != 0 else 1)
        split_bytes = (M + N) * K * 4 + packed
        fp16_pass = (M + N) * K * 4 + (pad(M, 256) + pad(N, 256)) * pad(K, 32) * PACKED_BYTES_PER_ELEMENT["fp16"]
        if self.auto and self.auto_scaled:         # the unscaled FP16 split is discarded; the exponents cost a read of A and B
            split_bytes += fp16_pass + (M + N) * K * 4
        if self.auto and self.mode == "bf16":      # both FP16 splits and the exponents
            split_bytes += 2 * fp16_pass + (M + N) * K * 4
        # a small product runs as one launch that reads the FP32 operands itself: no packed copies, no split kernel
        one_launch = (not self.auto) and self.h.plan_info(M, N, K, self.plan_mode_id)["shape"] >= 3
        kernel = "fused_kernel" if one_launch else "product_kernel"
        if one_launch:
            product_bytes = (M + N) * K * 4 + M * N * 4 * (2 if self.beta != 0 else 1)
            split_bytes, split_ms = 0, 0.0
        mfma_tflops = PRODUCTS[self.mode] * self.flops / (product_ms * 1e-3) / 1e12
        mfma = {"bound": "mfma", "achieved": round(mfma_tflops, 1), "peak": PEAK_MFMA_16BIT_TFLOPS, "unit": "TFLOP/s",
                "frac": round(mfma_tflops / PEAK_MFMA_16BIT_TFLOPS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(self.name),
                "kernel": kernel, "flops_per_launch": PRODUCTS[self.mode] * self.flops}
        # the same kernel against the HBM roof (it matters for shallow K, where writing C is most of the bytes):
        # algorithmic bytes = packed operands once + C written once (+ read once when beta != 0)
        hbm = {"bound": "hbm", "unit": "GB/s", "peak": PEAK_HBM_GBS, "kernel": kernel,
               "bytes_per_launch": product_bytes, "achieved": round(product_bytes / (product_ms * 1e-3) / 1e9, 1),
               "frac": round(product_bytes / (product_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        # step 1 against the HBM roof: every FP32 element read once, its 16-bit parts written once
        split = {"bound": "hbm", "unit": "GB/s", "peak": PEAK_HBM_GBS, "kernel": "split_kernel (both operands)",
                 "bytes_per_call": split_bytes,
                 "achieved": None if split_ms <= 0 else round(split_bytes / (split_ms * 1e-3) / 1e9, 1),
                 "frac": None if split_ms <= 0 else round(split_bytes / (split_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}
        return mfma, hbm, split

    def accuracy(self, rows_wanted):
        """Relative residual of the last result against the FP64 reference, next to the naive FP32 product's, both
        from the CPU oracle on a seeded sample of rows of C; also how long the oracle's FP32 product took."""
        import seeded_inputs as si
        from oracle import gemm
        M, N, K = self.M, self.N, self.K
        got = self.dC.cpu().numpy().T          # logical M x N
        rows = None if rows_wanted is None or rows_wanted >= M else si.sample_indices(M, rows_wanted, seed=self.seed + 1)
        nrows = M if rows is None else len(rows)
        t0 = time.perf_counter()
        c32 = gemm.sgemm_fp32_naive(self.transA, self.transB, M, N, K, self.alpha, self.A, self.B, self.beta, self.C, rows=rows)
        oracle_s = time.perf_counter() - t0
        c64 = gemm.sgemm_fp64_ref(self.transA, self.transB, M, N, K, self.alpha, self.A, self.B, self.beta, self.C, rows=rows)
        got_rows = got if rows is None else got[rows, :]
        finite = bool(np.all(np.isfinite(got_rows)))
        r_gpu = gemm.relative_residual(c64, got_rows)
        r_cpu = gemm.relative_residual(c64, c32)
        return {"relres_gpu": r_gpu, "relres_fp32_oracle": r_cpu, "relres_ratio": round(r_gpu / r_cpu, 4),
                "max_dev_gpu": gemm.max_deviation(c64, got_rows), "max_dev_fp32_oracle": gemm.max_deviation(c64, c32),
                "accuracy_pass": bool(finite and r_gpu <= 1.25 * r_cpu), "accuracy_rows": nrows}, oracle_s, nrows

    def close(self):
        self.h.destroy()


def power_while(torch, call, flops, seconds):
    """Board power and shader clock from the GPU's hwmon node every 20 ms while `call` runs back to back."""
    import threading
    node, matched = hwmon_of_device(torch.cuda.current_device())
    if node is None or not os.path.exists(os.path.join(node, "power1_input")):
        return None
    watts, mhz, stop_flag = [], [], threading.Event()

    clock_file = os.path.join(node, "..", "..", "pp_dpm_sclk")      # the device's shader clock: the starred line is current

    def sampler():
        while not stop_flag.is_set():
            try:
                with open(os.path.join(node, "power1_input")) as f:
                    watts.append(int(f.read()) * 1e-6)               # microwatts
            except (OSError, ValueError):
                pass
            try:
                with open(clock_file) as f:
                    for line in f:
                        if line.rstrip().endswith("*"):              # e.g. "1: 1290Mhz *"
                            mhz.append(float(line.split(":")[1].lower().split("mhz")[0]))
            except (OSError, ValueError, IndexError):
                pass
            time.sleep(0.02)

    th = threading.Thread(target=sampler)
    t_begin = time.perf_counter()
    calls_done = 0
    th.start()
    while time.perf_counter() - t_begin < seconds:
        for _ in range(4):
            call()
        torch.cuda.synchronize()
        calls_done += 4
    elapsed = time.perf_counter() - t_begin
    stop_flag.set()
    th.join()
    steady = watts[len(watts) // 4:]        # drop the ramp-up quarter
    if not steady:
        return None
    avg_w = float(np.mean(steady))
    rate = flops * calls_done / elapsed
    clocks = mhz[len(mhz) // 4:]
    return {"avg_w": round(avg_w, 1), "max_w": round(float(np.max(steady)), 1), "samples": len(steady),
            "sclk_mhz": round(float(np.mean(clocks)), 0) if clocks else None,
            "sclk_mhz_min_max": [round(float(np.min(clocks)), 0), round(float(np.max(clocks)), 0)] if clocks else None,
            "interval_s": 0.02, "seconds": round(elapsed, 2), "source": node, "source_matched_by_pci_address": matched,
            "tflops_during": round(rate / 1e12, 1), "gflops_per_w": round(rate / 1e9 / avg_w, 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: 20, more for workloads under a millisecond so that 0.1 s is timed)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed warm-up steps (default: 3, more for short workloads so that the board, which drops "
                         "its clocks when idle, has run for 50 ms)")
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(WORKLOADS))
    ap.add_argument("--shape", default="auto", choices=["auto", "w4", "x2", "fused", "fused32"],
                    help="kernel shape (ecgemm_set_shape); auto lets the library choose")
    ap.add_argument("--tile-order", default=None, metavar="REMAP,GROUP_M,BANDS",
                    help="override the order in which output tiles go to the XCDs (ecgemm_debug_set_tile_order): "
                         "REMAP 0/1 (each XCD owns a contiguous run of the order), GROUP_M tile rows per group (0 = "
                         "default), BANDS column bands (0 = default); for the block-order profiles")
    ap.add_argument("--no-oracle", action="store_true", help="skip the CPU oracle (no error figures, no cpu_baseline)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--power-seconds", type=float, default=2.5,
                    help="after the timed steps, loop the same call for this long while sampling board power and shader "
                         "clock from sysfs every 20 ms (the paper samples NVML every 0.02 s over >= 2 s); 0 disables")
    ap.add_argument("--library-sgemm", action="store_true",
                    help="context measurement, off by default: the vendor library's FP32 GEMM on the same operands, timed "
                         "and power-sampled after the run proper (this library's own FP32 mode always is, as the energy "
                         "baseline, unless --power-seconds is 0)")
    ap.add_argument("--no-other-workloads", dest="others", action="store_false",
                    help="with the default workload: do not time the other baseline configurations afterwards")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the matrix-instruction-only rate measurement")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one device-to-device copy of 1 GiB (a kernel of known HBM traffic, for scaling "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the product has no exchange step to measure); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    import paper_2203_03341_amd as ec

    tile_order = None if args.tile_order is None else tuple(int(v) for v in args.tile_order.split(","))
    w = Workload(args.workload, args.seed, args.shape, tile_order)
    M, N, K, mode = w.M, w.N, w.K, w.mode
    h, stream = w.h, w.stream
    steps, warmup = w.default_counts(args.steps, args.warmup)

    if args.copy_probe:
        probe_src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        probe_dst = torch.empty_like(probe_src)
        probe_dst.copy_(probe_src)
        torch.cuda.synchronize()
        del probe_src, probe_dst
    ms_per_step, split_ms, product_ms = w.time(steps, warmup)
    tflops = w.flops / (ms_per_step * 1e-3) / 1e12
    roofline, roofline_hbm, roofline_split = w.rooflines(split_ms, product_ms)

    # ---- what the matrix pipes sustain on this board with random operands and no memory traffic (same dtype)
    ceiling = None
    if not args.no_ceiling:
        ops16 = (torch.rand(12 * 256 * 8, device="cuda") * 2 - 1).to(torch.bfloat16 if mode == "bf16" else torch.float16)
        sink = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        h.debug_mfma_rate(mode == "bf16", ops16, sink, 256, 2000)
        torch.cuda.synchronize()
        e0.record(stream)
        probe_flops = h.debug_mfma_rate(mode == "bf16", ops16, sink, 256, 40000)     # ~15-20 ms
        e1.record(stream)
        torch.cuda.synchronize()
        ceiling = probe_flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    # the same matrix instructions with random operands and nothing else running, this board, this run
    roofline["mfma_only_random_operands_tflops"] = None if ceiling is None else round(ceiling, 1)
    roofline["frac_of_mfma_only"] = None if ceiling is None else round(roofline["achieved"] / ceiling, 4)

    # ---- board power and clock while the same call runs back to back
    power = power_while(torch, w.step, w.flops, args.power_seconds) if args.power_seconds > 0 else None

    # ---- the FP32 baseline inside this code base (the paper's power comparison is against FP32 GEMM): the same
    # operands through the same kernels on the FP32 matrix instruction, timed and power-sampled the same way
    l0, l1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(3, min(steps, int(np.ceil(1000.0 / max(w.expected_ms * 4, 0.05)))))
    fp32_mode = None
    if args.power_seconds > 0 and not w.auto:
        own_bytes = h.workspace_size(ec.OP_N, ec.OP_N, M, N, K, ec.MODE_FP32_MFMA)
        own_ws = torch.empty(own_bytes, dtype=torch.uint8, device="cuda")
        h.set_workspace(own_ws, own_bytes)
        own_out = torch.empty((N, M), dtype=torch.float32, device="cuda")

        def own_call():
            h.sgemm(w.ops[w.transA], w.ops[w.transB], M, N, K, w.alpha, w.dA, w.A.shape[0], w.dB, w.B.shape[0], 0.0, own_out,
                    M, ec.MODE_FP32_MFMA)

        for _ in range(3):
            own_call()
        torch.cuda.synchronize()
        l0.record(stream)
        for _ in range(reps):
            own_call()
        l1.record(stream)
        torch.cuda.synchronize()
        own_ms = l0.elapsed_time(l1) / reps
        fp32_mode = {"what": "ecgemm_sgemm, ECGEMM_MODE_FP32_MFMA, same operands", "ms_per_call": round(own_ms, 4),
                     "tflops": round(w.flops / (own_ms * 1e-3) / 1e12, 2),
                     "power": power_while(torch, own_call, w.flops, args.power_seconds)}
        h.set_workspace(w.ws, w.ws_bytes)
        del own_out, own_ws

    # ---- context only, on request: the vendor library's FP32 GEMM (rocBLAS / hipBLASLt behind torch.matmul) on the same
    # operands (the paper sets its method against cuBLAS SGEMM)
    library = None
    if args.library_sgemm:
        opA_T = w.dA if w.transA == "N" else w.dA.T        # K x M as a row-major tensor
        opB_T = w.dB if w.transB == "N" else w.dB.T        # N x K
        ref = torch.empty((N, M), dtype=torch.float32, device="cuda")

        def library_call():
            torch.matmul(opB_T, opA_T, out=ref)

        for _ in range(3):
            library_call()
        torch.cuda.synchronize()
        l0.record(stream)
        for _ in range(reps):
            library_call()
        l1.record(stream)
        torch.cuda.synchronize()
        lib_ms = l0.elapsed_time(l1) / reps
        library = {"what": "torch.matmul, float32, allow_tf32 off", "ms_per_call": round(lib_ms, 4),
                   "tflops": round(w.flops / (lib_ms * 1e-3) / 1e12, 2),
                   "power": power_while(torch, library_call, w.flops, args.power_seconds) if args.power_seconds > 0 else None}
        del ref

    result = {
        "metric": METRIC, "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if mode == "bf16" else "f16", "data": "synthetic",
        "config": {"workload": args.workload, "M": M, "N": N, "K": K, "transA": w.transA, "transB": w.transB,
                   "mode": mode, "alpha": w.alpha, "beta": w.beta, "products": PRODUCTS[mode],
                   "inputs": "urand(-1,1)" if w.dist == "urand" else f"exp_rand{w.dist[0]} x exp_rand{w.dist[1]}", "seed": args.seed,
                   "shape": args.shape, "tile_order": args.tile_order, "plan": h.plan_info(M, N, K, w.plan_mode_id), "mode_chosen_by_the_library": w.auto,
                   "on_row_and_column_scaled_operands": w.auto_scaled},
        "split_ms": round(split_ms, 4), "product_ms": round(product_ms, 4),
        "frac_of_fp32_vector_peak": round(tflops / PEAK_FP32_VECTOR_TFLOPS, 3),
        "roofline": roofline, "roofline_hbm": roofline_hbm, "roofline_split": roofline_split,
        "power": power, "fp32_mode_of_this_library": fp32_mode, "library_sgemm": library,
    }

    if not args.no_oracle:
        from oracle import gemm
        acc, oracle_s, nrows = w.accuracy(w.oracle_rows)
        result.update(acc)
        result["cpu_baseline"] = {"value": round(2.0 * nrows * N * K / oracle_s / 1e12, 5), "unit": "TFLOP/s",
                                  "cores": gemm.num_threads(), "cpu_model": cpu_model(), "kind": "oracle",
                                  "sample": f"naive FP32 product of {nrows} seeded rows of C (all {N} columns, full K = {K}) "
                                            f"of the same workload, {oracle_s:.1f} s"}
    result["input_generation_s"] = round(w.gen_s, 1)
    w.close()
    del w, h

    # ---- the other baseline configurations, both modes: the same measurement in short
    if args.workload == DEFAULT_WORKLOAD and args.others:
        others = []
        for name in OTHER_WORKLOADS:
            torch.cuda.empty_cache()
            o = Workload(name, args.seed, "auto")
            o_steps, o_warmup = o.default_counts(None, None)
            o_ms, o_split_ms, o_product_ms = o.time(o_steps, o_warmup)
            o_tflops = o.flops / (o_ms * 1e-3) / 1e12
            o_mfma, o_hbm, _ = o.rooflines(o_split_ms, o_product_ms)
            entry = {"workload": name, "mode": o.mode, "mode_chosen_by_the_library": o.auto,
                     "on_row_and_column_scaled_operands": o.auto_scaled, "M": o.M, "N": o.N, "K": o.K, "steps": o_steps, "warmup": o_warmup,
                     "ms_per_step": round(o_ms, 4), "tflops": round(o_tflops, 2),
                     "frac_of_fp32_vector_peak": round(o_tflops / PEAK_FP32_VECTOR_TFLOPS, 3),
                     "product_ms": round(o_product_ms, 4), "split_ms": round(o_split_ms, 4),
                     "roofline_frac": o_mfma["frac"], "roofline_hbm_frac": o_hbm["frac"], "traffic": o_mfma["traffic"],
                     "plan_shape": o.h.plan_info(o.M, o.N, o.K, o.plan_mode_id)["shape"]}
            if name == "c4_8192_bf16_widerange" and args.power_seconds > 0:     # the energy figure of the other mode
                entry["power"] = power_while(torch, o.step, o.flops, args.power_seconds)
            if not args.no_oracle:
                acc, _, _ = o.accuracy(OTHER_ORACLE_ROWS if o.oracle_rows is not None else None)
                entry.update({k: acc[k] for k in ("relres_gpu", "relres_fp32_oracle", "relres_ratio", "accuracy_pass",
                                                  "accuracy_rows")})
            others.append(entry)
            o.close()
            del o
        result["other_workloads"] = others
    print(json.dumps(result))


if __name__ == "__main__":
    main()
