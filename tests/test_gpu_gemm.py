"""Whole-path parity: ecgemm_sgemm through the C-ABI against the CPU oracle.

Pass rule (the accuracy bar of the method): the relative residual of the GPU result against the FP64
reference is at most 1.25 x that of the naive FP32 product on the same inputs.  The exact bits of an
FP32 GEMM depend on the summation order, so bit parity with any CPU loop is not defined; what is
unique is checked element by element instead:

  * against the exact-accumulation model of the method (same split, FP64 sums) the GPU result may only
    differ by its FP32 accumulation.  The matrix unit adds eight products to the accumulator per
    rounding, each rounding is to nearest (relative 2^-24) after an alignment that drops less than
    2^-24 of the largest addend, so |C_gpu - C_model| <= (K / 8 + 4) * 2^-23 * (|A| |B|) element-wise.
  * integer inputs whose partial sums stay below 2^24 must come out exact, bit for bit.
"""
import numpy as np
import pytest

import seeded_inputs as si
from oracle import gemm, model
from gpu_util import empty_colmajor, to_device, to_host

pytestmark = pytest.mark.gpu

RATIO = 1.25


def _modes():
    import paper_2203_03341_amd as ec
    return {"fp16": ec.MODE_FP16_SPLIT, "bf16": ec.MODE_BF16_FULL, "markidis": ec.MODE_FP16_MARKIDIS,
            "unscaled": ec.MODE_FP16_UNSCALED, "plain16": ec.MODE_FP16_PLAIN, "plainbf": ec.MODE_BF16_PLAIN,
            "outside": ec.MODE_FP16_OUTSIDE_ACC, "outside4": ec.MODE_FP16_OUTSIDE_ACC_4,
            "outside16": ec.MODE_FP16_OUTSIDE_ACC_16, "fp32": ec.MODE_FP32_MFMA}


def _model(mode, opA, opB):
    """Exact-accumulation model of a mode (FP64 sums of the same low-precision parts)."""
    return {"fp16": lambda: model.gemm_fp16_mode(opA, opB), "bf16": lambda: model.gemm_bf16_mode(opA, opB),
            "outside": lambda: model.gemm_fp16_mode(opA, opB), "outside4": lambda: model.gemm_fp16_mode(opA, opB),
            "outside16": lambda: model.gemm_fp16_mode(opA, opB),
            "markidis": lambda: model.gemm_fp16_mode(opA, opB, products=4, scaled=False),
            "unscaled": lambda: model.gemm_fp16_mode(opA, opB, products=3, scaled=False),
            "plain16": lambda: model.gemm_plain(opA, opB, "fp16"),
            "plainbf": lambda: model.gemm_plain(opA, opB, "bf16"),
            "fp32": lambda: opA.astype(np.float64) @ opB.astype(np.float64)}[mode]()


def _shapes():
    import paper_2203_03341_amd as ec
    return {None: ec.SHAPE_AUTO, "w4": ec.SHAPE_256x128_W4, "x2": ec.SHAPE_128x128_X2, "fused": ec.SHAPE_64x64_FUSED,
            "fused32": ec.SHAPE_32x32_FUSED}


def _gpu_sgemm(transA, transB, M, N, K, alpha, A, B, beta, C, mode, ldc=None, handle=None, shape=None):
    import torch
    import paper_2203_03341_amd as ec
    h = handle or ec.Handle()
    if shape is not None:
        h.set_shape(_shapes()[shape])
    dA, dB = to_device(A), to_device(B)
    ldc = ldc or (C.shape[0] if C is not None else M)
    if C is not None:
        dC = to_device(C)
    else:
        dC = empty_colmajor(ldc, N, fill=float("nan"))
    ops = {"N": ec.OP_N, "T": ec.OP_T}
    h.sgemm(ops[transA], ops[transB], M, N, K, alpha, dA, A.shape[0], dB, B.shape[0], beta, dC, ldc, _modes()[mode])
    torch.cuda.synchronize()
    out = to_host(dC, ldc, N)
    if handle is None:
        h.destroy()
    return out


def _inputs(M, N, K, transA, transB, dist, seed, pad=0):
    ar, ac = (M, K) if transA == "N" else (K, M)
    br, bc = (K, N) if transB == "N" else (N, K)
    if dist == "urand":
        A = si.urand(ar, ac, seed, si.ID_A, ld=ar + pad)
        B = si.urand(br, bc, seed, si.ID_B, ld=br + pad)
    else:
        (a_lo, a_hi), (b_lo, b_hi) = dist
        A = si.exp_rand(ar, ac, a_lo, a_hi, seed, si.ID_A, ld=ar + pad)
        B = si.exp_rand(br, bc, b_lo, b_hi, seed, si.ID_B, ld=br + pad)
    return A, B


def _check(transA, transB, M, N, K, alpha, beta, mode, dist, seed=0, pad=0, rows=None, elementwise=True,
           ratio_rule=True, shape=None):
    A, B = _inputs(M, N, K, transA, transB, dist, seed, pad)
    C = si.urand(M, N, seed, si.ID_C, ld=M + pad) if beta != 0 else None
    got_store = _gpu_sgemm(transA, transB, M, N, K, alpha, A, B, beta, C, mode, ldc=M + pad, shape=shape)
    got = got_store[:M, :N]
    if pad and beta != 0:
        # rows beyond M belong to the caller and must be left alone (they hold NaN from the generator)
        assert np.all(np.isnan(got_store[M:, :]))
    if rows is not None:
        got = got[rows, :]
    c64 = gemm.sgemm_fp64_ref(transA, transB, M, N, K, alpha, A, B, beta, C, rows=rows)
    c32 = gemm.sgemm_fp32_naive(transA, transB, M, N, K, alpha, A, B, beta, C, rows=rows)
    assert np.all(np.isfinite(got))
    r_gpu = gemm.relative_residual(c64, got)
    r_cpu = gemm.relative_residual(c64, c32)
    if ratio_rule:
        assert r_gpu <= RATIO * r_cpu, (mode, M, N, K, r_gpu, r_cpu, r_gpu / r_cpu)
    else:
        # a handful of products: the statistical rule means nothing (one FP32 product has a single 2^-24
        # rounding, the FP16 pair may be off by an ulp, 2^-23, per input); bound every element instead
        opA_, opB_ = gemm.logical(transA, A, M, K), gemm.logical(transB, B, K, N)
        mag_ = np.abs(alpha) * (np.abs(opA_).astype(np.float64) @ np.abs(opB_).astype(np.float64))
        assert np.all(np.abs(got - c64) <= (2.0 ** -22 + (K / 8 + 4) * 2.0 ** -23) * mag_ + 1e-300)
    if elementwise:
        opA = gemm.logical(transA, A, M, K)
        opB = gemm.logical(transB, B, K, N)
        if rows is not None:
            opA = opA[rows, :]
        mdl = _model(mode, opA, opB)
        mag = np.abs(opA).astype(np.float64) @ np.abs(opB).astype(np.float64)
        want = alpha * mdl
        bound = (K / 8 + 4) * 2.0 ** -23 * abs(alpha) * mag
        if beta != 0:
            cin = C[:M, :N] if rows is None else C[:M, :N][rows, :]
            want = want + beta * cin.astype(np.float64)
            bound = bound + 2.0 ** -22 * (np.abs(want) + np.abs(beta * cin))
        worst = np.max(np.abs(got - want) / (bound + 1e-300))
        assert worst <= 1.0, (mode, M, N, K, worst)
    return r_gpu, r_cpu


# ----- config 1 of the baseline and friends: small, full oracle, several tiles plus a ragged tail

@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_config1_256_cubed(mode):
    _check("N", "N", 256, 256, 256, 1.0, 0.0, mode, "urand", seed=0)


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
@pytest.mark.parametrize("transA", ["N", "T"])
@pytest.mark.parametrize("transB", ["N", "T"])
@pytest.mark.parametrize("shape", [None, "fused", "fused32"])
def test_transposes_ragged_and_alpha_beta(mode, transA, transB, shape):
    _check(transA, transB, 300, 200, 77, 1.5, 0.5, mode, "urand", seed=1, pad=3, shape=shape)
    _check(transA, transB, 513, 259, 130, -1.0, 1.0, mode, "urand", seed=2, pad=1, shape=shape)
    _check(transA, transB, 260, 132, 96, 1.0, 0.0, mode, "urand", seed=3, pad=0, shape=shape)   # 16-byte aligned rows


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_tiny_shapes(mode):
    for (M, N, K) in [(1, 1, 1), (2, 3, 5), (17, 5, 8), (31, 33, 15), (64, 1, 100), (1, 257, 33)]:
        _check("N", "N", M, N, K, 1.0, 0.0, mode, "urand", seed=M + N + K, ratio_rule=False)


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_small_integers_bit_exact(mode):
    """Exact products of small integers: every summation order gives the same FP32 bits."""
    M, N, K = 320, 192, 2048
    A = si.randint(M, K, -15, 15, 0, si.ID_A)
    B = si.randint(K, N, -15, 15, 0, si.ID_B)
    exact = (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float32)
    got = _gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, mode)
    assert np.array_equal(got[:M, :N].view(np.uint32), exact.view(np.uint32))
    # integers that need the low parts (|a| up to 2^15: 16 significant bits), sums still below 2^24
    A2 = si.randint(M, 16, -(2 ** 15), 2 ** 15, 1, si.ID_A)
    B2 = si.randint(16, N, -3, 3, 1, si.ID_B)
    exact2 = (A2.astype(np.int64) @ B2.astype(np.int64))
    assert np.abs(exact2).max() < 2 ** 24
    got2 = _gpu_sgemm("N", "N", M, N, 16, 1.0, A2, B2, 0.0, None, mode)[:M, :N]
    assert np.array_equal(got2.astype(np.int64), exact2)


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_degenerate_cases(mode):
    import torch
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    m = _modes()[mode]
    M, N, K = 70, 50, 40
    A, B = _inputs(M, N, K, "N", "N", "urand", 3)
    C = si.urand(M, N, 3, si.ID_C)
    dA, dB = to_device(A), to_device(B)
    # K == 0 and alpha == 0: C <- beta * C
    for (kk, alpha) in [(0, 1.0), (K, 0.0)]:
        dC = to_device(C)
        h.sgemm(ec.OP_N, ec.OP_N, M, N, kk, alpha, dA, M, dB, max(K, 1), 0.5, dC, M, m)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(dC, M, N), (np.float32(0.5) * C).astype(np.float32))
        dC = empty_colmajor(M, N, fill=float("nan"))
        h.sgemm(ec.OP_N, ec.OP_N, M, N, kk, alpha, dA, M, dB, max(K, 1), 0.0, dC, M, m)
        torch.cuda.synchronize()
        assert np.all(to_host(dC, M, N) == 0.0)
    # M == 0 / N == 0: nothing is touched, null pointers are fine
    h.sgemm(ec.OP_N, ec.OP_N, 0, N, K, 1.0, None, 1, dB, K, 0.0, None, 1, m)
    h.sgemm(ec.OP_N, ec.OP_N, M, 0, K, 1.0, dA, M, None, K, 0.0, None, M, m)
    # beta == 0 must not read C: NaN already there does not propagate
    dC = empty_colmajor(M, N, fill=float("nan"))
    h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, m)
    torch.cuda.synchronize()
    assert np.all(np.isfinite(to_host(dC, M, N)))
    h.destroy()


def test_importing_the_package_before_torch_leaves_the_gpu_usable():
    """PyTorch ships its own HIP runtime; the binding must not bring the system's copy into the process ahead of it
    (torch then reports no GPU).  Checked in a fresh interpreter, package first."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import paper_2203_03341_amd as ec, torch; assert torch.cuda.is_available(); "
            "h = ec.Handle(); x = torch.ones(4, device='cuda'); torch.cuda.synchronize(); h.destroy(); print('ok')")
    res = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0 and "ok" in res.stdout, res.stderr[-2000:]


@pytest.mark.parametrize("mode", ["fp16", "bf16", "fp32"])
def test_non_finite_inputs_stay_in_their_rows_and_columns(mode):
    """A NaN in A poisons its row of C, an infinity in B its column, and nothing else: exactly the entries that are not
    finite in the FP64 product.  (Whether an entry comes out as an infinity or as NaN is not promised: the parts of an
    infinity are an infinity and zero, and a correction product may turn the sum into NaN.)"""
    M, N, K = 300, 200, 150
    A, B = _inputs(M, N, K, "N", "N", "urand", 31)
    A, B = A.copy(order="F"), B.copy(order="F")
    A[3, 5] = np.nan            # A is M x K (column-major storage as a (ld, cols) array indexed [row, col])
    B[7, 2] = np.inf            # B is K x N
    got = _gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, mode)[:M, :N]
    with np.errstate(invalid="ignore", over="ignore"):
        ref = A.astype(np.float64) @ B.astype(np.float64)
    assert np.array_equal(np.isfinite(got), np.isfinite(ref))
    assert np.all(np.isnan(got[3, :])) and not np.any(np.isfinite(got[:, 2]))
    finite = np.isfinite(ref)
    assert np.max(np.abs(got[finite] - ref[finite])) < 1e-4


def test_invalid_arguments_are_rejected():
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    M = N = K = 64
    A, B = _inputs(M, N, K, "N", "N", "urand", 0)
    dA, dB = to_device(A), to_device(B)
    dC = empty_colmajor(M, N, fill=1.0)
    # (what is wrong, position of that argument in ecgemm_sgemm's parameter list, the handle being 1)
    bad_calls = [
        (dict(transA=7), 2), (dict(transB=-1), 3), (dict(mode=99), 15), (dict(mode=-1), 15), (dict(M=-1), 4), (dict(N=-2), 5),
        (dict(K=-3), 6), (dict(lda=M - 1), 9), (dict(ldb=K - 1), 11), (dict(ldc=M - 1), 14), (dict(A=None), 8), (dict(B=None), 10),
        (dict(C=None), 13), (dict(transA=5, C=None), 2),
    ]
    base = dict(transA=ec.OP_N, transB=ec.OP_N, M=M, N=N, K=K, alpha=1.0, A=dA, lda=M, B=dB, ldb=K, beta=0.0, C=dC,
                ldc=M, mode=ec.MODE_FP16_SPLIT)
    assert h.last_error_argument() == 0
    for call in (h.sgemm, h.sgemm_noalloc):
        for bad, position in bad_calls:
            args = dict(base, **bad)
            with pytest.raises(ec.EcgemmError) as ei:
                call(**args)
            assert ei.value.status == ec.ERR_INVALID_ARG, bad
            assert ei.value.argument == position == h.last_error_argument(), (bad, ei.value.argument)
    torch_sync = __import__("torch").cuda.synchronize
    torch_sync()
    assert np.all(to_host(dC, M, N) == 1.0)          # none of the refused calls touched C
    # a caller workspace that is too small is refused before anything is launched (with the split-first shape forced:
    # left to itself the library runs a product this small as one launch, which needs no workspace)
    import torch
    h.set_shape(ec.SHAPE_128x128_X2)
    ws = torch.empty(1024, dtype=torch.uint8, device="cuda")
    h.set_workspace(ws, 1024)
    with pytest.raises(ec.EcgemmError) as ei:
        h.sgemm(**base)
    assert ei.value.status == ec.ERR_ALLOC and ei.value.argument == 0
    torch.cuda.synchronize()
    assert np.all(to_host(dC, M, N) == 1.0)
    need = h.workspace_size(ec.OP_N, ec.OP_N, M, N, K, ec.MODE_FP16_SPLIT)
    assert need > 1024
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    h.set_workspace(ws, need)
    h.sgemm(**base)
    torch.cuda.synchronize()
    assert np.all(to_host(dC, M, N) != 1.0)
    h.set_workspace(None, 0)
    h.destroy()


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_bitwise_reproducible_and_stream(mode):
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = 512, 384, 4096          # K deep enough that the K range is divided among blocks
    A, B = _inputs(M, N, K, "N", "T", "urand", 5)
    h = ec.Handle()
    stream = torch.cuda.Stream()
    h.set_stream(stream.cuda_stream)
    h.set_timing(True)
    outs = []
    with torch.cuda.stream(stream):
        for _ in range(3):
            outs.append(_gpu_sgemm("N", "T", M, N, K, 1.0, A, B, 0.0, None, mode, handle=h))
    calls, split_ms, product_ms = h.get_timing()
    assert calls == 3 and split_ms > 0 and product_ms > 0
    h.destroy()
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))
    assert np.array_equal(outs[0].view(np.uint32), outs[2].view(np.uint32))


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
@pytest.mark.parametrize("size", [(1280, 1024, 3072), (300, 200, 260), (128, 128, 4096)])
def test_a_call_can_be_captured_in_a_graph_and_replayed(mode, size):
    """With a caller workspace the call only launches kernels (no allocation, no memset, no wait), so it can be recorded
    into a HIP graph.  Every replay, with eager work and synchronisations in between, must give the eager bits.
    The first size runs as split pair + product with every tile sliced along K + reduction, three kernels; the second
    as one launch that needs no workspace; the third as one launch with the depth in slices + reduction, whose partial
    sums are all the workspace holds."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = size
    A, B = _inputs(M, N, K, "N", "T", "urand", 12)
    C = si.urand(M, N, 12, si.ID_C)
    mode_id = _modes()[mode]
    h = ec.Handle()
    stream = torch.cuda.Stream()
    h.set_stream(stream.cuda_stream)
    nbytes = h.workspace_size(ec.OP_N, ec.OP_N, M, N, K, mode_id)
    plan = h.plan_info(M, N, K, mode_id)
    assert (plan["shape"] >= ec.SHAPE_64x64_FUSED) == (M <= 300) and (nbytes == 0) == (M == 300) and (plan["slices"] > 1) == (M != 300)
    workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    h.set_workspace(workspace, max(nbytes, 256))
    dA, dB, dC_in = to_device(A), to_device(B), to_device(C)
    dC = torch.empty_like(dC_in)
    other = torch.empty_like(dC_in)

    def call(out):
        out.copy_(dC_in)
        h.sgemm(ec.OP_N, ec.OP_T, M, N, K, 1.5, dA, A.shape[0], dB, B.shape[0], 0.5, out, M, mode_id)

    with torch.cuda.stream(stream):
        call(dC)
    stream.synchronize()
    eager = dC.cpu().numpy().copy()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        call(dC)
    for _ in range(3):
        with torch.cuda.stream(stream):
            dC.fill_(float("nan"))
            h.sgemm(ec.OP_N, ec.OP_T, M, N, K, -2.0, dA, A.shape[0], dB, B.shape[0], 0.0, other, M, mode_id)  # eager work
        stream.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(dC.cpu().numpy().view(np.uint32), eager.view(np.uint32))
    del graph
    h.destroy()


def test_two_handles_on_two_streams_do_not_interfere():
    """Each handle owns its workspace and its settings; calls enqueued alternately on two streams, in different modes
    and with different pre-scaling, give the bits each gives alone."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = 900, 700, 1300
    A, B = _inputs(M, N, K, "N", "N", "urand", 21)
    dA, dB = to_device(A), to_device(B)
    handles, streams, outs, alone = [], [], [], []
    for i, (mode, scale) in enumerate((("fp16", 3), ("bf16", 0))):
        h = ec.Handle()
        h.set_scaling(scale, -scale)
        alone.append(_gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, mode, handle=h))
        st = torch.cuda.Stream()
        h.set_stream(st.cuda_stream)
        handles.append((h, _modes()[mode]))
        streams.append(st)
        outs.append(empty_colmajor(M, N, fill=float("nan")))
    torch.cuda.synchronize()
    for _ in range(6):
        for (h, mode_id), st, out in zip(handles, streams, outs):
            with torch.cuda.stream(st):
                h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, out, M, mode_id)
    torch.cuda.synchronize()
    for out, want in zip(outs, alone):
        assert np.array_equal(to_host(out, M, N).view(np.uint32), want.view(np.uint32))
    for h, _ in handles:
        h.destroy()


# ----- the shape sweep of the baseline (config 5), reduced in size where the full oracle would take minutes

@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_deep_k_uses_split_k(mode):
    _check("N", "N", 256, 256, 16384, 1.0, 0.0, mode, "urand", seed=7)


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_tall_skinny(mode):
    rows = si.sample_indices(4096, 512, seed=1)
    _check("N", "N", 4096, 4096, 256, 1.0, 0.0, mode, "urand", seed=8, rows=rows)


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_odd_sizes_transA(mode):
    M, N, K = 1023, 751, 1251          # config 5's 4095 x 3001 x 5003 at a quarter of the size, same raggedness
    _check("T", "N", M, N, K, 1.0, 0.0, mode, "urand", seed=9)


# ----- seeded random shapes: tile and slice boundaries nobody thought of by hand

@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_shapes_transposes_and_scalars(seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(8):
        M, N = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        K = int(rng.choice([rng.integers(1, 130), rng.integers(130, 1100), rng.integers(1100, 2600)]))
        transA, transB = str(rng.choice(["N", "T"])), str(rng.choice(["N", "T"]))
        alpha = float(rng.choice([1.0, -1.0, 0.5, 1.5]))
        beta = float(rng.choice([0.0, 0.0, 1.0, -0.5]))
        mode = str(rng.choice(["fp16", "bf16"]))
        shape = rng.choice([None, None, "w4", "x2", "fused", "fused32"])
        shape = None if shape is None else str(shape)
        pad = int(rng.integers(0, 4))
        print(f"case {seed}.{case}: {transA}{transB} {M}x{N}x{K} alpha {alpha} beta {beta} {mode} shape {shape} pad {pad}", flush=True)
        _check(transA, transB, M, N, K, alpha, beta, mode, "urand", seed=seed * 100 + case, pad=pad, shape=shape,
               ratio_rule=K >= 64)


@pytest.mark.parametrize("seed", [0, 1])
def test_random_deep_products_of_few_tiles(seed):
    # few tiles and a deep k: the planner cuts the depth into slices over the blocks of one launch (or of the
    # split-first shapes beyond 8192); depths on both sides of every boundary it has, ragged last slices included
    import paper_2203_03341_amd as ec
    rng = np.random.default_rng(2000 + seed)
    h = ec.Handle()
    for case in range(6):
        M, N = int(rng.integers(1, 260)), int(rng.integers(1, 260))
        K = int(rng.choice([rng.integers(2600, 8192), rng.integers(8193, 24000), rng.choice([4096, 8191, 8192, 8193, 16385])]))
        transA, transB = str(rng.choice(["N", "T"])), str(rng.choice(["N", "T"]))
        alpha = float(rng.choice([1.0, -0.5, 1.5]))
        beta = float(rng.choice([0.0, 1.0, -0.5]))
        mode = str(rng.choice(["fp16", "bf16"]))
        pad = int(rng.integers(0, 4))
        p = h.plan_info(M, N, K, _modes()[mode])
        print(f"case {seed}.{case}: {transA}{transB} {M}x{N}x{K} alpha {alpha} beta {beta} {mode} pad {pad}: shape {p['shape']}, "
              f"{p['slices']} slices", flush=True)
        assert p["slices"] > 1
        _check(transA, transB, M, N, K, alpha, beta, mode, "urand", seed=seed * 100 + case, pad=pad)
    h.destroy()


# ----- every kernel shape on its own (the automatic choice exercises only one per size)

@pytest.mark.parametrize("mode", ["fp16", "bf16"])
@pytest.mark.parametrize("shape", ["w4", "x2", "fused", "fused32"])
def test_every_kernel_shape(mode, shape):
    _check("T", "N", 513, 259, 130, -1.0, 1.0, mode, "urand", seed=2, pad=1, shape=shape)        # ragged, several tiles
    _check("N", "T", 700, 900, 1500, 1.5, 0.5, mode, "urand", seed=3, shape=shape)               # every tile sliced along K
    _check("N", "N", 1, 1, 1, 1.0, 0.0, mode, "urand", seed=4, ratio_rule=False, shape=shape)


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
@pytest.mark.parametrize("shape", ["w4", "x2", "fused"])
def test_whole_tiles_followed_by_a_sliced_tail(mode, shape):
    """3000 x 3000: 288 tiles of 256 x 128 (256 whole + 32 in two slices) or 576 of 128 x 128 (512 whole + 64 sliced)."""
    rows = si.sample_indices(3000, 160, seed=2)
    _check("N", "N", 3000, 3000, 1100, 1.0, 0.5, mode, "urand", seed=5, rows=rows, shape=shape)


@pytest.mark.parametrize("case", [(8192, 8192, 2048, 1), (8192, 2048, 8192, 2), (4096, 4096 + 128, 16384, 4), (2048, 8192, 32800, 8)])
def test_every_arrangement_of_the_xcds_over_the_tile_grid(case):
    """The tile a workgroup takes depends on how the 8 XCDs are laid over the tile grid (8 x 1, 4 x 2, 2 x 4, 1 x 8, by
    the size of a panel of A; the third case has bands of unequal width and sliced tiles): every tile must still be computed exactly once.  All of C is compared with the FP32
    matrix-unit mode (different kernel, same arrangement rule but other panel sizes), sampled rows with the oracle."""
    import paper_2203_03341_amd as ec
    M, N, K, n = case
    assert ec.plan_info(M, N, K, ec.MODE_FP16_SPLIT)["column_bands"] == n
    _check("N", "N", M, N, K, 1.0, 0.0, "fp16", "urand", seed=9, rows=si.stratified_indices(M, 64, seed=4))
    A, B = _inputs(M, N, K, "N", "N", "urand", 9)
    got = _gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, "fp16")[:M, :N]
    other = _gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, "fp32")[:M, :N]
    assert np.max(np.abs(got - other)) < 1e-4 * np.sqrt(K / 3.0)     # entries are about sqrt(K / 3) large


def test_deep_k_in_one_item_keeps_fp32_accuracy():
    """693 tiles over a depth of 32279 with no slices: every element is one FP32 accumulator over 2018 matrix
    instructions.  The rounding of that accumulator is what is left of the error; it must stay under the naive FP32
    product's (measured: 0.35 of it)."""
    import paper_2203_03341_amd as ec
    M, N, K = 2235, 9758, 32279
    assert ec.plan_info(M, N, K, ec.MODE_FP16_SPLIT)["slices"] == 1
    for mode in ("fp16", "bf16"):
        r_gpu, r_cpu = _check("N", "N", M, N, K, 1.0, 0.0, mode, "urand", seed=29, pad=1, rows=si.stratified_indices(M, 64, seed=3))
        assert r_gpu < 0.6 * r_cpu


def test_column_bands_under_a_persistent_grid():
    """K <= 4096 runs as one workgroup per CU walking through its XCD's list; with BF16 panels of 24 MiB that list is
    laid out in two column bands."""
    import paper_2203_03341_amd as ec
    p = ec.plan_info(8192, 8192, 4096, ec.MODE_BF16_FULL)
    assert (p["persistent"], p["column_bands"]) == (1, 2)
    _check("N", "N", 8192, 8192, 4096, 1.0, 0.0, "bf16", "urand", seed=23, rows=si.stratified_indices(8192, 64, seed=9))
    A, B = _inputs(8192, 8192, 4096, "N", "N", "urand", 23)
    got = _gpu_sgemm("N", "N", 8192, 8192, 4096, 1.0, A, B, 0.0, None, "bf16")[:8192, :8192]
    other = _gpu_sgemm("N", "N", 8192, 8192, 4096, 1.0, A, B, 0.0, None, "fp16")[:8192, :8192]
    assert np.max(np.abs(got - other)) < 1e-4 * np.sqrt(4096 / 3.0)


@pytest.mark.parametrize("case", [("T", "N", 4321, 5700, 16500, "fp16", 4), ("N", "T", 6000, 3333, 9000, "bf16", 2)])
def test_column_bands_of_unequal_width_with_ragged_edges(case):
    """Sizes that are multiples of nothing: 17 x 45 and 24 x 27 tiles, bands of 12 + 11 + 11 + 11 and 14 + 13 tile
    columns, partial tiles on both edges, transposed operands with padded leading dimensions, alpha and beta."""
    import paper_2203_03341_amd as ec
    tA, tB, M, N, K, mode, bands = case
    assert ec.plan_info(M, N, K, ec.MODE_FP16_SPLIT if mode == "fp16" else ec.MODE_BF16_FULL)["column_bands"] == bands
    _check(tA, tB, M, N, K, 1.5, 0.5, mode, "urand", seed=13, pad=3, rows=si.stratified_indices(M, 64, seed=6))


@pytest.mark.parametrize("case", [(960, 2304, 18688, "fp16"), (512, 512, 16384, "bf16"), (3000, 3000, 1100, "fp16"),
                                  (640, 832, 9509, "bf16")])
def test_slice_counts_picked_by_the_cost_estimate(case):
    """Plans whose leftover tiles are cut into 3, 27, 2 and a dozen slices (whatever the estimate finds cheapest): the
    slices must cover the depth exactly once, ragged last slice included, and the fixed-order sum must give the same
    bits on every run."""
    import paper_2203_03341_amd as ec
    M, N, K, mode = case
    p = ec.plan_info(M, N, K, ec.MODE_FP16_SPLIT if mode == "fp16" else ec.MODE_BF16_FULL)
    assert p["slices"] > 1 and p["sliced_tiles"] > 0
    _check("N", "N", M, N, K, 1.0, 0.0, mode, "urand", seed=17, rows=si.stratified_indices(M, 64, seed=8))
    A, B = _inputs(M, N, K, "N", "N", "urand", 17)
    first = _gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, mode)
    again = _gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, mode)
    assert np.array_equal(first.view(np.uint32), again.view(np.uint32))


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_shapes_agree_bit_for_bit_when_nothing_is_sliced(mode):
    """Every shape adds up the k steps of an element in the same order; only slicing along K changes the bits."""
    M, N, K = 600, 500, 400
    A, B = _inputs(M, N, K, "N", "N", "urand", 6)
    outs = [_gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, mode, shape=sh) for sh in ("w4", "x2", "fused", "fused32", None)]
    for other in outs[1:]:
        assert np.array_equal(outs[0].view(np.uint32), other.view(np.uint32))


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
@pytest.mark.parametrize("fused", ["fused", "fused32"])
@pytest.mark.parametrize("transA,transB,pad", [("N", "N", 0), ("T", "T", 0), ("N", "T", 1), ("T", "N", 3), ("T", "N", 0)])
def test_one_launch_shape_splits_like_the_split_kernels(mode, transA, transB, pad, fused):
    """The one-launch shape splits in its own registers, with a short form for ordinary values and the split kernels'
    own arithmetic for the rest (values beyond the FP16 or BF16 range, which saturate; infinities; NaN), decided per
    wave and chunk of 64 k.  Whatever the mix, every bit of C equals what the split-first shape gives: operands with
    such values sprinkled over some rows and depths, every operand layout (transposes, aligned and unaligned leading
    dimensions), a depth that ends inside a chunk."""
    M, N, K = 150, 200, 300
    A, B = _inputs(M, N, K, transA, transB, "urand", 31, pad)
    opA, opB = gemm.logical(transA, A, M, K), gemm.logical(transB, B, K, N)   # views: writes go to A and B
    awkward = np.array([70000.0, -65520.0, 65519.0, 3.39e38, -3.4e38, np.inf, -np.inf, 1e-41, 65504.0, 1e30,
                        1e-6, -3e-8, 6.1e-5, 5.96e-8, -8.9e-8, 2.0 ** -14, 2.0 ** -126], dtype=np.float32)   # last row: FP16 subnormals
    rng = np.random.default_rng(5)
    for op, rows, cols in ((opA, M, K), (opB, K, N)):
        for v in awkward:
            for _ in range(3):
                op[rng.integers(rows), rng.integers(cols)] = v
    opA[7, 130] = np.nan
    outs = [_gpu_sgemm(transA, transB, M, N, K, 1.0, A, B, 0.0, None, mode, shape=sh)[:M, :N] for sh in ("x2", fused)]
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))
    assert np.all(np.isnan(outs[1][7, :])) and np.isfinite(outs[1]).sum() > M * N // 2
    # and with the handle's power-of-two pre-scaling, which is applied before the split
    import paper_2203_03341_amd as ec
    outs = []
    for sh in ("x2", fused):
        h = ec.Handle()
        h.set_scaling(3, -2)
        outs.append(_gpu_sgemm(transA, transB, M, N, K, 1.0, A, B, 0.0, None, mode, handle=h, shape=sh)[:M, :N])
        h.destroy()
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_one_launch_shape_with_leading_dimensions_beyond_32_bit_offsets(mode):
    """The loop that covers the bulk of the depth addresses a chunk's values with 32-bit offsets from the chunk's
    first value, which holds up to leading dimensions of 2^23; beyond, the kernel takes its general loop.  Operands
    with rows contiguous and a leading dimension of 2^23 + 4 (4.4 GB of zeros each, the matrix in the first rows of
    every column) must give the bits of the same operands stored compactly."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = 100, 70, 130
    ld = (1 << 23) + 4
    A, B = _inputs(M, N, K, "N", "T", "urand", 41)                      # op(A) = A (M x K), op(B) = B^T with B N x K: rows contiguous in both
    h = ec.Handle()
    h.set_shape(ec.SHAPE_64x64_FUSED)
    mode_id = _modes()[mode]
    outs = []
    for wide in (False, True):
        if wide:
            dA = torch.zeros((K, ld), dtype=torch.float32, device="cuda")
            dB = torch.zeros((K, ld), dtype=torch.float32, device="cuda")
            dA[:, :M] = to_device(A)[:, :M]
            dB[:, :N] = to_device(B)[:, :N]
            lda = ldb = ld
        else:
            dA, dB, lda, ldb = to_device(A), to_device(B), A.shape[0], B.shape[0]
        dC = empty_colmajor(M, N, fill=float("nan"))
        h.sgemm(ec.OP_N, ec.OP_T, M, N, K, 1.0, dA, lda, dB, ldb, 0.0, dC, M, mode_id)
        torch.cuda.synchronize()
        outs.append(to_host(dC, M, N))
        del dA, dB
    h.destroy()
    assert np.all(np.isfinite(outs[0]))
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
@pytest.mark.parametrize("transA,transB,size", [("N", "N", (128, 128, 4096)), ("T", "N", (300, 200, 5000)), ("N", "T", (33, 700, 3000)),
                                                 ("T", "T", (64, 64, 4101))])
def test_one_launch_plans_with_the_depth_in_slices(mode, transA, transB, size):
    """Deep products of few tiles run as one launch whose blocks take a slice of the depth each, plus the reduction
    kernel that adds the slices in ascending order.  The result must pass the accuracy rule against the oracle, and
    with alpha = 1, beta = 0 it must equal, bit for bit, the FP32 sum in the same order of the products of the slices
    computed one by one (each of them a one-launch call of its own)."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = size
    mode_id = _modes()[mode]
    p = ec.plan_info(M, N, K, mode_id)
    assert p["shape"] >= ec.SHAPE_64x64_FUSED and p["slices"] > 1 and p["sliced_tiles"] == p["tiles_m"] * p["tiles_n"]
    _check(transA, transB, M, N, K, 1.5, 0.5, mode, "urand", seed=51, pad=1)
    A, B = _inputs(M, N, K, transA, transB, "urand", 52)
    whole = _gpu_sgemm(transA, transB, M, N, K, 1.0, A, B, 0.0, None, mode)[:M, :N]
    chunks = -(-K // 64)
    per_slice = 64 * (-(-(-(-chunks // p["slices"])) // 8) * 8)      # equal shares of 64-deep chunks, rounded up to whole runs of 512
    opA, opB = gemm.logical(transA, A, M, K), gemm.logical(transB, B, K, N)
    total = None
    for k0 in range(0, K, per_slice):
        k1 = min(K, k0 + per_slice)
        a = np.asfortranarray(opA[:, k0:k1])                          # (these calls see both operands untransposed; the values and
        b = np.asfortranarray(opB[k0:k1, :])                          # their order along the depth are what the slice of the big call sees)
        # (a slice of 1024 or more is itself cut at multiples of 512 by its own call, across blocks; inside the big
        # call's block the same runs of 512 are added in registers, in the same order)
        assert ec.plan_info(M, N, k1 - k0, mode_id)["shape"] >= ec.SHAPE_64x64_FUSED
        part = _gpu_sgemm("N", "N", M, N, k1 - k0, 1.0, a, b, 0.0, None, mode)[:M, :N]
        total = part if total is None else (total + part).astype(np.float32)
    assert k1 == K and -(-K // per_slice) == p["slices"]
    assert np.array_equal(whole.view(np.uint32), total.view(np.uint32))


def test_one_launch_shapes_equal_the_split_first_shape_on_random_small_problems():
    """Random sizes up to 300 x 300 x 512 (one slice of depth in every shape), both transposes, padded leading
    dimensions of every alignment, alpha and beta, magnitudes over 16 binades, now and then a value beyond the FP16
    or BF16 range: the two one-launch shapes give the bits of the split-first shape."""
    import torch
    import paper_2203_03341_amd as ec
    rng = np.random.default_rng(123)
    h = ec.Handle()
    for trial in range(80):
        M, N, K = int(rng.integers(1, 300)), int(rng.integers(1, 300)), int(rng.integers(1, 513))
        if trial % 7 == 0:
            K = int(rng.choice([64, 128, 256, 512, 4, 8, 63, 65]))
        transA, transB = str(rng.choice(["N", "T"])), str(rng.choice(["N", "T"]))
        mode = _modes()[str(rng.choice(["fp16", "bf16"]))]
        pad_a, pad_b, pad_c = (int(rng.choice([0, 0, 1, 3, 4])) for _ in range(3))
        ar, ac = (M, K) if transA == "N" else (K, M)
        br, bc = (K, N) if transB == "N" else (N, K)
        A = si.urand(ar, ac, trial, si.ID_A, ld=ar + pad_a)
        A[:ar, :] *= np.float32(2.0 ** int(rng.integers(-8, 8)))
        B = si.urand(br, bc, trial, si.ID_B, ld=br + pad_b)
        if trial % 5 == 0:
            A[int(rng.integers(0, ar)), int(rng.integers(0, ac))] = np.float32(rng.choice([7e4, -1e30, 3.39e38, 1e-7]))
        C = si.urand(M, N, trial, si.ID_C, ld=M + pad_c)
        alpha, beta = float(rng.choice([1.0, 1.5, -0.25])), float(rng.choice([0.0, 0.5, 1.0]))
        dA, dB = to_device(A), to_device(B)
        ops = {"N": ec.OP_N, "T": ec.OP_T}
        outs = []
        for shape in (ec.SHAPE_128x128_X2, ec.SHAPE_64x64_FUSED, ec.SHAPE_32x32_FUSED):
            h.set_shape(shape)
            assert h.plan_info(M, N, K, mode)["slices"] == 1
            dC = to_device(C)
            h.sgemm(ops[transA], ops[transB], M, N, K, alpha, dA, A.shape[0], dB, B.shape[0], beta, dC, C.shape[0], mode)
            torch.cuda.synchronize()
            outs.append(to_host(dC, C.shape[0], N)[:M, :])
        case = (trial, M, N, K, transA, transB, mode, pad_a, pad_b, pad_c, alpha, beta)
        assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32)), case
        assert np.array_equal(outs[0].view(np.uint32), outs[2].view(np.uint32)), case
    h.destroy()


def test_the_tile_order_knob_moves_tiles_between_xcds_and_changes_no_bit():
    """ecgemm_debug_set_tile_order (the experiment knob behind the block-order profiles): hardware round-robin instead
    of contiguous runs per XCD, plain column-major order, forced column bands.  Where no tile is sliced along K the
    result is the same bit for bit; where the last tiles of the order are sliced, which tiles those are moves with the
    order, and the results agree to FP32 rounding."""
    import torch
    import paper_2203_03341_amd as ec
    for K, sliced in ((768, False), (1536, True)):
        M, N = 2048 + 256, 4096 + 128
        A, B = _inputs(M, N, K, "N", "T", "urand", 21)
        h = ec.Handle()
        ref = _gpu_sgemm("N", "T", M, N, K, 1.0, A, B, 0.0, None, "fp16", handle=h)
        assert (h.plan_info(M, N, K, ec.MODE_FP16_SPLIT)["sliced_tiles"] > 0) == sliced
        for order in [(0, 0, 0), (0, 1024, 1), (1, 1, 8), (1, 3, 5), (0, 2, 2)]:
            h.debug_set_tile_order(*order)
            info = h.plan_info(M, N, K, ec.MODE_FP16_SPLIT)
            assert (order[1] == 0 or info["group_m"] == order[1]) and (order[2] == 0 or info["column_bands"] == order[2])
            got = _gpu_sgemm("N", "T", M, N, K, 1.0, A, B, 0.0, None, "fp16", handle=h)
            if sliced:
                assert gemm.relative_residual(ref, got) < 2e-7, order
            else:
                assert np.array_equal(got, ref), order
        with pytest.raises(ec.EcgemmError) as err:
            h.debug_set_tile_order(2, 0, 0)
        assert err.value.argument == 2
        h.destroy()
    torch.cuda.synchronize()


def test_a_shape_the_mode_has_no_kernel_for_is_refused():
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    h.set_shape(ec.SHAPE_128x128_X2)
    A, B = _inputs(64, 64, 64, "N", "N", "urand", 0)
    dA, dB, dC = to_device(A), to_device(B), empty_colmajor(64, 64, fill=0.0)
    with pytest.raises(ec.EcgemmError) as err:
        h.sgemm(ec.OP_N, ec.OP_N, 64, 64, 64, 1.0, dA, 64, dB, 64, 0.0, dC, 64, ec.MODE_FP16_MARKIDIS)
    assert err.value.status == ec.ERR_UNSUPPORTED
    with pytest.raises(ec.EcgemmError):
        h.set_shape(7)
    h.set_shape(ec.SHAPE_AUTO)
    h.sgemm(ec.OP_N, ec.OP_N, 64, 64, 64, 1.0, dA, 64, dB, 64, 0.0, dC, 64, ec.MODE_FP16_MARKIDIS)
    # the fused shape has no use for operands split beforehand
    h.set_shape(ec.SHAPE_64x64_FUSED)
    packed = empty_colmajor(ec.split_size(64, 64, ec.MODE_FP16_SPLIT) // 4, 1, fill=0.0)
    with pytest.raises(ec.EcgemmError) as err:
        h.product(64, 64, 64, 1.0, packed, packed, 0.0, dC, 64, ec.MODE_FP16_SPLIT)
    assert err.value.status == ec.ERR_UNSUPPORTED
    # a problem whose 128 x 128 tiles can be counted in 32 bits may have too many tiles of a forced smaller shape
    big = (1 << 22, 1 << 21, 32)
    h.set_shape(ec.SHAPE_AUTO)
    assert h.plan_info(*big, ec.MODE_FP16_SPLIT)["tiles_m"] * h.plan_info(*big, ec.MODE_FP16_SPLIT)["tiles_n"] <= 1 << 30
    for small_tiles in (ec.SHAPE_64x64_FUSED, ec.SHAPE_32x32_FUSED):
        h.set_shape(small_tiles)
        with pytest.raises(ec.EcgemmError) as err:
            h.plan_info(*big, ec.MODE_FP16_SPLIT)
        assert err.value.status == ec.ERR_UNSUPPORTED and "tiles" in str(err.value)
        with pytest.raises(ec.EcgemmError):
            h.workspace_size(ec.OP_N, ec.OP_N, *big, ec.MODE_FP16_SPLIT)
        assert h.plan_info(1 << 20, 1 << 20, 32, ec.MODE_FP16_SPLIT)["grid"] == (1 << 40) // (64 * 64 if small_tiles == ec.SHAPE_64x64_FUSED else 32 * 32)
    h.destroy()


# ----- exponent ranges (section "Effect of the exponent range of input matrices")

def test_fp16_mode_limited_exponent_range():
    """Type 1 inputs, widened to the baseline's [-15, 15]: the top binade saturates at 65504 in the split."""
    _check("N", "N", 512, 512, 512, 1.0, 0.0, "fp16", ((-15, 15), (-15, 15)), seed=0)
    _check("N", "N", 512, 512, 512, 1.0, 0.0, "fp16", ((-15, 14), (-15, 14)), seed=1)


def test_bf16_mode_full_exponent_range():
    """Wide-range A times Type-1 B (finite in FP32), and both wide but bounded so products stay finite."""
    _check("N", "N", 512, 512, 512, 1.5, 0.5, "bf16", ((-100, 100), (-15, 14)), seed=0)
    _check("N", "N", 512, 512, 512, 1.0, 0.0, "bf16", ((-50, 50), (-50, 50)), seed=1)
    _check("N", "N", 384, 256, 640, 1.0, 0.0, "bf16", ((-100, -35), (-15, 14)), seed=2)


def test_fp16_mode_fails_outside_its_range_like_the_paper_says():
    """Type 4: inputs in exp_rand(-100, -35) are below anything halfhalf can hold; the result is (nearly)
    all zeros and the error is of order one, while the BF16 mode still meets the bar."""
    M = N = K = 256
    A, B = _inputs(M, N, K, "N", "N", ((-100, -35), (-15, 14)), 0)
    c64 = gemm.sgemm_fp64_ref("N", "N", M, N, K, 1.0, A, B)
    got = _gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, "fp16")[:M, :N]
    assert gemm.relative_residual(c64, got) > 0.1
    _check("N", "N", M, N, K, 1.0, 0.0, "bf16", ((-100, -35), (-15, 14)), seed=0)


# ----- the baseline's own sizes, in the launch configuration bench.py times; oracle on seeded sample rows of C

def _full_size(M, N, K, transA, transB, alpha, beta, mode, dist, nrows, seed=0):
    """The oracle on `nrows` rows of C, one out of every M / nrows consecutive rows (at most 64 apart in every test
    below), all columns: no output tile, and no wave's part of one, is left uncompared."""
    assert M / nrows <= 64
    rows = si.stratified_indices(M, -(-M // nrows), seed=11 + seed)
    return _check(transA, transB, M, N, K, alpha, beta, mode, dist, seed=seed, rows=rows)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_config2_4096_cubed(mode, seed):
    _full_size(4096, 4096, 4096, "N", "N", 1.0, 0.0, mode, "urand", 256, seed=seed)


@pytest.mark.timeout(400)          # the oracle's two products over 256 rows of 16384 x 16384 take most of a minute
def test_config3_16384_cubed_fp16_limited_exponent():
    _full_size(16384, 16384, 16384, "N", "N", 1.0, 0.0, "fp16", ((-15, 15), (-15, 15)), 256)


def test_config4_8192_cubed_bf16_wide_exponent():
    # the literal config (both operands exp_rand(-100, 100)) overflows FP32 everywhere; graded stand-in as in bench.py
    _full_size(8192, 8192, 8192, "N", "N", 1.5, 0.5, "bf16", ((-100, 100), (-15, 14)), 128)


def test_config4_literal_is_non_finite_for_everyone():
    """Both operands exp_rand(-100, 100): products reach 2^200, so the FP32 oracle and the GPU both overflow."""
    M = N = 256
    K = 8192
    A, B = _inputs(M, N, K, "N", "N", ((-100, 100), (-100, 100)), 0)
    c32 = gemm.sgemm_fp32_naive("N", "N", M, N, K, 1.0, A, B)
    got = _gpu_sgemm("N", "N", M, N, K, 1.0, A, B, 0.0, None, "bf16")[:M, :N]
    assert np.mean(~np.isfinite(c32)) > 0.99 and np.mean(~np.isfinite(got)) > 0.99


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_config5_full_shapes(mode):
    _full_size(16384, 16384, 256, "N", "N", 1.0, 0.0, mode, "urand", 256)
    _full_size(1024, 1024, 65536, "N", "N", 1.0, 0.0, mode, "urand", 64)
    _full_size(4095, 3001, 5003, "T", "N", 1.0, 0.0, mode, "urand", 256)


# ----- the comparison methods of the paper, run through the same kernels

@pytest.mark.parametrize("mode", ["markidis", "unscaled", "plain16", "plainbf"])
def test_comparison_methods_match_their_models(mode):
    """Element by element against the exact-accumulation model of each method (the pass rule does not apply:
    these methods are less accurate than FP32 by design)."""
    for (M, N, K, seed) in [(300, 200, 77, 1), (256, 256, 1024, 2)]:
        A, B = _inputs(M, N, K, "N", "T", "urand", seed, pad=1)
        got = _gpu_sgemm("N", "T", M, N, K, 1.0, A, B, 0.0, None, mode, ldc=M)[:M, :N]
        opA, opB = gemm.logical("N", A, M, K), gemm.logical("T", B, K, N)
        mag = np.abs(opA).astype(np.float64) @ np.abs(opB).astype(np.float64)
        slack = 2.0 if mode == "markidis" else 1.0     # one accumulator: the small products are aligned to the big sum
        assert np.all(np.abs(got - _model(mode, opA, opB)) <= slack * (K / 8 + 4) * 2.0 ** -23 * mag)


def test_fp32_on_the_matrix_unit_is_an_fp32_gemm():
    """ECGEMM_MODE_FP32_MFMA, the baseline of the comparison: no splitting, FP32 products and sums on the matrix unit.
    It must be as good as the naive FP32 loop (it adds two products per rounding), element by element within the FP32
    accumulation bound, and exact on small integers; the method's two modes must not be worse than it."""
    for (tA, tB, M, N, K, alpha, beta, pad) in [("N", "N", 300, 200, 77, 1.5, 0.5, 3), ("T", "T", 513, 259, 130, -1.0, 1.0, 1),
                                                ("N", "T", 700, 900, 1500, 1.0, 0.0, 0), ("T", "N", 1, 1, 1, 1.0, 0.0, 0)]:
        _check(tA, tB, M, N, K, alpha, beta, "fp32", "urand", seed=21, pad=pad, ratio_rule=K >= 64)
    rows = si.sample_indices(3000, 128, seed=3)
    r32, r_cpu = _check("N", "N", 3000, 3000, 1100, 1.0, 0.0, "fp32", "urand", seed=22, rows=rows)
    r16, _ = _check("N", "N", 3000, 3000, 1100, 1.0, 0.0, "fp16", "urand", seed=22, rows=rows)
    assert r16 <= 1.25 * r32 and r32 <= 1.25 * r_cpu


def test_error_ordering_of_the_papers_first_figure():
    """A 16 x k, B k x 16, uniform(-1, 1), k = 4096: plain FP16 is orders of magnitude worse than everything
    else, Markidis' method sits in between, the method matches FP32."""
    k = 4096
    res = {m: [] for m in ("plain16", "markidis", "unscaled", "fp16", "bf16", "fp32")}
    for seed in range(4):
        A, B = _inputs(16, 16, k, "N", "N", "urand", seed)
        c64 = gemm.sgemm_fp64_ref("N", "N", 16, 16, k, 1.0, A, B)
        res["fp32"].append(gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", 16, 16, k, 1.0, A, B)))
        for m in ("plain16", "markidis", "unscaled", "fp16", "bf16"):
            res[m].append(gemm.relative_residual(c64, _gpu_sgemm("N", "N", 16, 16, k, 1.0, A, B, 0.0, None, m)[:16, :16]))
    mean = {m: float(np.mean(v)) for m, v in res.items()}
    assert mean["plain16"] > 100 * mean["fp32"]
    assert mean["fp16"] <= 1.25 * mean["fp32"] and mean["bf16"] <= 1.25 * mean["fp32"]
    assert mean["markidis"] >= mean["fp16"]


@pytest.mark.parametrize("mode", ["fp16", "bf16", "markidis"])
def test_product_on_presplit_operands_equals_sgemm(mode):
    """ecgemm_split + ecgemm_product is bitwise ecgemm_sgemm, for both storage orders of B and with split-K."""
    import torch
    import paper_2203_03341_amd as ec
    m = _modes()[mode]
    h = ec.Handle()
    for (M, N, K, transA, transB) in [(300, 200, 77, "N", "N"), (513, 130, 4096, "T", "T")]:
        A, B = _inputs(M, N, K, transA, transB, "urand", 3, pad=2)
        C = si.urand(M, N, 3, si.ID_C)
        want = _gpu_sgemm(transA, transB, M, N, K, 1.5, A, B, 0.5, C, mode, handle=h)
        dA, dB, dC = to_device(A), to_device(B), to_device(C)
        pa = torch.empty(ec.split_size(M, K, m), dtype=torch.uint8, device="cuda")
        pb = torch.empty(ec.split_size(N, K, m), dtype=torch.uint8, device="cuda")
        h.split(ec.OP_N if transA == "N" else ec.OP_T, M, K, dA, A.shape[0], m, pa)
        h.split(ec.OP_T if transB == "N" else ec.OP_N, N, K, dB, B.shape[0], m, pb)
        h.product(M, N, K, 1.5, pa, pb, 0.5, dC, M, m)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(dC, M, N).view(np.uint32), want.view(np.uint32))
    h.destroy()


def test_prescaling_brings_small_inputs_into_the_fp16_window():
    """Type 3 of the paper (both inputs exp_rand(-35, -15)) loses accuracy in FP16 mode; the paper's remedy is a
    scaling before the product.  With exact power-of-two factors chosen from the measured exponent range the FP16
    mode meets the FP32 bar again, and the factors are undone exactly in the epilogue."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = 384, 320, 512
    A, B = _inputs(M, N, K, "N", "N", ((-35, -15), (-35, -15)), 0)
    C = si.urand(M, N, 0, si.ID_C)
    C *= np.float32(2.0 ** -40)                                  # same scale as the product, so beta matters
    c64 = gemm.sgemm_fp64_ref("N", "N", M, N, K, 1.5, A, B, 0.5, C)
    r_cpu = gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", M, N, K, 1.5, A, B, 0.5, C))
    h = ec.Handle()
    dA, dB = to_device(A), to_device(B)
    assert h.exponent_range(M, K, dA, M) == (-35, -15)
    assert h.exponent_range(K, N, dB, K) == (-35, -15)
    assert h.exponent_range(0, 0, None, 1) == (2 ** 31 - 1, -2 ** 31)
    plain = _gpu_sgemm("N", "N", M, N, K, 1.5, A, B, 0.5, C, "fp16", handle=h)[:M, :N]
    assert gemm.relative_residual(c64, plain) > 2 * r_cpu         # degraded, as the paper reports
    shift = 14 - (-15)                                            # top binade of the inputs lands on 2^14
    h.set_scaling(shift, shift)
    scaled = _gpu_sgemm("N", "N", M, N, K, 1.5, A, B, 0.5, C, "fp16", handle=h)[:M, :N]
    assert gemm.relative_residual(c64, scaled) <= RATIO * r_cpu
    h.set_shape(ec.SHAPE_64x64_FUSED)                            # the one-kernel path scales in its own split
    fused = _gpu_sgemm("N", "N", M, N, K, 1.5, A, B, 0.5, C, "fp16", handle=h)[:M, :N]
    assert np.array_equal(fused.view(np.uint32), scaled.view(np.uint32))
    h.set_shape(ec.SHAPE_AUTO)
    h.set_scaling(0, 0)
    again = _gpu_sgemm("N", "N", M, N, K, 1.5, A, B, 0.5, C, "fp16", handle=h)[:M, :N]
    assert np.array_equal(again.view(np.uint32), plain.view(np.uint32))
    with pytest.raises(ec.EcgemmError):
        h.set_scaling(100, 100)
    h.destroy()


@pytest.mark.parametrize("transA,transB", [("N", "N"), ("T", "T")])
def test_row_and_column_scaling_for_rows_of_different_magnitude(transA, transB):
    """Rows of op(A) and columns of op(B) spread over 2^-60 .. 2^20: no single factor brings them all into the FP16
    window, one power of two per row / column does.  The exponents come from the library (bit for bit what numpy
    computes), the scaling is exact, and the FP16 mode meets the FP32 bar again."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = 520, 390, 1100           # several tiles, ragged; K deep enough that the tiles are sliced along K
    rng = np.random.default_rng(11)
    ea = rng.integers(-60, 21, size=M)
    eb = rng.integers(-60, 21, size=N)
    opA = np.ldexp(si.urand(M, K, 3, si.ID_A)[:M, :K], ea[:, None]).astype(np.float32)
    opB = np.ldexp(si.urand(K, N, 3, si.ID_B)[:K, :N], eb[None, :]).astype(np.float32)
    opA[7, :] = 0.0                    # a row without a non-zero element gets the exponent 0
    A = np.asfortranarray(opA if transA == "N" else opA.T)
    B = np.asfortranarray(opB if transB == "N" else opB.T)
    C = si.urand(M, N, 3, si.ID_C)[:M, :N].copy(order="F")
    C *= np.float32(2.0 ** -20)
    c64 = gemm.sgemm_fp64_ref(transA, transB, M, N, K, 1.5, A, B, 0.5, C)
    c32 = gemm.sgemm_fp32_naive(transA, transB, M, N, K, 1.5, A, B, 0.5, C)
    ops = {"N": ec.OP_N, "T": ec.OP_T}
    h = ec.Handle()
    dA, dB = to_device(A), to_device(B)
    sa = torch.full((M,), 12345, dtype=torch.int32, device="cuda")
    sb = torch.full((N,), 12345, dtype=torch.int32, device="cuda")
    h.row_scales(ops[transA], M, K, dA, A.shape[0], 14, sa)
    h.row_scales(ec.OP_T if transB == "N" else ec.OP_N, N, K, dB, B.shape[0], 14, sb)
    torch.cuda.synchronize()

    def expected(rows):
        amax = np.max(np.abs(rows), axis=1)
        return np.where(amax > 0, 14 - (np.frexp(amax)[1] - 1), 0)       # frexp: amax = f * 2^e with f in [0.5, 1)

    assert np.array_equal(sa.cpu().numpy(), expected(opA))
    assert np.array_equal(sb.cpu().numpy(), expected(opB.T))

    def run(scaled):
        dC = to_device(C)
        if scaled:
            h.sgemm_scaled(ops[transA], ops[transB], M, N, K, 1.5, dA, A.shape[0], dB, B.shape[0], 0.5, dC, M,
                           ec.MODE_FP16_SPLIT, sa, sb)
        else:
            h.sgemm(ops[transA], ops[transB], M, N, K, 1.5, dA, A.shape[0], dB, B.shape[0], 0.5, dC, M, ec.MODE_FP16_SPLIT)
        torch.cuda.synchronize()
        return to_host(dC, M, N)

    # the residual norm is dominated by the largest rows and columns; what the scaling saves are the small ones, so
    # the check runs row by row: relative residual of every row of C against the FP32 product's
    def row_residuals(x):
        return np.linalg.norm((c64 - x).astype(np.float64), axis=1) / np.maximum(np.linalg.norm(c64, axis=1), 1e-300)

    r_cpu = row_residuals(c32)
    plain = row_residuals(run(False))
    scaled = run(True)
    assert np.all(np.isfinite(scaled))
    r_gpu = row_residuals(scaled)
    live = np.linalg.norm(c64, axis=1) > 0
    with np.errstate(invalid="ignore", divide="ignore"):
        lost = ~np.isfinite(plain) | (plain > 10 * r_cpu)
    assert np.mean(lost[live]) > 0.5                                 # most rows are lost without the scaling
    assert gemm.relative_residual(c64, scaled) <= RATIO * gemm.relative_residual(c64, c32)
    # Row by row: every single row is as good as FP32's (within a factor of two), whichever shape runs it.  The
    # library takes a one-launch shape for this size by itself; that kernel scales in its own split and adds the depth
    # up in slices of 512, as the split-first shapes slice this depth in two, because the error of the matrix unit's
    # accumulation grows with the length of the sum (the paper's section "Avoiding RZ during Tensor Core
    # accumulation"; with one accumulator over all 69 k steps one row of 520 came out at 3.0 times FP32's).
    # Where nothing is sliced every shape gives the same bits.
    assert np.all(r_gpu[live] <= 2.0 * r_cpu[live] + 1e-12)
    for shape in (ec.SHAPE_128x128_X2, ec.SHAPE_256x128_W4, ec.SHAPE_64x64_FUSED, ec.SHAPE_32x32_FUSED):
        h.set_shape(shape)
        forced = run(True)
        assert np.all(np.isfinite(forced)) and np.all(row_residuals(forced)[live] <= 2.0 * r_cpu[live] + 1e-12)
        assert gemm.relative_residual(c64, forced) <= RATIO * gemm.relative_residual(c64, c32)
    shallow = 96                                                      # too shallow for any shape to slice
    outs = []
    for shape in (ec.SHAPE_64x64_FUSED, ec.SHAPE_128x128_X2, ec.SHAPE_256x128_W4, ec.SHAPE_32x32_FUSED):
        h.set_shape(shape)
        assert h.plan_info(M, N, shallow, ec.MODE_FP16_SPLIT)["slices"] == 1
        dC = to_device(C)
        h.sgemm_scaled(ops[transA], ops[transB], M, N, shallow, 1.5, dA, A.shape[0], dB, B.shape[0], 0.5, dC, M,
                       ec.MODE_FP16_SPLIT, sa, sb)
        torch.cuda.synchronize()
        outs.append(to_host(dC, M, N))
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))
    assert np.array_equal(outs[1].view(np.uint32), outs[2].view(np.uint32))
    assert np.array_equal(outs[2].view(np.uint32), outs[3].view(np.uint32))
    h.set_shape(ec.SHAPE_AUTO)
    with pytest.raises(ec.EcgemmError):                              # one vector without the other
        h.sgemm_scaled(ops[transA], ops[transB], M, N, K, 1.0, dA, A.shape[0], dB, B.shape[0], 0.0, to_device(C), M,
                       ec.MODE_FP16_SPLIT, sa, None)
    h.destroy()


@pytest.mark.parametrize("shape", [None, "x2", "fused", "fused32"])
def test_scaling_exponents_that_only_cancel_together(shape):
    """Rows of op(A) near 2^120 and columns of op(B) near 2^-125: the product is an ordinary number, but either scaling
    exponent alone (-106, +126) would push the scaled product out of the FP32 range before the other brings it back.
    The two are undone as one sum."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = 200, 260, 96
    opA = np.ldexp(si.urand(M, K, 5, si.ID_A)[:M, :K], 120).astype(np.float32)
    opB = np.ldexp(si.urand(K, N, 5, si.ID_B)[:K, :N], -125).astype(np.float32)
    A, B = np.asfortranarray(opA), np.asfortranarray(opB)
    h = ec.Handle()
    h.set_shape(_shapes()[shape])
    dA, dB = to_device(A), to_device(B)
    sa = torch.empty(M, dtype=torch.int32, device="cuda")
    sb = torch.empty(N, dtype=torch.int32, device="cuda")
    h.row_scales(ec.OP_N, M, K, dA, M, 14, sa)
    h.row_scales(ec.OP_T, N, K, dB, K, 14, sb)
    dC = empty_colmajor(M, N, fill=float("nan"))
    h.sgemm_scaled(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, ec.MODE_FP16_SPLIT, sa, sb)
    torch.cuda.synchronize()
    got = to_host(dC, M, N)
    assert sa.cpu().numpy().min() <= -105 and sb.cpu().numpy().max() >= 125
    c64 = gemm.sgemm_fp64_ref("N", "N", M, N, K, 1.0, A, B)
    c32 = gemm.sgemm_fp32_naive("N", "N", M, N, K, 1.0, A, B)
    assert np.all(np.isfinite(got)) and gemm.relative_residual(c64, got) <= RATIO * gemm.relative_residual(c64, c32)
    h.destroy()


@pytest.mark.parametrize("mode", ["outside", "outside4", "outside16"])
def test_accumulating_outside_the_matrix_unit_as_the_paper_does(mode):
    """The paper's listing verbatim (zeroed temporary, FP32 vector adds every k step), and the same with the matrix unit
    left to sum 4 or 16 k steps by itself before its sum joins the one kept outside: each meets the same bar as the
    default FP16 mode; one FP32 rounding per 16 products or more instead of per 8, so the element-wise bound holds too."""
    _check("N", "N", 300, 200, 77, 1.5, 0.5, mode, "urand", seed=1, pad=3)
    _check("T", "N", 512, 384, 4096, 1.0, 0.0, mode, "urand", seed=2)
    _check("N", "T", 640, 130, 16 * 37, 1.0, 0.0, mode, "urand", seed=4)      # a depth that ends in the middle of an interval
    rows = si.sample_indices(4096, 128, seed=3)
    r_out, r_cpu = _check("N", "N", 4096, 4096, 4096, 1.0, 0.0, mode, "urand", seed=0, rows=rows)
    r_def, _ = _check("N", "N", 4096, 4096, 4096, 1.0, 0.0, "fp16", "urand", seed=0, rows=rows)
    assert r_out < r_cpu and r_def < r_cpu          # neither needs the detour to beat the FP32 sum here


def test_choose_mode_follows_the_papers_types():
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    n = 256

    def choose(ra, rb):
        A, B = _inputs(n, n, n, "N", "T", (ra, rb), 0)
        return h.choose_mode(ec.OP_N, ec.OP_T, n, n, n, to_device(A), n, to_device(B), n)

    assert choose((-15, 13), (-15, 13)) == (ec.MODE_FP16_SPLIT, 1, 1)            # Type 1: fits as it is
    assert choose((-35, -15), (-35, -15)) == (ec.MODE_FP16_SPLIT, 29, 29)        # Type 3: fits after scaling
    assert choose((-15, 14), (-100, -35))[0] == ec.MODE_BF16_FULL                 # Type 2: one operand spans 66 binades
    assert choose((-100, 100), (-15, 14))[0] == ec.MODE_BF16_FULL
    # the recommendation meets the bar when followed
    A, B = _inputs(n, n, n, "N", "T", ((-60, -40), (5, 30)), 1)
    mode, sa, sb = h.choose_mode(ec.OP_N, ec.OP_T, n, n, n, to_device(A), n, to_device(B), n)
    assert (mode, sa, sb) == (ec.MODE_FP16_SPLIT, 54, -16)
    h.set_scaling(sa, sb)
    got = _gpu_sgemm("N", "T", n, n, n, 1.0, A, B, 0.0, None, "fp16", handle=h)[:n, :n]
    c64 = gemm.sgemm_fp64_ref("N", "T", n, n, n, 1.0, A, B)
    assert gemm.relative_residual(c64, got) <= RATIO * gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "T", n, n, n, 1.0, A, B))
    h.destroy()


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_operand_with_more_than_2_pow_31_elements(mode):
    """A is 70000 x 32768 (2.3e9 elements, 8.5 GiB; its packed form crosses 4 GiB byte offsets as well): catches
    32-bit index arithmetic anywhere on the path.  A is drawn on the device from torch's seeded generator (moving
    8.5 GiB through numpy would take minutes); the oracle gets the sampled rows of that same A."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = 70000, 192, 32768
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)
    dA = torch.empty((K, M), dtype=torch.float32, device="cuda")          # column-major M x K, lda = M
    dA.uniform_(-1.0, 1.0, generator=gen)
    B = si.urand(K, N, 7, si.ID_B)
    dB = to_device(B)
    dC = empty_colmajor(M, N, fill=float("nan"))
    h = ec.Handle()
    h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, _modes()[mode])
    torch.cuda.synchronize()
    rows = np.concatenate([si.sample_indices(M, 40, seed=5), np.array([0, 65535, 65536, M - 1])])
    A_rows = np.asfortranarray(dA[:, torch.from_numpy(rows).cuda()].T.contiguous().cpu().numpy())   # len(rows) x K
    got = dC[:, torch.from_numpy(rows).cuda()].T.contiguous().cpu().numpy()                         # len(rows) x N
    h.destroy()
    del dA
    torch.cuda.empty_cache()
    c64 = gemm.sgemm_fp64_ref("N", "N", len(rows), N, K, 1.0, A_rows, B)
    c32 = gemm.sgemm_fp32_naive("N", "N", len(rows), N, K, 1.0, A_rows, B)
    assert np.all(np.isfinite(got))
    assert gemm.relative_residual(c64, got) <= RATIO * gemm.relative_residual(c64, c32)
    mdl = _model(mode, A_rows, gemm.logical("N", B, K, N))
    mag = np.abs(A_rows).astype(np.float64) @ np.abs(B[:K, :N]).astype(np.float64)
    assert np.all(np.abs(got - mdl) <= (K / 8 + 4) * 2.0 ** -23 * mag)


def test_sizes_beyond_the_supported_depth_are_refused():
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    dummy = empty_colmajor(8, 8, fill=0.0)
    with pytest.raises(ec.EcgemmError) as ei:       # nothing is read or allocated before the check
        h.sgemm(ec.OP_T, ec.OP_N, 4, 4, 1 << 26, 1.0, dummy, 1 << 26, dummy, 1 << 26, 0.0, dummy, 4, ec.MODE_FP16_SPLIT)
    assert ei.value.status == ec.ERR_INVALID_ARG
    with pytest.raises(ec.EcgemmError) as ei:       # more output tiles than a 32-bit item count holds
        h.sgemm(ec.OP_N, ec.OP_N, 1 << 23, 1 << 23, 1, 1.0, dummy, 1 << 23, dummy, 1, 0.0, dummy, 1 << 23, ec.MODE_FP16_SPLIT)
    assert ei.value.status == ec.ERR_INVALID_ARG
    h.destroy()
