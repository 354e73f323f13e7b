"""ECGEMM_MODE_AUTO through the C-ABI: the choice against the oracle's criterion, the result against the chosen arrangement.

The choice (FP16 mode, FP16 mode on row / column scaled operands, BF16 mode) is an integer decided by floating
point: both sides sum the same FP64 terms (|x|^2 and the squared part the FP16 pair loses), in different orders,
and compare against 2^-24.  The test inputs sit well away from that threshold (2^-24.6 or below on the passing side,
2^-20.4 or above on the other), so the order cannot decide.  What the call returns must be, bit for bit, what the
chosen arrangement returns when called directly: ecgemm_sgemm in that mode, or ecgemm_row_scales (target 14) followed
by ecgemm_sgemm_scaled in FP16 mode.
"""
import numpy as np
import pytest

import seeded_inputs as si
from oracle import gemm, model, split
from gpu_util import empty_colmajor, to_device, to_host

pytestmark = pytest.mark.gpu

TYPE1, TYPE3, TYPE4 = (-15, 14), (-35, -15), (-100, -35)       # exp_rand ranges of the paper's input types


def _draw(rows, cols, dist, seed, matrix_id, pad):
    if dist == "urand":
        return si.urand(rows, cols, seed, matrix_id, ld=rows + pad)
    return si.exp_rand(rows, cols, dist[0], dist[1], seed, matrix_id, ld=rows + pad)


def _problem(transA, transB, M, N, K, dist_a, dist_b, seed, pad):
    ar, ac = (M, K) if transA == "N" else (K, M)
    br, bc = (K, N) if transB == "N" else (N, K)
    return _draw(ar, ac, dist_a, seed, si.ID_A, pad), _draw(br, bc, dist_b, seed, si.ID_B, pad), si.urand(M, N, seed, si.ID_C)


def _run(h, call, transA, transB, M, N, K, alpha, A, B, beta, C, mode):
    import torch
    import paper_2203_03341_amd as ec
    ops = {"N": ec.OP_N, "T": ec.OP_T}
    dA, dB, dC = to_device(A), to_device(B), to_device(C)
    call(ops[transA], ops[transB], M, N, K, alpha, dA, A.shape[0], dB, B.shape[0], beta, dC, C.shape[0], mode)
    torch.cuda.synchronize()
    return to_host(dC, C.shape[0], N)


def _run_scaled(h, transA, transB, M, N, K, alpha, A, B, beta, C):
    """ecgemm_row_scales (target 14) for both operands, then ecgemm_sgemm_scaled in FP16 mode; also the exponents."""
    import torch
    import paper_2203_03341_amd as ec
    ops = {"N": ec.OP_N, "T": ec.OP_T}
    dA, dB, dC = to_device(A), to_device(B), to_device(C)
    sa = torch.empty(M, dtype=torch.int32, device="cuda")
    sb = torch.empty(N, dtype=torch.int32, device="cuda")
    h.row_scales(ops[transA], M, K, dA, A.shape[0], 14, sa)
    h.row_scales(ec.OP_T if transB == "N" else ec.OP_N, N, K, dB, B.shape[0], 14, sb)
    h.sgemm_scaled(ops[transA], ops[transB], M, N, K, alpha, dA, A.shape[0], dB, B.shape[0], beta, dC, C.shape[0],
                   ec.MODE_FP16_SPLIT, sa, sb)
    torch.cuda.synchronize()
    return to_host(dC, C.shape[0], N), sa.cpu().numpy(), sb.cpu().numpy()


def _check(h, transA, transB, M, N, K, dist_a, dist_b, seed=0, pad=0, alpha=1.5, beta=0.5, noalloc=False):
    import paper_2203_03341_amd as ec
    A, B, C = _problem(transA, transB, M, N, K, dist_a, dist_b, seed, pad)
    opA, opB = gemm.logical(transA, A, M, K), gemm.logical(transB, B, K, N)
    want = split.automatic_choice(opA, opB)
    got = _run(h, h.sgemm_noalloc if noalloc else h.sgemm, transA, transB, M, N, K, alpha, A, B, beta, C, ec.MODE_AUTO)
    chosen = h.auto_choice()
    assert chosen == {"fp16": (ec.MODE_FP16_SPLIT, False), "fp16 scaled": (ec.MODE_FP16_SPLIT, True),
                      "bf16": (ec.MODE_BF16_FULL, False)}[want], (dist_a, dist_b, want, chosen)
    if want == "fp16 scaled":
        direct, sa, sb = _run_scaled(h, transA, transB, M, N, K, alpha, A, B, beta, C)
        assert np.array_equal(sa, split.row_scale_exponents(opA)) and np.array_equal(sb, split.row_scale_exponents(opB.T))
    else:
        direct = _run(h, h.sgemm, transA, transB, M, N, K, alpha, A, B, beta, C, chosen[0])
    assert np.array_equal(got.view(np.uint32), direct.view(np.uint32))
    # and the point of choosing: the result meets the accuracy bar of the method whatever the inputs
    c64 = gemm.sgemm_fp64_ref(transA, transB, M, N, K, alpha, A, B, beta, C)
    c32 = gemm.sgemm_fp32_naive(transA, transB, M, N, K, alpha, A, B, beta, C)
    assert gemm.relative_residual(c64, got[:M, :]) <= 1.25 * gemm.relative_residual(c64, c32)
    # element by element against the exact-accumulation model of the chosen arrangement: the GPU differs from it only
    # by its FP32 accumulation (one rounding per eight products) and the rounding of alpha c + beta C
    if want == "fp16 scaled":
        ea, eb = split.row_scale_exponents(opA), split.row_scale_exponents(opB.T)
        sA, sB = split.scale_rows(opA, ea), split.scale_rows(opB.T, eb).T.copy()
        undo = lambda x: np.ldexp(np.ldexp(x, -ea[:, None].astype(np.int32)), -eb[None, :].astype(np.int32))
        mdl = undo(model.gemm_fp16_mode(sA, sB))
        mag = undo(np.abs(sA).astype(np.float64) @ np.abs(sB).astype(np.float64))
    else:
        mdl = model.gemm_fp16_mode(opA, opB) if want == "fp16" else model.gemm_bf16_mode(opA, opB)
        mag = np.abs(opA).astype(np.float64) @ np.abs(opB).astype(np.float64)
    cin = C[:M, :N].astype(np.float64)
    expect = alpha * mdl + beta * cin
    bound = (K / 8 + 4) * 2.0 ** -23 * abs(alpha) * mag + 2.0 ** -22 * (np.abs(expect) + np.abs(beta * cin))
    assert np.max(np.abs(got[:M, :] - expect) / (bound + 1e-300)) <= 1.0, (want, dist_a, dist_b)
    return want


@pytest.mark.parametrize("transA,transB,pad", [("N", "N", 0), ("T", "T", 0), ("N", "T", 1), ("T", "N", 3)])
def test_choice_and_result_for_the_papers_input_types(transA, transB, pad):
    """Every split kernel variant (both storage orders, aligned and not) measures the same thing; ragged sizes with
    several blocks per operand; either operand alone takes the call out of the plain FP16 mode."""
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    M, N, K = 300, 260, 200
    chosen = [
        _check(h, transA, transB, M, N, K, "urand", "urand", seed=1, pad=pad),
        _check(h, transA, transB, M, N, K, TYPE1, TYPE1, seed=2, pad=pad),
        _check(h, transA, transB, M, N, K, TYPE3, TYPE3, seed=3, pad=pad),
        _check(h, transA, transB, M, N, K, TYPE4, TYPE1, seed=4, pad=pad),
        _check(h, transA, transB, M, N, K, TYPE1, TYPE3, seed=5, pad=pad),
    ]
    assert chosen == ["fp16", "fp16", "fp16 scaled", "fp16 scaled", "fp16 scaled"]
    h.destroy()


def test_each_candidate_runs_as_its_fixed_mode_would():
    """Sizes that a fixed mode runs as one launch on the FP32 operands (256^3), with the split-first kernels (1536^3),
    and 768 x 1280 x 3584, where the FP16 mode takes one launch and the BF16 mode splits first: whichever candidate
    wins runs that way, so that the bits are the fixed mode's.  (The checks are those of every other case here: the
    oracle's choice, bit equality with the direct call, the accuracy bar.)"""
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    one_launch = lambda size, mode: h.plan_info(*size, mode)["shape"] >= ec.SHAPE_64x64_FUSED
    small, mixed, large = (256, 256, 256), (768, 1280, 3584), (1536, 1536, 1536)
    assert one_launch(small, ec.MODE_FP16_SPLIT) and one_launch(small, ec.MODE_BF16_FULL)
    assert one_launch(mixed, ec.MODE_FP16_SPLIT) and not one_launch(mixed, ec.MODE_BF16_FULL)
    assert not one_launch(large, ec.MODE_FP16_SPLIT) and not one_launch(large, ec.MODE_BF16_FULL)
    chosen = []
    for (m, n, k) in (small, mixed, large):
        chosen.append(_check(h, "N", "N", m, n, k, "urand", "urand", seed=21))       # plain FP16
        chosen.append(_check(h, "N", "N", m, n, k, TYPE3, TYPE3, seed=22))           # FP16 on scaled operands
    assert chosen == ["fp16", "fp16 scaled"] * 3
    # the BF16 candidate: rows too short for the pair to match an FP32 sum (K = 8), at a size of one launch and at
    # 1024 x 1024 x 8, and then a shape whose BF16 plan splits first
    chosen = [_check(h, "N", "T", 256, 256, 8, TYPE3, TYPE3, seed=23), _check(h, "T", "N", 2500, 2500, 8, TYPE3, TYPE3, seed=24)]
    assert chosen == ["bf16"] * 2
    assert h.plan_info(256, 256, 8, ec.MODE_BF16_FULL)["shape"] >= ec.SHAPE_64x64_FUSED and h.plan_info(2500, 2500, 8, ec.MODE_BF16_FULL)["shape"] < ec.SHAPE_64x64_FUSED
    h.destroy()


def test_sliced_tiles_large_operands_and_the_builtin_workspace():
    """Deep K (tiles sliced along K, gated reduction kernels), operands of more than 8192 split blocks (one launch per
    operand instead of the pair launch), and the entry point that allocates nothing."""
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    wide = (-100, 100)          # an operand spread over the FP32 exponent range (the other stays moderate, or C overflows)
    for dist_a, dist_b in (("urand", "urand"), (TYPE3, TYPE3), (wide, TYPE1)):
        _check(h, "N", "N", 512, 384, 4608, dist_a, dist_b, seed=6)
        _check(h, "T", "N", 1100, 900, 1300, dist_a, dist_b, seed=7, pad=1, noalloc=True)
        _check(h, "N", "T", 2304, 2048, 2080, dist_a, dist_b, seed=8, alpha=1.0, beta=0.0)
    h.destroy()


def test_tiny_and_degenerate_shapes():
    """One element, one row, one column, depths that end inside the first block: the choice and the bits still equal
    the oracle's choice and the direct calls' bits."""
    import torch
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    for (M, N, K) in [(1, 1, 1), (2, 3, 5), (17, 5, 8), (31, 33, 15), (64, 1, 100), (1, 257, 33)]:
        for dist in ("urand", TYPE4):
            A, B, C = _problem("N", "T", M, N, K, dist, dist, M + N + K, 2)
            opA, opB = gemm.logical("N", A, M, K), gemm.logical("T", B, K, N)
            want = split.automatic_choice(opA, opB)
            got = _run(h, h.sgemm, "N", "T", M, N, K, 1.0, A, B, 0.0, C, ec.MODE_AUTO)
            chosen = h.auto_choice()
            assert chosen == {"fp16": (ec.MODE_FP16_SPLIT, False), "fp16 scaled": (ec.MODE_FP16_SPLIT, True),
                              "bf16": (ec.MODE_BF16_FULL, False)}[want], (M, N, K, dist, want, chosen)
            if want == "fp16 scaled":
                direct, _, _ = _run_scaled(h, "N", "T", M, N, K, 1.0, A, B, 0.0, C)
            else:
                direct = _run(h, h.sgemm, "N", "T", M, N, K, 1.0, A, B, 0.0, C, chosen[0])
            assert np.array_equal(got.view(np.uint32), direct.view(np.uint32)), (M, N, K, dist)
    h.destroy()


def test_special_values_and_prescaling():
    import torch
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    M, N, K = 200, 150, 512
    A, B, C = _problem("N", "N", M, N, K, "urand", "urand", 9, 0)
    ops = (ec.OP_N, ec.OP_N)
    FP16, SCALED, BF16 = (ec.MODE_FP16_SPLIT, False), (ec.MODE_FP16_SPLIT, True), (ec.MODE_BF16_FULL, False)

    def choice_for(A_host, B_host):
        dA, dB, dC = to_device(A_host), to_device(B_host), to_device(C)
        h.sgemm(*ops, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, ec.MODE_AUTO)
        return h.auto_choice(), to_host(dC, M, N)

    assert choice_for(A, B)[0] == FP16
    # a NaN or an infinity leaves only the full-range mode; a finite value beyond the FP16 range is an ordinary row
    # maximum once its row is scaled
    for poison, want in ((np.nan, BF16), (np.inf, BF16), (np.float32(1e6), SCALED)):
        bad = A.copy(order="F")
        bad[17, 5] = poison
        assert choice_for(bad, B)[0] == want, poison
        assert choice_for(A, B)[0] == FP16                    # (and the previous call's choice does not stick)
    zeros = np.zeros_like(A)
    mode, out = choice_for(zeros, B)                          # nothing to lose in an all-zero operand
    assert mode == FP16 and np.all(out == 0.0)
    # the handle's pre-scaling moves Type 3 inputs into the window of the pair: the choice is made after it
    A3, B3, _ = _problem("N", "N", M, N, K, TYPE3, TYPE3, 10, 0)
    assert choice_for(A3, B3)[0] == SCALED
    h.set_scaling(29, 29)
    mode, scaled = choice_for(A3, B3)
    assert mode == FP16
    direct = _run(h, h.sgemm, "N", "N", M, N, K, 1.0, A3, B3, 0.0, C, ec.MODE_FP16_SPLIT)
    assert np.array_equal(scaled.view(np.uint32), direct.view(np.uint32))
    # a global factor that does not help (Type 4 stays out of reach of one factor of 2^29): the scaled candidate takes
    # it into account, its rows end up at 2^14 all the same, and the result is that of the direct calls on this handle
    A4, B4, _ = _problem("N", "N", M, N, K, TYPE4, TYPE1, 11, 0)
    mode, out4 = choice_for(A4, B4)
    assert mode == SCALED
    h.set_scaling(0, 0)
    mode, out4_plain = choice_for(A4, B4)
    assert mode == SCALED and np.array_equal(out4.view(np.uint32), out4_plain.view(np.uint32))
    c64 = gemm.sgemm_fp64_ref("N", "N", M, N, K, 1.0, A4, B4)
    assert gemm.relative_residual(c64, out4) <= 1.25 * gemm.relative_residual(c64, gemm.sgemm_fp32_naive("N", "N", M, N, K, 1.0, A4, B4))
    # rows too short for either FP16 arrangement to be worth it (a handful of elements carry each dot product): the
    # exact three-term split, although the pair would represent the scaled operands
    short = 96
    A5, B5, _ = _problem("N", "N", M, N, short, TYPE3, TYPE3, 12, 0)
    assert split.fp16_pair_represents(split.scale_rows(A5[:M, :short], split.row_scale_exponents(A5[:M, :short])),
                                      split.scale_rows(B5[:short, :N].T, split.row_scale_exponents(B5[:short, :N].T)))
    dA, dB, dC = to_device(A5), to_device(B5), to_device(C)
    h.sgemm(*ops, M, N, short, 1.0, dA, M, dB, short, 0.0, dC, M, ec.MODE_AUTO)
    assert h.auto_choice() == BF16 and split.automatic_choice(A5[:M, :short], B5[:short, :N]) == "bf16"
    h.destroy()


def test_workspace_size_caller_workspace_and_refusals():
    import torch
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    M, N, K = 700, 520, 3000
    A, B, C = _problem("N", "N", M, N, K, TYPE3, TYPE3, 11, 0)
    dA, dB, dC = to_device(A), to_device(B), to_device(C)
    need = h.workspace_size(ec.OP_N, ec.OP_N, M, N, K, ec.MODE_AUTO)
    assert need > max(h.workspace_size(ec.OP_N, ec.OP_N, M, N, K, m) for m in (ec.MODE_FP16_SPLIT, ec.MODE_BF16_FULL))
    want, _, _ = _run_scaled(h, "N", "N", M, N, K, 1.0, A, B, 0.0, C)
    guard = 4096
    buf = torch.full((need + guard,), 0x5A, dtype=torch.uint8, device="cuda")
    h.set_workspace(buf, need)
    h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, ec.MODE_AUTO)
    assert h.auto_choice() == (ec.MODE_FP16_SPLIT, True)
    assert np.array_equal(to_host(dC, M, N).view(np.uint32), want.view(np.uint32))
    assert bool((buf[need:] == 0x5A).all())                     # nothing is written past the size asked for
    h.set_workspace(buf, need - 256)
    with pytest.raises(ec.EcgemmError) as err:
        h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, ec.MODE_AUTO)
    assert err.value.status == ec.ERR_ALLOC
    h.set_workspace(None, 0)
    # no choice to report: the last call failed, was in a fixed mode, or did nothing
    for make_call in (lambda: None,
                      lambda: h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, ec.MODE_FP16_SPLIT),
                      lambda: h.sgemm(ec.OP_N, ec.OP_N, M, N, 0, 1.0, dA, M, dB, K, 0.0, dC, M, ec.MODE_AUTO)):
        make_call()
        with pytest.raises(ec.EcgemmError) as err:
            h.auto_choice()
        assert err.value.status == ec.ERR_INVALID_ARG and err.value.argument == 1
    # where the automatic mode does not exist
    scales_a = torch.zeros(M, dtype=torch.int32, device="cuda")
    scales_b = torch.zeros(N, dtype=torch.int32, device="cuda")
    with pytest.raises(ec.EcgemmError) as err:
        h.sgemm_scaled(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, ec.MODE_AUTO, scales_a, scales_b)
    assert err.value.status == ec.ERR_UNSUPPORTED
    h.set_shape(ec.SHAPE_64x64_FUSED)
    with pytest.raises(ec.EcgemmError) as err:
        h.sgemm(ec.OP_N, ec.OP_N, M, N, K, 1.0, dA, M, dB, K, 0.0, dC, M, ec.MODE_AUTO)
    assert err.value.status == ec.ERR_UNSUPPORTED
    with pytest.raises(ec.EcgemmError) as err:
        h.workspace_size(ec.OP_N, ec.OP_N, M, N, K, ec.MODE_AUTO)
    assert err.value.status == ec.ERR_UNSUPPORTED
    h.set_shape(ec.SHAPE_AUTO)
    packed = torch.empty(ec.split_size(M, K, ec.MODE_BF16_FULL), dtype=torch.uint8, device="cuda")
    with pytest.raises(ec.EcgemmError) as err:
        h.split(ec.OP_N, M, K, dA, M, ec.MODE_AUTO, packed)
    assert err.value.status == ec.ERR_INVALID_ARG and err.value.argument == 7
    with pytest.raises(ec.EcgemmError) as err:
        h.product(M, N, K, 1.0, packed, packed, 0.0, dC, M, ec.MODE_AUTO)
    assert err.value.status == ec.ERR_INVALID_ARG and err.value.argument == 11
    with pytest.raises(ec.EcgemmError) as err:
        ec.plan_info(M, N, K, ec.MODE_AUTO)
    assert err.value.status == ec.ERR_INVALID_ARG
    h.destroy()


def test_one_captured_graph_takes_either_branch_depending_on_the_data():
    """The call never waits for the GPU, so it can be recorded into a HIP graph; the choice is made again on every
    replay, from whatever the operand buffers hold then."""
    import torch
    import paper_2203_03341_amd as ec
    M, N, K = 640, 512, 1536
    inputs = {"fp16": _problem("N", "T", M, N, K, "urand", "urand", 13, 0),
              "scaled": _problem("N", "T", M, N, K, TYPE3, TYPE4, 14, 0),
              "bf16": _problem("N", "T", M, N, K, "urand", TYPE1, 15, 0)}
    inputs["bf16"][0][3, 4] = np.nan            # only the full-range mode is left
    h = ec.Handle()
    stream = torch.cuda.Stream()
    h.set_stream(stream.cuda_stream)
    nbytes = h.workspace_size(ec.OP_N, ec.OP_T, M, N, K, ec.MODE_AUTO)
    workspace = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    h.set_workspace(workspace, nbytes)
    dev = {k: tuple(to_device(x) for x in v) for k, v in inputs.items()}
    dA, dB, dC_in = (torch.empty_like(t) for t in dev["fp16"])
    dC = torch.empty_like(dC_in)

    def load(which):
        for dst, src in zip((dA, dB, dC_in), dev[which]):
            dst.copy_(src)

    def call(mode):
        dC.copy_(dC_in)
        h.sgemm(ec.OP_N, ec.OP_T, M, N, K, 1.5, dA, M, dB, N, 0.5, dC, M, mode)

    eager = {}
    with torch.cuda.stream(stream):
        for which, mode in (("fp16", ec.MODE_FP16_SPLIT), ("bf16", ec.MODE_BF16_FULL)):
            load(which)
            call(mode)
            stream.synchronize()
            eager[which] = dC.cpu().numpy().copy()
        load("scaled")
        dC.copy_(dC_in)
        sa = torch.empty(M, dtype=torch.int32, device="cuda")
        sb = torch.empty(N, dtype=torch.int32, device="cuda")
        h.row_scales(ec.OP_N, M, K, dA, M, 14, sa)
        h.row_scales(ec.OP_N, N, K, dB, N, 14, sb)          # B is stored N x K (transB == T): its columns are the rows here
        h.sgemm_scaled(ec.OP_N, ec.OP_T, M, N, K, 1.5, dA, M, dB, N, 0.5, dC, M, ec.MODE_FP16_SPLIT, sa, sb)
        stream.synchronize()
        eager["scaled"] = dC.cpu().numpy().copy()
        load("fp16")
        call(ec.MODE_AUTO)                      # once eagerly, so that nothing is created during the capture
        stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        call(ec.MODE_AUTO)
    for which in ("bf16", "fp16", "scaled", "scaled", "fp16", "bf16"):
        with torch.cuda.stream(stream):
            load(which)
            dC.fill_(float("nan"))
        stream.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, want = dC.cpu().numpy(), eager[which]
        assert np.array_equal(np.isnan(got), np.isnan(want)), which
        assert np.array_equal(got.view(np.uint32)[~np.isnan(got)], want.view(np.uint32)[~np.isnan(want)]), which
    del graph
    h.destroy()
