"""ecgemm_sgemm_noalloc (the entry point for callers that cannot allocate) against ecgemm_sgemm, through the C-ABI.

Both run the same kernels on the same plan, so the results must agree bit for bit; the first is also held to the
oracle's pass rule.  Two calls in a row share the library's built-in workspace, the second with a smaller input, so
that anything the first left behind and the second failed to overwrite would show."""
import numpy as np
import pytest

import seeded_inputs as si
from oracle import gemm
from gpu_util import empty_colmajor, to_device, to_host

pytestmark = pytest.mark.gpu


def _pair(h, transA, transB, M, N, K, alpha, beta, mode, seed):
    import torch
    import paper_2203_03341_amd as ec
    ar, ac = (M, K) if transA == "N" else (K, M)
    br, bc = (K, N) if transB == "N" else (N, K)
    A = si.urand(ar, ac, seed, si.ID_A, ld=ar + 3)
    B = si.exp_rand(br, bc, -8, 8, seed, si.ID_B, ld=br + 1)
    C = si.urand(M, N, seed, si.ID_C, ld=M + 2)
    dA, dB = to_device(A), to_device(B)
    ops = {"N": ec.OP_N, "T": ec.OP_T}
    out = []
    for call in (h.sgemm, h.sgemm_noalloc):
        dC = to_device(C)
        call(ops[transA], ops[transB], M, N, K, alpha, dA, A.shape[0], dB, B.shape[0], beta, dC, C.shape[0], mode)
        torch.cuda.synchronize()
        out.append(to_host(dC, C.shape[0], N))
    want, got = out
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))            # padding rows of C included: untouched by both
    c64 = gemm.sgemm_fp64_ref(transA, transB, M, N, K, alpha, A, B, beta, C)
    c32 = gemm.sgemm_fp32_naive(transA, transB, M, N, K, alpha, A, B, beta, C)
    assert gemm.relative_residual(c64, got[:M, :]) <= 1.25 * gemm.relative_residual(c64, c32)


@pytest.mark.parametrize("mode", ["fp16", "bf16"])
def test_noalloc_entry_point_equals_sgemm_on_two_calls_in_a_row(mode):
    import paper_2203_03341_amd as ec
    mode_id = ec.MODE_FP16_SPLIT if mode == "fp16" else ec.MODE_BF16_FULL
    h = ec.Handle()
    # 21 x 9 tiles of 128 x 128 with ragged edges, deep enough for sliced tiles in the automatic plan ...
    _pair(h, "T", "N", 1300, 1100, 2100, 1.5, 0.5, mode_id, seed=11)
    # ... then a smaller product in the same array, which still holds the first one's operands and partial sums
    _pair(h, "N", "T", 200, 333, 130, -1.0, 0.0, mode_id, seed=12)
    # a problem whose workspace exceeds the built-in array is refused with ECGEMM_ERR_ALLOC before anything is enqueued
    big = 4096
    assert h.workspace_size(ec.OP_N, ec.OP_N, big, big, big, mode_id) > ec.NOALLOC_WORKSPACE_BYTES
    dC = empty_colmajor(8, 8, fill=3.0)
    with pytest.raises(ec.EcgemmError) as err:
        h.sgemm_noalloc(ec.OP_N, ec.OP_N, big, big, big, 1.0, dC, big, dC, big, 0.0, dC, big, mode_id)   # pointers never read
    assert err.value.status == ec.ERR_ALLOC
    h.destroy()


def test_noalloc_entry_point_with_every_kernel_shape():
    """The forced shapes go through the same entry point (the one-launch shapes use none of the array)."""
    import paper_2203_03341_amd as ec
    h = ec.Handle()
    for shape in (ec.SHAPE_256x128_W4, ec.SHAPE_128x128_X2, ec.SHAPE_64x64_FUSED, ec.SHAPE_32x32_FUSED):
        h.set_shape(shape)
        _pair(h, "N", "N", 700, 520, 1536, 1.0, 0.0, ec.MODE_FP16_SPLIT, seed=13)
        _pair(h, "T", "T", 130, 90, 64, 2.0, 1.0, ec.MODE_FP16_SPLIT, seed=14)
    h.destroy()
