"""ctypes binding of libecgemm.so: argument marshalling only, every step runs in the HIP kernels.

The functions mirror include/ecgemm.h one to one.  Matrices are torch CUDA tensors used purely as
device memory: a column-major (ld, cols) matrix is any float32 tensor whose storage holds it, and
the binding passes `data_ptr()` straight through.  There is no CPU fallback: if the shared library
is missing or fails to load, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libecgemm.so")

OP_N, OP_T = 0, 1
MODE_FP16_SPLIT, MODE_BF16_FULL = 0, 1
MODE_FP16_MARKIDIS, MODE_FP16_UNSCALED, MODE_FP16_PLAIN, MODE_BF16_PLAIN, MODE_FP16_OUTSIDE_ACC = 2, 3, 4, 5, 6  # comparisons
MODE_FP32_MFMA = 7  # plain FP32 on the matrix unit
MODE_FP16_OUTSIDE_ACC_4, MODE_FP16_OUTSIDE_ACC_16 = 8, 9
MODE_AUTO = 10
OK, ERR_INVALID_ARG, ERR_ALLOC, ERR_HIP, ERR_UNSUPPORTED = 0, 1, 2, 3, 4
SHAPE_AUTO, SHAPE_256x128_W4, SHAPE_128x128_X2, SHAPE_64x64_FUSED, SHAPE_32x32_FUSED = 0, 1, 2, 3, 4

EXPORTS = ["ecgemm_create", "ecgemm_destroy", "ecgemm_set_stream", "ecgemm_workspace_size", "ecgemm_plan_info", "ecgemm_set_workspace",
           "ecgemm_sgemm", "ecgemm_sgemm_scaled", "ecgemm_sgemm_noalloc", "ecgemm_auto_choice", "ecgemm_last_error_argument", "ecgemm_row_scales", "ecgemm_set_shape", "ecgemm_debug_set_tile_order", "ecgemm_debug_tile_order", "ecgemm_set_scaling", "ecgemm_exponent_range", "ecgemm_choose_mode", "ecgemm_product", "ecgemm_split", "ecgemm_split_size", "ecgemm_debug_mfma", "ecgemm_debug_mfma_rate", "ecgemm_set_timing", "ecgemm_get_timing",
           "ecgemm_last_error_string", "ecgemm_status_string"]


class PlanInfo(ctypes.Structure):
    """ecgemm_plan_info_t"""
    _fields_ = [("shape", ctypes.c_int), ("tile_m", ctypes.c_int), ("tile_n", ctypes.c_int), ("tiles_m", ctypes.c_int),
                ("tiles_n", ctypes.c_int), ("whole_tiles", ctypes.c_int), ("sliced_tiles", ctypes.c_int),
                ("slices", ctypes.c_int), ("persistent", ctypes.c_int), ("group_m", ctypes.c_int),
                ("column_bands", ctypes.c_int), ("grid", ctypes.c_int64),
                ("workspace_bytes", ctypes.c_size_t), ("estimated_us", ctypes.c_double)]

    def as_dict(self) -> dict:
        return {name: (float if name == "estimated_us" else int)(getattr(self, name)) for name, _ in self._fields_}


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no fallback path)")
    # PyTorch ships its own copy of the HIP runtime.  If this library were loaded first it would pull in the system's
    # copy, torch would then find a second runtime in the process and report no GPU: let torch load its copy first
    # (the library then binds to the one already there).
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    i64, f32, vp, sz = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
    lib.ecgemm_create.argtypes = [ctypes.POINTER(vp)]
    lib.ecgemm_destroy.argtypes = [vp]
    lib.ecgemm_set_stream.argtypes = [vp, vp]
    lib.ecgemm_workspace_size.argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, i64, i64, ctypes.c_int, ctypes.POINTER(sz)]
    lib.ecgemm_set_workspace.argtypes = [vp, vp, sz]
    lib.ecgemm_plan_info.argtypes = [vp, i64, i64, i64, ctypes.c_int, ctypes.POINTER(PlanInfo)]
    lib.ecgemm_sgemm.argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, i64, i64, f32, vp, i64, vp, i64, f32, vp, i64,
                                 ctypes.c_int]
    lib.ecgemm_sgemm_noalloc.argtypes = lib.ecgemm_sgemm.argtypes
    lib.ecgemm_last_error_argument.argtypes = [vp]
    lib.ecgemm_auto_choice.argtypes = [vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.ecgemm_sgemm_scaled.argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, i64, i64, f32, vp, i64, vp, i64, f32, vp, i64,
                                        ctypes.c_int, vp, vp]
    lib.ecgemm_row_scales.argtypes = [vp, ctypes.c_int, i64, i64, vp, i64, ctypes.c_int, vp]
    lib.ecgemm_set_shape.argtypes = [vp, ctypes.c_int]
    lib.ecgemm_debug_set_tile_order.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    lib.ecgemm_debug_tile_order.argtypes = [vp, i64, i64, i64, ctypes.c_int, vp, vp, ctypes.POINTER(i64)]
    lib.ecgemm_set_scaling.argtypes = [vp, ctypes.c_int, ctypes.c_int]
    lib.ecgemm_exponent_range.argtypes = [vp, i64, i64, vp, i64, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.ecgemm_choose_mode.argtypes = [vp, ctypes.c_int, ctypes.c_int, i64, i64, i64, vp, i64, vp, i64,
                                       ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.ecgemm_product.argtypes = [vp, i64, i64, i64, f32, vp, vp, f32, vp, i64, ctypes.c_int]
    lib.ecgemm_split.argtypes = [vp, ctypes.c_int, i64, i64, vp, i64, ctypes.c_int, vp]
    lib.ecgemm_split_size.argtypes = [i64, i64, ctypes.c_int, ctypes.POINTER(sz)]
    lib.ecgemm_debug_mfma.argtypes = [vp, ctypes.c_int, i64, vp, vp, vp, vp]
    lib.ecgemm_debug_mfma_rate.argtypes = [vp, ctypes.c_int, vp, vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
    lib.ecgemm_set_timing.argtypes = [vp, ctypes.c_int]
    lib.ecgemm_get_timing.argtypes = [vp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(f32), ctypes.POINTER(f32)]
    lib.ecgemm_last_error_string.argtypes = [vp]
    lib.ecgemm_last_error_string.restype = ctypes.c_char_p
    lib.ecgemm_status_string.argtypes = [ctypes.c_int]
    lib.ecgemm_status_string.restype = ctypes.c_char_p
    for name in EXPORTS:       # (ecgemm_last_error_argument returns a plain int as well)
        if getattr(lib, name).restype is not ctypes.c_char_p:
            getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


NOALLOC_WORKSPACE_BYTES = 64 << 20      # ECGEMM_NOALLOC_WORKSPACE_BYTES


class EcgemmError(RuntimeError):
    def __init__(self, status: int, detail: str, argument: int = 0):
        self.status = status
        self.argument = argument        # ecgemm_last_error_argument at the time of the failure
        super().__init__(f"{_lib.ecgemm_status_string(status).decode()}: {detail}")


def _ptr(t) -> int:
    """Device address of a torch tensor (or a raw integer address, or None)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return t.data_ptr()


class Handle:
    """Owns one ecgemm_handle_t.  Methods have the names and argument order of the C functions."""

    def __init__(self):
        h = ctypes.c_void_p()
        st = _lib.ecgemm_create(ctypes.byref(h))
        if st != OK:
            raise EcgemmError(st, "ecgemm_create")
        self._h = h

    def _check(self, st: int):
        if st != OK:
            raise EcgemmError(st, _lib.ecgemm_last_error_string(self._h).decode(), _lib.ecgemm_last_error_argument(self._h))

    def last_error_argument(self) -> int:
        return _lib.ecgemm_last_error_argument(self._h)

    def destroy(self):
        if self._h:
            st = _lib.ecgemm_destroy(self._h)
            self._h = None
            if st != OK:
                raise EcgemmError(st, "ecgemm_destroy")

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def set_stream(self, stream_ptr: int):
        self._check(_lib.ecgemm_set_stream(self._h, stream_ptr))

    def workspace_size(self, transA: int, transB: int, M: int, N: int, K: int, mode: int) -> int:
        out = ctypes.c_size_t()
        self._check(_lib.ecgemm_workspace_size(self._h, transA, transB, M, N, K, mode, ctypes.byref(out)))
        return out.value

    def plan_info(self, M: int, N: int, K: int, mode: int) -> dict:
        info = PlanInfo()
        self._check(_lib.ecgemm_plan_info(self._h, M, N, K, mode, ctypes.byref(info)))
        return info.as_dict()

    def set_workspace(self, buffer, nbytes: int):
        self._check(_lib.ecgemm_set_workspace(self._h, _ptr(buffer), nbytes))

    def sgemm(self, transA: int, transB: int, M: int, N: int, K: int, alpha: float, A, lda: int, B, ldb: int,
              beta: float, C, ldc: int, mode: int):
        self._check(_lib.ecgemm_sgemm(self._h, transA, transB, M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                      _ptr(C), ldc, mode))

    def auto_choice(self):
        """(mode, on row / column scaled operands?) of the last sgemm / sgemm_noalloc call (MODE_AUTO); waits for the stream."""
        mode, scaled = ctypes.c_int(-1), ctypes.c_int(-1)
        self._check(_lib.ecgemm_auto_choice(self._h, ctypes.byref(mode), ctypes.byref(scaled)))
        return mode.value, bool(scaled.value)

    def sgemm_noalloc(self, transA: int, transB: int, M: int, N: int, K: int, alpha: float, A, lda: int, B, ldb: int,
                      beta: float, C, ldc: int, mode: int):
        self._check(_lib.ecgemm_sgemm_noalloc(self._h, transA, transB, M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                              _ptr(C), ldc, mode))

    def sgemm_scaled(self, transA: int, transB: int, M: int, N: int, K: int, alpha: float, A, lda: int, B, ldb: int,
                     beta: float, C, ldc: int, mode: int, row_log2_scale_a, col_log2_scale_b):
        self._check(_lib.ecgemm_sgemm_scaled(self._h, transA, transB, M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                             _ptr(C), ldc, mode, _ptr(row_log2_scale_a), _ptr(col_log2_scale_b)))

    def row_scales(self, op: int, rows: int, depth: int, src, ld: int, target_exponent: int, log2_scale):
        self._check(_lib.ecgemm_row_scales(self._h, op, rows, depth, _ptr(src), ld, target_exponent, _ptr(log2_scale)))

    def set_shape(self, shape: int):
        self._check(_lib.ecgemm_set_shape(self._h, shape))

    def debug_set_tile_order(self, xcd_remap: int, group_m: int, column_bands: int):
        self._check(_lib.ecgemm_debug_set_tile_order(self._h, xcd_remap, group_m, column_bands))

    def set_scaling(self, log2_scale_a: int, log2_scale_b: int):
        self._check(_lib.ecgemm_set_scaling(self._h, log2_scale_a, log2_scale_b))

    def exponent_range(self, rows: int, cols: int, src, ld: int):
        lo, hi = ctypes.c_int(), ctypes.c_int()
        self._check(_lib.ecgemm_exponent_range(self._h, rows, cols, _ptr(src), ld, ctypes.byref(lo), ctypes.byref(hi)))
        return lo.value, hi.value

    def choose_mode(self, transA: int, transB: int, M: int, N: int, K: int, A, lda: int, B, ldb: int):
        """(mode, log2_scale_a, log2_scale_b) recommended for this product."""
        mode, sa, sb = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        self._check(_lib.ecgemm_choose_mode(self._h, transA, transB, M, N, K, _ptr(A), lda, _ptr(B), ldb, ctypes.byref(mode),
                                            ctypes.byref(sa), ctypes.byref(sb)))
        return mode.value, sa.value, sb.value

    def product(self, M: int, N: int, K: int, alpha: float, packedA, packedB, beta: float, C, ldc: int, mode: int):
        self._check(_lib.ecgemm_product(self._h, M, N, K, alpha, _ptr(packedA), _ptr(packedB), beta, _ptr(C), ldc, mode))

    def split(self, op: int, rows: int, depth: int, src, ld: int, mode: int, packed):
        self._check(_lib.ecgemm_split(self._h, op, rows, depth, _ptr(src), ld, mode, _ptr(packed)))

    def debug_mfma(self, bf16: bool, count: int, a, b, c, d):
        self._check(_lib.ecgemm_debug_mfma(self._h, int(bf16), count, _ptr(a), _ptr(b), _ptr(c), _ptr(d)))

    def debug_mfma_rate(self, bf16: bool, operands, sink, blocks: int, iters: int) -> float:
        """Enqueues the matrix-instruction-only kernel; returns the flops it performs."""
        flops = ctypes.c_double()
        self._check(_lib.ecgemm_debug_mfma_rate(self._h, int(bf16), _ptr(operands), _ptr(sink), blocks, iters, ctypes.byref(flops)))
        return flops.value

    def set_timing(self, enabled: bool):
        self._check(_lib.ecgemm_set_timing(self._h, int(enabled)))

    def get_timing(self):
        """(calls, split_ms, product_ms) summed over the calls since timing was enabled / last read."""
        calls, a, b = ctypes.c_int(), ctypes.c_float(), ctypes.c_float()
        self._check(_lib.ecgemm_get_timing(self._h, ctypes.byref(calls), ctypes.byref(a), ctypes.byref(b)))
        return calls.value, a.value, b.value


def workspace_size(transA: int, transB: int, M: int, N: int, K: int, mode: int) -> int:
    """ecgemm_workspace_size without a handle (none is needed)."""
    out = ctypes.c_size_t()
    st = _lib.ecgemm_workspace_size(None, transA, transB, M, N, K, mode, ctypes.byref(out))
    if st != OK:
        raise EcgemmError(st, "ecgemm_workspace_size")
    return out.value


def plan_info(M: int, N: int, K: int, mode: int) -> dict:
    """ecgemm_plan_info without a handle (automatic kernel shape)."""
    info = PlanInfo()
    st = _lib.ecgemm_plan_info(None, M, N, K, mode, ctypes.byref(info))
    if st != OK:
        raise EcgemmError(st, "ecgemm_plan_info")
    return info.as_dict()


def debug_tile_order(M: int, N: int, K: int, mode: int, handle=None):
    """(tile_m, tile_n, disagreements): coordinates of the output tiles in hand-out order (numpy int32 arrays) and the
    number of tiles on which the kernels' reciprocal arithmetic and plain division disagree."""
    import numpy as np
    info = PlanInfo()
    h = handle._h if handle is not None else None
    st = _lib.ecgemm_plan_info(h, M, N, K, mode, ctypes.byref(info))
    if st != OK:
        raise EcgemmError(st, "ecgemm_plan_info")
    tiles = info.tiles_m * info.tiles_n
    tile_m, tile_n = np.full(tiles, -1, dtype=np.int32), np.full(tiles, -1, dtype=np.int32)
    bad = ctypes.c_int64(-1)
    st = _lib.ecgemm_debug_tile_order(h, M, N, K, mode, tile_m.ctypes.data, tile_n.ctypes.data, ctypes.byref(bad))
    if st != OK:
        raise EcgemmError(st, "ecgemm_debug_tile_order")
    return tile_m, tile_n, bad.value


def split_size(rows: int, depth: int, mode: int) -> int:
    out = ctypes.c_size_t()
    st = _lib.ecgemm_split_size(rows, depth, mode, ctypes.byref(out))
    if st != OK:
        raise EcgemmError(st, "ecgemm_split_size")
    return out.value


def status_string(status: int) -> str:
    return _lib.ecgemm_status_string(status).decode()
