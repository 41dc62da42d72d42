"""ctypes binding of libabft with the same names as the C ABI (include/abft.h).

Argument marshalling only: tensors become device pointers, Python numbers
become C scalars.  Every step of the protected GEMM runs in the HIP library;
there is no fallback: if libabft.so cannot be loaded the import of this module
raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libabft.so")

__all__ = [
    "ABFT_I8", "ABFT_BF16", "ABFT_F16", "ABFT_OFF", "ABFT_DETECT", "ABFT_DETECT_CORRECT",
    "ABFT_B_CHECKSUM_CACHED", "ABFT_STORED_SUMS", "ABFT_A_CHECKSUM_GIVEN", "ABFT_WS_C_MAX", "abft_supply_a", "abft_gemm_done_event", "ABFT_DISC_FUSED", "ABFT_DISC_STORED", "ABFT_OK", "ABFT_EINVAL", "ABFT_EALIGN", "ABFT_ESHAPE", "ABFT_EWORKSPACE",
    "ABFT_EHIP", "ABFT_ESTATE", "ABFT_CLEAN", "ABFT_LOCALISED", "ABFT_CHECKSUM_SUSPECT", "ABFT_TOO_MANY",
    "ABFT_INJECT_STORED_C", "ABFT_INJECT_ACCUMULATOR", "ABFT_INJECT_OPERAND_A", "ABFT_INJECT_OPERAND_B",
    "ABFT_WS_A_SUM", "ABFT_WS_B_SUM", "ABFT_WS_CC_PRED", "ABFT_WS_RC_PRED", "ABFT_WS_CC_OBS",
    "ABFT_WS_RC_OBS", "ABFT_WS_CC_VOBS", "ABFT_WS_RC_VOBS", "ABFT_WS_TAU", "ABFT_WS_S_PRED", "ABFT_WS_MAXABS", "ABFT_WS_CC_STO", "ABFT_WS_RC_STO",
    "abft_shape", "abft_config", "abft_result", "AbftError", "lib", "lib_path", "exported_symbols",
    "abft_create", "abft_destroy", "abft_encode_b", "abft_gemm", "abft_gemm_bias", "abft_gemm_static", "abft_verify", "abft_correct",
    "abft_correct_checksum", "abft_inject", "abft_discrepancy", "abft_workspace", "abft_tile_shape", "abft_strerror", "abft_last_hip_error",
    "abft_version", "abft_mfma_peak", "abft_profile_begin", "abft_profile_end", "make_shape", "make_result", "DTYPE_CODE",
]

ABFT_I8, ABFT_BF16, ABFT_F16 = 0, 1, 2
DTYPE_CODE = {"i8": ABFT_I8, "bf16": ABFT_BF16, "f16": ABFT_F16}
ABFT_OFF, ABFT_DETECT, ABFT_DETECT_CORRECT = 0, 1, 2
ABFT_B_CHECKSUM_CACHED = 0x10
ABFT_STORED_SUMS = 0x20
ABFT_A_CHECKSUM_GIVEN = 0x40
ABFT_WS_C_MAX = 13
ABFT_DISC_FUSED, ABFT_DISC_STORED = 0, 1
ABFT_OK, ABFT_EINVAL, ABFT_EALIGN, ABFT_ESHAPE, ABFT_EWORKSPACE, ABFT_EHIP, ABFT_ESTATE = 0, -1, -2, -3, -4, -5, -6
ABFT_CLEAN, ABFT_LOCALISED, ABFT_CHECKSUM_SUSPECT, ABFT_TOO_MANY = 0, 1, 2, 3
ABFT_INJECT_STORED_C, ABFT_INJECT_ACCUMULATOR, ABFT_INJECT_OPERAND_A, ABFT_INJECT_OPERAND_B = 0, 1, 2, 3
(ABFT_WS_A_SUM, ABFT_WS_B_SUM, ABFT_WS_CC_PRED, ABFT_WS_RC_PRED, ABFT_WS_CC_OBS, ABFT_WS_RC_OBS,
 ABFT_WS_CC_VOBS, ABFT_WS_RC_VOBS, ABFT_WS_TAU, ABFT_WS_S_PRED, ABFT_WS_MAXABS,
 ABFT_WS_CC_STO, ABFT_WS_RC_STO) = range(13)


class abft_shape(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("batch", ctypes.c_int64),
                ("lda", ctypes.c_int64), ("ldb", ctypes.c_int64), ("ldc", ctypes.c_int64),
                ("strideA", ctypes.c_int64), ("strideB", ctypes.c_int64), ("strideC", ctypes.c_int64),
                ("transB", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class abft_config(ctypes.Structure):
    _fields_ = [("max_rows", ctypes.c_int64), ("max_cols", ctypes.c_int64), ("max_depth", ctypes.c_int64),
                ("max_batch", ctypes.c_int64), ("device", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class abft_result(ctypes.Structure):
    _fields_ = [("row_flag", ctypes.c_void_p), ("col_flag", ctypes.c_void_p), ("counts", ctypes.c_void_p),
                ("tau", ctypes.c_float), ("tau_cols", ctypes.c_float)]


class AbftError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {abft_strerror(code)} ({code})")


_SIGS = {
    "abft_create": (ctypes.c_int, [ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(abft_config)]),
    "abft_destroy": (ctypes.c_int, [ctypes.c_void_p]),
    "abft_encode_b": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                     ctypes.POINTER(abft_shape), ctypes.c_void_p]),
    "abft_gemm": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                 ctypes.c_int, ctypes.c_int, ctypes.POINTER(abft_shape),
                                 ctypes.POINTER(abft_result), ctypes.c_void_p]),
    "abft_gemm_bias": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.POINTER(abft_shape),
                                      ctypes.POINTER(abft_result), ctypes.c_void_p]),
    "abft_gemm_static": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int, ctypes.c_int, ctypes.POINTER(abft_shape),
                                        ctypes.POINTER(abft_result), ctypes.c_void_p]),
    "abft_supply_a": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "abft_gemm_done_event": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p]),
    "abft_verify": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(abft_shape),
                                   ctypes.POINTER(abft_result), ctypes.c_void_p]),
    "abft_correct": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                    ctypes.c_int, ctypes.POINTER(abft_shape), ctypes.POINTER(abft_result),
                                    ctypes.c_void_p]),
    "abft_correct_checksum": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                             ctypes.POINTER(abft_shape), ctypes.POINTER(abft_result),
                                             ctypes.c_void_p]),
    "abft_inject": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(abft_shape),
                                   ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_void_p]),
    "abft_discrepancy": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(abft_shape), ctypes.c_int,
                                        ctypes.c_void_p, ctypes.c_void_p]),
    "abft_workspace": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(abft_shape),
                                      ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_int64)]),
    "abft_tile_shape": (ctypes.c_int, [ctypes.c_int, ctypes.POINTER(abft_shape), ctypes.POINTER(ctypes.c_int),
                                       ctypes.POINTER(ctypes.c_int)]),
    "abft_profile_begin": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int]),
    "abft_profile_end": (ctypes.c_int, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_double),
                                        ctypes.POINTER(ctypes.c_int)]),
    "abft_mfma_peak": (ctypes.c_int, [ctypes.c_int, ctypes.c_double, ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]),
    "abft_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "abft_last_hip_error": (ctypes.c_int, [ctypes.c_void_p]),
    "abft_version": (ctypes.c_int, []),
}

_lib = None


def lib_path() -> str:
    return _LIB_PATH


def exported_symbols():
    """Names the header declares (and the binding expects the library to export)."""
    return sorted(_SIGS)


def lib():
    """The loaded libabft.so; built in-tree first if no built library is there."""
    global _lib
    if _lib is None:
        # torch first: its HIP runtime must be the one libabft binds to, so that device
        # pointers and stream handles mean the same thing on both sides
        import torch  # noqa: F401
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build(force=True)
        L = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(L, name)          # AttributeError if a declared symbol is not exported
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _ptr(x):
    """Device pointer of a tensor-like (anything with data_ptr()), an int, or None."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return ctypes.c_void_p(x.data_ptr())
    return ctypes.c_void_p(int(x))


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def make_shape(M, N, K, batch=1, lda=None, ldb=None, ldc=None, strideA=None, strideB=None, strideC=None,
               transB=True) -> abft_shape:
    lda = K if lda is None else lda
    ldb = (K if transB else N) if ldb is None else ldb
    ldc = N if ldc is None else ldc
    strideA = M * lda if strideA is None else strideA
    strideB = (N if transB else K) * ldb if strideB is None else strideB
    strideC = M * ldc if strideC is None else strideC
    return abft_shape(M, N, K, batch, lda, ldb, ldc, strideA, strideB, strideC, 1 if transB else 0, 0)


def make_result(row_flag, col_flag, counts, tau: float = 0.0, tau_cols: float = 0.0) -> abft_result:
    return abft_result(_ptr(row_flag), _ptr(col_flag), _ptr(counts), float(tau), float(tau_cols))


def abft_strerror(code: int) -> str:
    return lib().abft_strerror(int(code)).decode()


def abft_version() -> int:
    return int(lib().abft_version())


def abft_last_hip_error(ctx) -> int:
    return int(lib().abft_last_hip_error(ctx))


def abft_create(max_rows: int, max_cols: int, max_depth: int, max_batch: int = 1, device: int = 0):
    cfg = abft_config(max_rows, max_cols, max_depth, max_batch, device, 0)
    out = ctypes.c_void_p()
    rc = lib().abft_create(ctypes.byref(out), ctypes.byref(cfg))
    if rc != ABFT_OK:
        raise AbftError(rc, "abft_create")
    return out


def abft_destroy(ctx) -> int:
    return int(lib().abft_destroy(ctx))


def abft_encode_b(ctx, B, dtype: int, shape: abft_shape, stream=None) -> int:
    return int(lib().abft_encode_b(ctx, _ptr(B), dtype, ctypes.byref(shape), _stream(stream)))


def abft_gemm(ctx, A, B, C, dtype: int, mode: int, shape: abft_shape, result: abft_result | None = None,
              stream=None) -> int:
    r = ctypes.byref(result) if result is not None else None
    return int(lib().abft_gemm(ctx, _ptr(A), _ptr(B), _ptr(C), dtype, mode, ctypes.byref(shape), r,
                               _stream(stream)))


def abft_gemm_bias(ctx, A, B, bias, C, dtype: int, mode: int, shape: abft_shape, result: abft_result | None = None,
                   stream=None) -> int:
    r = ctypes.byref(result) if result is not None else None
    return int(lib().abft_gemm_bias(ctx, _ptr(A), _ptr(B), _ptr(bias), _ptr(C), dtype, mode, ctypes.byref(shape), r,
                                    _stream(stream)))


def abft_gemm_static(A, B, C, dtype: int, mode: int, shape: abft_shape, result: abft_result | None = None,
                     stream=None) -> int:
    r = ctypes.byref(result) if result is not None else None
    return int(lib().abft_gemm_static(_ptr(A), _ptr(B), _ptr(C), dtype, mode, ctypes.byref(shape), r,
                                      _stream(stream)))


def abft_gemm_done_event(ctx, event) -> int:
    """event: a hipEvent_t handle as an integer (torch.cuda.Event(...).cuda_event after its first record), or None"""
    return int(lib().abft_gemm_done_event(ctx, ctypes.c_void_p(int(event)) if event else None))


def abft_supply_a(ctx, a, amax=None) -> int:
    return int(lib().abft_supply_a(ctx, _ptr(a), _ptr(amax)))


def abft_verify(ctx, C, dtype: int, shape: abft_shape, result: abft_result, stream=None) -> int:
    return int(lib().abft_verify(ctx, _ptr(C), dtype, ctypes.byref(shape), ctypes.byref(result),
                                 _stream(stream)))


def abft_correct(ctx, A, B, C, dtype: int, shape: abft_shape, result: abft_result, stream=None) -> int:
    return int(lib().abft_correct(ctx, _ptr(A), _ptr(B), _ptr(C), dtype, ctypes.byref(shape),
                                  ctypes.byref(result), _stream(stream)))


def abft_correct_checksum(ctx, C, dtype: int, shape: abft_shape, result: abft_result, stream=None) -> int:
    return int(lib().abft_correct_checksum(ctx, _ptr(C), dtype, ctypes.byref(shape), ctypes.byref(result),
                                           _stream(stream)))


def abft_inject(ctx, C, dtype: int, shape: abft_shape, batch_idx: int, row: int, col: int, bit: int,
                where: int = ABFT_INJECT_STORED_C, stream=None) -> int:
    return int(lib().abft_inject(ctx, _ptr(C), dtype, ctypes.byref(shape), batch_idx, row, col, bit, where,
                                 _stream(stream)))


def abft_discrepancy(ctx, dtype: int, shape: abft_shape, source: int, stats, stream=None) -> int:
    return int(lib().abft_discrepancy(ctx, dtype, ctypes.byref(shape), source, _ptr(stats), _stream(stream)))


def abft_workspace(ctx, which: int, shape: abft_shape):
    """(device pointer, element count) of a workspace vector."""
    p = ctypes.c_void_p()
    n = ctypes.c_int64()
    rc = lib().abft_workspace(ctx, which, ctypes.byref(shape), ctypes.byref(p), ctypes.byref(n))
    if rc != ABFT_OK:
        raise AbftError(rc, "abft_workspace")
    return p.value, n.value


def abft_profile_begin(ctx, max_calls: int) -> int:
    return int(lib().abft_profile_begin(ctx, int(max_calls)))


def abft_profile_end(ctx):
    """(average ms per call [encode, gemm, compare, total], number of calls recorded)."""
    ms = (ctypes.c_double * 4)()
    n = ctypes.c_int()
    rc = lib().abft_profile_end(ctx, ms, ctypes.byref(n))
    if rc != ABFT_OK:
        raise AbftError(rc, "abft_profile_end")
    return [float(x) for x in ms], n.value


def abft_mfma_peak(dtype: int, seconds: float = 0.1):
    """(1e12 operations per second of a matrix-instruction-only kernel, shader clock in MHz)."""
    t, c = ctypes.c_double(), ctypes.c_double()
    rc = lib().abft_mfma_peak(dtype, float(seconds), ctypes.byref(t), ctypes.byref(c))
    if rc != ABFT_OK:
        raise AbftError(rc, "abft_mfma_peak")
    return t.value, c.value


def abft_tile_shape(dtype: int, shape: abft_shape):
    tm, tn = ctypes.c_int(), ctypes.c_int()
    rc = lib().abft_tile_shape(dtype, ctypes.byref(shape), ctypes.byref(tm), ctypes.byref(tn))
    if rc != ABFT_OK:
        raise AbftError(rc, "abft_tile_shape")
    return tm.value, tn.value
