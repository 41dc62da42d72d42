"""Plumbing shared by the GPU parity tests, bench.py and the smoke run: upload operands, call the
library through its C-ABI binding, read results and workspace vectors back as numpy arrays.
No arithmetic of the method lives here, and nothing here is called inside a timed region (the
methods of Run synchronise)."""
from __future__ import annotations

import numpy as np
import torch

import paper_2310_03841_amd as ab


class _DevView:
    def __init__(self, ptr, n, typestr):
        self.__cuda_array_interface__ = {"shape": (int(n),), "typestr": typestr, "data": (int(ptr), False),
                                         "version": 2}


def read_ws(ctx, which, shape, kind):
    """Workspace vector as a numpy array; kind 'i' -> int32 (ring values), 'u' -> uint32, 'f' -> float32."""
    ptr, n = ab.abft_workspace(ctx, which, shape)
    torch.cuda.synchronize()
    t = torch.as_tensor(_DevView(ptr, n, "<u4"), device="cuda").clone().cpu().numpy().view(np.uint32)
    if kind == "f":
        return t.view(np.float32).copy()
    if kind == "i":
        return t.view(np.int32).copy()
    return t.copy()


def pad_ld(n, elem_bytes):
    q = 16 // elem_bytes
    return (n + q - 1) // q * q


def to_dev(arr: np.ndarray, ld: int):
    """Host array (..., rows, cols) -> device tensor with rows padded to ld elements (pad = garbage-ish)."""
    a = np.ascontiguousarray(arr)
    rows, cols = a.shape[-2], a.shape[-1]
    if ld != cols:
        pad_shape = a.shape[:-1] + (ld,)
        # fill the pad with a recognisable non-zero pattern: the library must never use it
        p = np.full(pad_shape, 0x55 if a.dtype.itemsize == 1 else 0x3C55, dtype=a.dtype)
        p[..., :cols] = a
        a = p
    tdt = {np.dtype(np.int8): torch.int8, np.dtype(np.uint16): torch.int16, np.dtype(np.int32): torch.int32}[a.dtype]
    return torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to("cuda").view(tdt)


class Run:
    """One protected GEMM problem on the GPU."""

    def __init__(self, ctx, dtype: str, A: np.ndarray, B: np.ndarray, trans_b: bool):
        self.ctx, self.dtype, self.code = ctx, dtype, ab.DTYPE_CODE[dtype]
        self.batch, self.M, self.K = A.shape
        self.N = B.shape[1] if trans_b else B.shape[2]
        es = 1 if dtype == "i8" else 2
        osz = 4 if dtype == "i8" else 2
        self.lda = pad_ld(self.K, es)
        self.ldb = pad_ld(self.K if trans_b else self.N, es)
        self.ldc = pad_ld(self.N, osz)
        self.trans_b = trans_b
        self.dA = to_dev(A, self.lda)
        self.dB = to_dev(B, self.ldb)
        out_t = torch.int32 if dtype == "i8" else torch.int16
        self.dC = torch.full((self.batch, self.M, self.ldc), 0x5A5A if osz == 2 else 0x5A5A5A5A, dtype=out_t,
                             device="cuda")
        self.shape = ab.make_shape(self.M, self.N, self.K, batch=self.batch, lda=self.lda, ldb=self.ldb,
                                   ldc=self.ldc, transB=trans_b)
        self.row_flag = torch.full((self.batch * self.M,), 7, dtype=torch.uint8, device="cuda")
        self.col_flag = torch.full((self.batch * self.N,), 7, dtype=torch.uint8, device="cuda")
        self.counts = torch.full((8,), 99, dtype=torch.int32, device="cuda")
        self.tau = 0.0
        self.tau_cols = 0.0

    def result(self):
        return ab.make_result(self.row_flag, self.col_flag, self.counts, self.tau, self.tau_cols)

    def gemm(self, mode=ab.ABFT_DETECT):
        rc = ab.abft_gemm(self.ctx, self.dA, self.dB, self.dC, self.code, mode, self.shape,
                          None if (mode & 0xF) == ab.ABFT_OFF else self.result())
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
        torch.cuda.synchronize()

    def gemm_bias(self, bias, mode=ab.ABFT_DETECT):
        """bias: device tensor of N float32 (bf16 / f16) or int32 (i8) values"""
        rc = ab.abft_gemm_bias(self.ctx, self.dA, self.dB, bias, self.dC, self.code, mode, self.shape,
                               None if (mode & 0xF) == ab.ABFT_OFF else self.result())
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
        torch.cuda.synchronize()

    def inject_operand(self, which, b, row, col, bit):
        """which: 'A' or 'B'; (row, col) index the operand array as stored"""
        where, ptr = (ab.ABFT_INJECT_OPERAND_A, self.dA) if which == "A" else (ab.ABFT_INJECT_OPERAND_B, self.dB)
        rc = ab.abft_inject(self.ctx, ptr, self.code, self.shape, b, row, col, bit, where)
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
        torch.cuda.synchronize()

    def verify(self):
        rc = ab.abft_verify(self.ctx, self.dC, self.code, self.shape, self.result())
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
        torch.cuda.synchronize()

    def correct(self):
        rc = ab.abft_correct(self.ctx, self.dA, self.dB, self.dC, self.code, self.shape, self.result())
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
        torch.cuda.synchronize()

    def correct_checksum(self):
        rc = ab.abft_correct_checksum(self.ctx, self.dC, self.code, self.shape, self.result())
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
        torch.cuda.synchronize()

    def inject(self, b, i, j, bit, where=ab.ABFT_INJECT_STORED_C):
        rc = ab.abft_inject(self.ctx, self.dC, self.code, self.shape, b, i, j, bit, where)
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)

    # ---- read back
    def C(self):
        c = self.dC.cpu().numpy()[:, :, :self.N]
        return c.view(np.uint16) if self.dtype != "i8" else c

    def flags(self):
        return (self.row_flag.cpu().numpy().reshape(self.batch, self.M).astype(bool),
                self.col_flag.cpu().numpy().reshape(self.batch, self.N).astype(bool))

    def cnt(self):
        return self.counts.cpu().numpy().astype(np.int64)

    def ws(self, which):
        kind = "i" if self.dtype == "i8" else "f"
        if which in (ab.ABFT_WS_TAU, ab.ABFT_WS_MAXABS, ab.ABFT_WS_C_MAX):
            kind = "f"
        v = read_ws(self.ctx, which, self.shape, kind)
        return v.reshape(self.batch, -1)
