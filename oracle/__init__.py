"""CPU oracle for the checksum-protected GEMM  --  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The product (the HIP library and its
Python binding) never does, and the two share no code.

The loops live in ``abft_oracle.c`` (plain C, int64 / fp64, k ascending); this
file marshals arrays into them and adds the steps that are not loops: exact
decoding of the storage types, rounding of the fp64 result to the storage type,
bit flips, the flag rule, localisation and correction.

Steps, in the order of the paper's checksum description (Sec. III-B.1,
"Checksums"; the row/column form is the ABFT scheme cited in Sec. I / II-B):
  decode          storage bits -> int64 / fp64, exactly
  gemm            C_ref = A B
  encode          a = e^T A, b = B e                     (length K each)
  predict         cc_pred = a B, rc_pred = A b, s_pred = a.b
  observe         cc_obs = e^T X, rc_obs = X e, s_obs    (X = output as stored)
  flags           integer: obs != pred (Sec. III-B.1 item (2): equality check
                  suffices for fixed point); floating point: |obs-pred| above a
                  tolerance (same item: threshold instead of equality)
  localise        flagged rows x flagged columns
  correct         flagged elements take the recomputed value (replay,
                  Sec. III-B.3, at element granularity)
  with_bias       the layer bias added to every output row and its share in
                  every checksum (Sec. III-B.1 "Checksums")
  calibrated_*    thresholds read off pooled fault-free discrepancies at a
                  confidence level (Sec. III-B.1 "Eps Generation")

Readings of the paper where it is silent (kept in one place):
  * integer checksums live in the ring Z/2^32 (Sec. III-B.1 item (1) names the
    overflow problem, gives no remedy); both the exact-int64 flags and the
    mod-2^32 flags are produced, the latter is what hardware can compute.
  * the floating-point tolerance is one number per GEMM,
    tau = 1e-3 * K * max|A| * max|B|, used for both row and column checks; the
    comparison is written  not(|d| <= tau)  so NaN and Inf always flag.

Pinned in tests/test_oracle_pins.py (integer identity, brute-force flips,
closed forms, numpy matmul cross-check, flip delta linearity, rounding against
library conversions).  Floating-point flag behaviour for flips whose magnitude
is within a factor two of tau has no external pin: "parity unpinned" there.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "abft_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile abft_oracle.c with gcc (OpenMP over output rows)."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_load().oracle_threads())


def _p(x: np.ndarray):
    return x.ctypes.data_as(ctypes.c_void_p)


_L = ctypes.c_long


# ----------------------------------------------------------------------------
# decode / round / flip
# ----------------------------------------------------------------------------
def decode(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Storage bits -> exact int64 (i8, i32) or fp64 (bf16, f16)."""
    if dtype in ("i8", "i32"):
        return np.asarray(bits).astype(np.int64)
    u = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "bf16":
        return (u.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if dtype == "f16":
        return u.view(np.float16).astype(np.float64)
    raise ValueError(dtype)


_FMT = {  # significand bits (with the hidden one), min normal exponent, max finite exponent
    "bf16": (8, -126, 127),
    "f16": (11, -14, 15),
}


def round_to_format(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp64 to the nearest bf16/fp16 value (ties to even), returned as fp64.

    One rounding straight from fp64 (no detour through fp32).  Overflow goes
    to +-Inf as round-to-nearest does (the paper notes this behaviour in
    Sec. III-B.1 item (1)); values below the subnormal quantum round to zero."""
    p, emin, emax = _FMT[dtype]
    x = np.asarray(x, dtype=np.float64)
    out = np.array(x, dtype=np.float64, copy=True)
    fin = np.isfinite(x) & (x != 0.0)
    m, e = np.frexp(x[fin])              # x = m * 2^e, 0.5 <= |m| < 1
    q = np.maximum(e - p, emin + 1 - p)  # exponent of the last kept bit
    r = np.ldexp(np.rint(np.ldexp(x[fin], -q)), q)
    big = np.abs(r) >= np.ldexp(1.0, emax + 1)
    r[big] = np.copysign(np.inf, r[big])
    out[fin] = r
    return out


def encode_bits(v: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 values that are exactly representable in dtype -> uint16 bit patterns."""
    if dtype == "bf16":
        return (np.asarray(v, dtype=np.float64).astype(np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    if dtype == "f16":
        return np.asarray(v, dtype=np.float64).astype(np.float16).view(np.uint16)
    raise ValueError(dtype)


def store(C_ref: np.ndarray, dtype: str) -> np.ndarray:
    """The output as it is stored: int32 for the i8 path, bf16/f16 bits otherwise."""
    if dtype == "i8":
        assert np.all(np.abs(C_ref) < 2 ** 31), "int32 output would overflow"
        return C_ref.astype(np.int32)
    return encode_bits(round_to_format(C_ref, dtype), dtype)


def decode_stored(X: np.ndarray, dtype: str) -> np.ndarray:
    return decode(X, "i32" if dtype == "i8" else dtype)


def flip(X: np.ndarray, row: int, col: int, bit: int) -> np.ndarray:
    """Copy of the stored matrix X with one bit of one element inverted (the single-bit-flip fault
    model of Sec. II-A / III-A).  X is an output (int32 or uint16 bits) or an operand (int8 or
    uint16 bits: flips in inputs and weights are the other injection sites the paper names)."""
    Y = np.array(X, copy=True)
    if Y.dtype == np.int32:
        u = Y.view(np.uint32)
        u[row, col] ^= np.uint32(1 << bit)
    elif Y.dtype == np.int8:
        assert 0 <= bit < 8
        u = Y.view(np.uint8)
        u[row, col] ^= np.uint8(1 << bit)
    else:
        assert Y.dtype == np.uint16 and 0 <= bit < 16
        Y[row, col] ^= np.uint16(1 << bit)
    return Y


# ----------------------------------------------------------------------------
# loops (in C)
# ----------------------------------------------------------------------------
def _strides_b(Bm: np.ndarray, trans_b: bool):
    """Logical B(k, j) strides (in elements) of the stored array."""
    if trans_b:      # stored N x K
        N, K = Bm.shape
        return N, K, 1, K      # b_rs (k step) = 1, b_cs (j step) = K
    K, N = Bm.shape
    return N, K, N, 1


def gemm(A: np.ndarray, Bm: np.ndarray, trans_b: bool) -> np.ndarray:
    """C_ref = A B.  A: (M,K) int8 or fp64.  Bm as stored: (N,K) if trans_b else (K,N)."""
    lib = _load()
    A = np.ascontiguousarray(A)
    Bm = np.ascontiguousarray(Bm)
    M, K = A.shape
    N, K2, brs, bcs = _strides_b(Bm, trans_b)
    assert K == K2
    if A.dtype == np.int8:
        assert Bm.dtype == np.int8
        C = np.empty((M, N), dtype=np.int64)
        lib.oracle_gemm_i8(_p(A), _L(K), _L(1), _p(Bm), _L(brs), _L(bcs), _L(M), _L(N), _L(K), _p(C))
    else:
        assert A.dtype == np.float64 and Bm.dtype == np.float64
        C = np.empty((M, N), dtype=np.float64)
        lib.oracle_gemm_f64(_p(A), _L(K), _L(1), _p(Bm), _L(brs), _L(bcs), _L(M), _L(N), _L(K), _p(C))
    return C


def _wide(x):
    x = np.ascontiguousarray(x)
    return x.astype(np.int64) if x.dtype.kind == "i" else x.astype(np.float64)


def encode(A: np.ndarray, Bm: np.ndarray, trans_b: bool):
    """a[k] = sum_i A[i,k];  b[k] = sum_j B[k,j]."""
    lib = _load()
    A, Bm = _wide(A), _wide(Bm)
    M, K = A.shape
    N, _, brs, bcs = _strides_b(Bm, trans_b)
    a = np.empty(K, dtype=A.dtype)
    b = np.empty(K, dtype=A.dtype)
    fn = lib.oracle_encode_i64 if A.dtype == np.int64 else lib.oracle_encode_f64
    fn(_p(A), _L(K), _L(1), _p(Bm), _L(brs), _L(bcs), _L(M), _L(N), _L(K), _p(a), _p(b))
    return a, b


def predict(A: np.ndarray, Bm: np.ndarray, a: np.ndarray, b: np.ndarray, trans_b: bool):
    """cc_pred = a B (length N), rc_pred = A b (length M), s_pred = a . b."""
    lib = _load()
    A, Bm = _wide(A), _wide(Bm)
    M, K = A.shape
    N, _, brs, bcs = _strides_b(Bm, trans_b)
    cc = np.empty(N, dtype=A.dtype)
    rc = np.empty(M, dtype=A.dtype)
    s = np.empty(1, dtype=A.dtype)
    fn = lib.oracle_predict_i64 if A.dtype == np.int64 else lib.oracle_predict_f64
    fn(_p(A), _L(K), _L(1), _p(Bm), _L(brs), _L(bcs), _p(np.ascontiguousarray(a)),
       _p(np.ascontiguousarray(b)), _L(M), _L(N), _L(K), _p(cc), _p(rc), _p(s))
    return cc, rc, s[0]


def observe(X: np.ndarray):
    """cc_obs = e^T X, rc_obs = X e, s_obs = sum X for a decoded (int64 / fp64) matrix."""
    lib = _load()
    X = _wide(X)
    M, N = X.shape
    cc = np.empty(N, dtype=X.dtype)
    rc = np.empty(M, dtype=X.dtype)
    s = np.empty(1, dtype=X.dtype)
    fn = lib.oracle_observe_i64 if X.dtype == np.int64 else lib.oracle_observe_f64
    with np.errstate(all="ignore"):
        fn(_p(X), _L(M), _L(N), _p(cc), _p(rc), _p(s))
    return cc, rc, s[0]


# ----------------------------------------------------------------------------
# flags, localisation, correction
# ----------------------------------------------------------------------------
def flags_int(obs: np.ndarray, pred: np.ndarray):
    """(flag_exact, flag_ring): difference non-zero in Z, and non-zero modulo 2^32."""
    d = obs.astype(np.int64) - pred.astype(np.int64)
    return d != 0, np.mod(d, 2 ** 32) != 0


def tau(K: int, max_a: float, max_b: float, rel: float = 1e-3) -> float:
    """Tolerance of the floating-point check: rel * K * max|A| * max|B|."""
    return float(rel) * float(K) * float(max_a) * float(max_b)


def flags_fp(obs: np.ndarray, pred: np.ndarray, tol: float) -> np.ndarray:
    """flag = not(|obs - pred| <= tol); NaN or Inf anywhere in the difference flags."""
    with np.errstate(all="ignore"):
        return ~(np.abs(obs - pred) <= tol)


CLEAN, LOCALISED, CHECKSUM_SUSPECT = 0, 1, 2


def localise(row_flag: np.ndarray, col_flag: np.ndarray):
    """Candidate set E = flagged rows x flagged cols and the status code.

    Flags on one side only cannot come from a single corrupted output element
    (it always disturbs one row sum and one column sum): the checksum itself is
    the suspect then."""
    rows = np.flatnonzero(row_flag)
    cols = np.flatnonzero(col_flag)
    if rows.size == 0 and cols.size == 0:
        return [], CLEAN
    if rows.size == 0 or cols.size == 0:
        return [], CHECKSUM_SUSPECT
    return [(int(i), int(j)) for i in rows for j in cols], LOCALISED


def correct(X: np.ndarray, clean: np.ndarray, E) -> np.ndarray:
    """Replay at element granularity: every element of E takes the recomputed clean value."""
    Y = np.array(X, copy=True)
    for (i, j) in E:
        Y[i, j] = clean[i, j]
    return Y


def correct_by_checksum(X: np.ndarray, cc_obs, rc_obs, cc_pred, rc_pred):
    """Checksum-only correction of the classic scheme the paper builds on (Sec. II-B; the paper
    itself replays, Sec. III-B.3): integers only.  With exactly one row i and one column j
    flagged and the same discrepancy d on both (modulo 2^32), the corrupted element is
    X[i, j] and X[i, j] - d is its value.  Anything else is left alone.

    X: int32 stored output.  Returns (Y, fixed) with fixed in {0, 1}."""
    _, rf = flags_int(rc_obs, rc_pred)
    _, cf = flags_int(cc_obs, cc_pred)
    Y = np.array(X, copy=True)
    if rf.sum() != 1 or cf.sum() != 1:
        return Y, 0
    i, j = int(np.flatnonzero(rf)[0]), int(np.flatnonzero(cf)[0])
    dr = (int(rc_obs[i]) - int(rc_pred[i])) % 2 ** 32
    dc = (int(cc_obs[j]) - int(cc_pred[j])) % 2 ** 32
    if dr != dc:
        return Y, 0
    v = (int(Y[i, j]) - dr) % 2 ** 32
    Y[i, j] = v - 2 ** 32 if v >= 2 ** 31 else v
    return Y, 1


# ----------------------------------------------------------------------------
# one protected GEMM, all steps
# ----------------------------------------------------------------------------
@dataclass
class Protected:
    dtype: str
    C_ref: np.ndarray            # int64 / fp64 exact-accumulation product
    C_stored: np.ndarray         # int32 / uint16 bits
    a: np.ndarray
    b: np.ndarray
    cc_pred: np.ndarray
    rc_pred: np.ndarray
    s_pred: object
    tau: float = 0.0
    max_a: float = 0.0
    max_b: float = 0.0
    extra: dict = field(default_factory=dict)


def with_bias(C_ref, cc_pred, rc_pred, s_pred, bias):
    """A layer with a bias: every row of the output has the bias vector added, so the checksum
    product is adjusted by the bias (Sec. III-B.1 "Checksums": the product of the two input-side
    checksums, adjusted by the layer bias, is what the sum of the activations is compared with).
    Summed over the M rows a column gains M bias[j]; summed over the columns a row gains
    sum_j bias[j]; the scalar gains M sum_j bias[j].  bias: int64 (integer path) or fp64, length N."""
    M = C_ref.shape[0]
    bias = np.asarray(bias, dtype=C_ref.dtype)
    assert bias.shape == (C_ref.shape[1],)
    sb = bias.sum()
    return C_ref + bias[None, :], cc_pred + M * bias, rc_pred + sb, s_pred + M * sb


def protected_gemm(A_bits: np.ndarray, B_bits: np.ndarray, dtype: str, trans_b: bool, bias=None) -> Protected:
    """Run decode, gemm, encode, predict on one (un-batched) pair of stored operands.
    bias: optional length-N vector (int32 values for the integer path, fp32 otherwise) added to
    every row of the product before it is stored."""
    if dtype == "i8":
        A = np.ascontiguousarray(A_bits, dtype=np.int8)
        Bm = np.ascontiguousarray(B_bits, dtype=np.int8)
        C_ref = gemm(A, Bm, trans_b)
        a, b = encode(A, Bm, trans_b)
        cc, rc, s = predict(A, Bm, a, b, trans_b)
        if bias is not None:
            C_ref, cc, rc, s = with_bias(C_ref, cc, rc, s, np.asarray(bias).astype(np.int64))
        return Protected(dtype, C_ref, store(C_ref, dtype), a, b, cc, rc, s)
    A = decode(A_bits, dtype)
    Bm = decode(B_bits, dtype)
    C_ref = gemm(A, Bm, trans_b)
    a, b = encode(A, Bm, trans_b)
    cc, rc, s = predict(A, Bm, a, b, trans_b)
    if bias is not None:
        C_ref, cc, rc, s = with_bias(C_ref, cc, rc, s, np.asarray(bias, dtype=np.float32).astype(np.float64))
    K = A.shape[1]
    ma, mb = float(np.max(np.abs(A))), float(np.max(np.abs(Bm)))
    return Protected(dtype, C_ref, store(C_ref, dtype), a, b, cc, rc, s,
                     tau=tau(K, ma, mb), max_a=ma, max_b=mb)


def check(P: Protected, X_stored: np.ndarray):
    """Observe a stored output (clean or corrupted) and flag it against P's predictions.

    Returns (row_flag, col_flag, E, status, cc_obs, rc_obs)."""
    X = decode_stored(X_stored, P.dtype)
    cc_obs, rc_obs, _ = observe(X)
    if P.dtype == "i8":
        col_exact, col_flag = flags_int(cc_obs, P.cc_pred)
        row_exact, row_flag = flags_int(rc_obs, P.rc_pred)
    else:
        col_flag = flags_fp(cc_obs, P.cc_pred, P.tau)
        row_flag = flags_fp(rc_obs, P.rc_pred, P.tau)
    E, status = localise(row_flag, col_flag)
    return row_flag, col_flag, E, status, cc_obs, rc_obs


STO_TOL_FACTOR = 1e-2


def check_stored(P: Protected, X_stored: np.ndarray):
    """The tightened storage check (floating point): flag a row / column of a stored output when
    its sum differs from the prediction by more than tau (as `check` does) OR from the sum of the
    clean stored output P.C_stored by more than STO_TOL_FACTOR * tau.  Both of the latter are
    sums of rounded values, exact here (fp64), so the difference is the corruption itself;
    the factor leaves room for the fp32 summation order of an implementation.
    (Sec. III-B.1: the sum of the layer's activations is the checked quantity; which reference
    it is compared with is this build's reading, see the list of readings.)

    Returns (row_flag, col_flag, E, status)."""
    assert P.dtype != "i8"
    row_flag, col_flag, _, _, cc_obs, rc_obs = check(P, X_stored)
    cc_sto, rc_sto, _ = observe(decode_stored(P.C_stored, P.dtype))
    col_flag = col_flag | flags_fp(cc_obs, cc_sto, STO_TOL_FACTOR * P.tau)
    row_flag = row_flag | flags_fp(rc_obs, rc_sto, STO_TOL_FACTOR * P.tau)
    E, status = localise(row_flag, col_flag)
    return row_flag, col_flag, E, status


def discrepancy_stats(P: Protected, X_stored: np.ndarray):
    """Statistics of d = observed - predicted over the rows and the columns of a stored output
    (Sec. III-B.1 "Eps Generation": the threshold is read off the fault-free distribution of the
    checksum discrepancy).  Returns {"rows": (sum, sumsq, maxabs, count), "cols": (...)} in fp64."""
    cc_obs, rc_obs, _ = observe(decode_stored(X_stored, P.dtype))
    out = {}
    for name, obs, pred in (("rows", rc_obs, P.rc_pred), ("cols", cc_obs, P.cc_pred)):
        d = np.asarray(obs, dtype=np.float64) - np.asarray(pred, dtype=np.float64)
        out[name] = (float(d.sum()), float((d * d).sum()), float(np.max(np.abs(d))), int(d.size))
    return out


def confidence_z(confidence: float) -> float:
    """Half-width, in standard deviations, of the central interval of a normal distribution that
    holds `confidence` of its mass (0.999 -> 3.2905, 0.9999 -> 3.8906): the confidence levels at
    which the paper reads its thresholds off the fitted discrepancy distribution (Sec. III-B.1
    "Eps Generation", Sec. IV-C)."""
    from statistics import NormalDist
    assert 0.0 < confidence < 1.0
    return NormalDist().inv_cdf(0.5 + 0.5 * confidence)


def calibrated_thresholds(row_stats, col_stats, confidence: float):
    """Eps generation over pooled fault-free runs, one threshold for the row check and one for the
    column check: each is |mean| + z(confidence) * std of the discrepancies of its side, pooled
    over every (sum, sumsq, maxabs, count) tuple given for that side.  Returns (tau_rows, tau_cols)."""
    z = confidence_z(confidence)
    return calibrated_tau(row_stats, z), calibrated_tau(col_stats, z)


def calibrated_tau(stats, z: float) -> float:
    """Threshold at z standard deviations from pooled discrepancy statistics (normal fit, the
    paper's default): |mean| + z * std over every (sum, sumsq, maxabs, count) tuple in `stats`."""
    n = sum(t[3] for t in stats)
    s = sum(t[0] for t in stats)
    s2 = sum(t[1] for t in stats)
    mean = s / n
    var = max(s2 / n - mean * mean, 0.0)
    return abs(mean) + z * var ** 0.5

