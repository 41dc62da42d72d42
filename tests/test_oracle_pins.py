"""Pins for the CPU oracle: it is checked against things other than itself.

Each test names what fixes the expected value: the ring identity
e^T(AB) = (e^T A)B, brute force over all single-bit flips, closed forms,
numpy's int64/float64 matmul and sums as a textbook routine, linearity of the
check in an injected delta, and library conversions for the roundings.
"""
import numpy as np
import pytest
import torch

import abft_inputs as gen
import oracle as orc

pytestmark = []


def _int_case(M, N, K, trans_b, seed):
    A, B = gen.gen_operands("i8", M, N, K, seed, seed + 1, trans_b=trans_b)
    return A[0], B[0]


# ---------------------------------------------------------------- P4: numpy cross-check
@pytest.mark.parametrize("M,N,K,trans_b", [(5, 7, 3, True), (5, 7, 3, False), (33, 17, 65, True),
                                           (64, 48, 32, False), (197, 96, 128, True)])
def test_gemm_i8_matches_numpy_int64(M, N, K, trans_b):
    A, B = _int_case(M, N, K, trans_b, 11)
    Bl = B.T if trans_b else B                      # logical K x N
    want = A.astype(np.int64) @ Bl.astype(np.int64)
    got = orc.gemm(A, B, trans_b)
    assert got.dtype == np.int64 and np.array_equal(got, want)
    a, b = orc.encode(A, B, trans_b)
    assert np.array_equal(a, A.astype(np.int64).sum(axis=0))
    assert np.array_equal(b, Bl.astype(np.int64).sum(axis=1))
    cc, rc, s = orc.predict(A, B, a, b, trans_b)
    assert np.array_equal(cc, a @ Bl.astype(np.int64))
    assert np.array_equal(rc, A.astype(np.int64) @ b)
    assert s == int(a @ b)
    co, ro, so = orc.observe(want)
    assert np.array_equal(co, want.sum(axis=0)) and np.array_equal(ro, want.sum(axis=1)) and so == want.sum()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("trans_b", [True, False])
def test_gemm_fp_matches_numpy_float64(dtype, trans_b):
    M, N, K = 37, 29, 83
    A, B = gen.gen_operands(dtype, M, N, K, 5, 6, trans_b=trans_b)
    Ad, Bd = orc.decode(A[0], dtype), orc.decode(B[0], dtype)
    Bl = Bd.T if trans_b else Bd
    want = Ad @ Bl
    got = orc.gemm(Ad, Bd, trans_b)
    assert np.max(np.abs(got - want)) <= 1e-12 * np.max(np.abs(want))
    a, b = orc.encode(Ad, Bd, trans_b)
    np.testing.assert_allclose(a, Ad.sum(axis=0), rtol=0, atol=1e-12 * M)
    np.testing.assert_allclose(b, Bl.sum(axis=1), rtol=0, atol=1e-12 * N)
    cc, rc, s = orc.predict(Ad, Bd, a, b, trans_b)
    np.testing.assert_allclose(cc, a @ Bl, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(rc, Ad @ b, rtol=1e-12, atol=1e-12)
    assert abs(s - a @ b) <= 1e-12 * max(1.0, abs(s))


# ---------------------------------------------------------------- P1 + P6: integer identity
@pytest.mark.parametrize("M,N,K,trans_b", [(1, 1, 1, True), (3, 4, 5, False), (16, 16, 16, True),
                                           (197, 768, 768, True), (70, 130, 257, False)])
def test_integer_identity_exact_and_in_ring(M, N, K, trans_b):
    A, B = _int_case(M, N, K, trans_b, 1000 + M)
    P = orc.protected_gemm(A, B, "i8", trans_b)
    cc_obs, rc_obs, s_obs = orc.observe(P.C_ref)
    assert np.array_equal(cc_obs, P.cc_pred) and np.array_equal(rc_obs, P.rc_pred)
    assert s_obs == P.s_pred == P.cc_pred.sum() == P.rc_pred.sum()
    rf, cf, E, status, _, _ = orc.check(P, P.C_stored)
    assert not rf.any() and not cf.any() and E == [] and status == orc.CLEAN


def test_integer_identity_holds_through_wraparound():
    # all operands -128: C = K * 2^14; column sums M*K*2^14 exceed 2^32 but the
    # ring identity (and the exact one in int64) still hold.
    M, N, K = 36928, 2, 4096
    A = np.full((M, K), -128, dtype=np.int8)
    B = np.full((N, K), -128, dtype=np.int8)
    P = orc.protected_gemm(A, B, "i8", True)
    assert np.all(P.C_ref == 2 ** 26)
    assert P.cc_pred[0] == M * 2 ** 26 and P.cc_pred[0] >= 2 ** 32
    assert np.all(P.a == -128 * M) and np.all(P.b == -128 * N)
    rf, cf, E, status, cc_obs, _ = orc.check(P, P.C_stored)
    assert status == orc.CLEAN and not rf.any() and not cf.any()
    # a wrapped 32-bit sum of the stored int32 values equals the wrapped prediction
    wrapped = int(P.C_stored.astype(np.int64)[:, 0].sum() % 2 ** 32)
    assert wrapped == int(P.cc_pred[0] % 2 ** 32)


# ---------------------------------------------------------------- P3: closed forms
def test_closed_forms():
    M, N, K = 6, 9, 4
    one = np.ones((M, K), dtype=np.int8)
    Bt = np.ones((N, K), dtype=np.int8)
    P = orc.protected_gemm(one, Bt, "i8", True)
    assert np.all(P.C_ref == K) and np.all(P.cc_pred == M * K) and np.all(P.rc_pred == N * K)
    assert P.s_pred == M * N * K
    # B = identity: C = A, cc = e^T A, rc = A e  (both storage orders of B)
    A = gen.gen_int8((7, 5), 3)
    I = np.eye(5, dtype=np.int8)
    for tb in (True, False):
        P = orc.protected_gemm(A, I, "i8", tb)
        assert np.array_equal(P.C_ref, A.astype(np.int64))
        assert np.array_equal(P.cc_pred, A.astype(np.int64).sum(0))
        assert np.array_equal(P.rc_pred, A.astype(np.int64).sum(1))
    # a single non-zero of A at (2, 3) selects row 3 of logical B into row 2 of C
    A1 = np.zeros((4, 6), dtype=np.int8)
    A1[2, 3] = 5
    Bk = gen.gen_int8((6, 8), 4)              # stored K x N
    P = orc.protected_gemm(A1, Bk, "i8", False)
    want = np.zeros((4, 8), dtype=np.int64)
    want[2] = 5 * Bk[3].astype(np.int64)
    assert np.array_equal(P.C_ref, want)
    # transposed storage of the same logical B gives the same product
    P2 = orc.protected_gemm(A1, np.ascontiguousarray(Bk.T), "i8", True)
    assert np.array_equal(P2.C_ref, want)


def test_softmax_times_ones_closed_form():
    # rows of attn sum to ~1, V = 1  =>  every output ~1, rc ~ N, cc ~ M
    M, N, K = 19, 8, 19
    attn = gen.gen_softmax_bits((M, K), 77, "bf16")
    V = gen.f32_to_bf16_bits(np.ones((K, N), dtype=np.float32))
    P = orc.protected_gemm(attn, V, "bf16", False)
    assert np.max(np.abs(P.C_ref - 1.0)) < 0.02
    assert np.max(np.abs(P.rc_pred - N)) < 0.02 * N and np.max(np.abs(P.cc_pred - M)) < 0.02 * M


# ---------------------------------------------------------------- P2: brute force over every flip
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 4, 5), (5, 7, 3)])
def test_every_single_bit_flip_is_flagged_and_localised(M, N, K):
    A, B = _int_case(M, N, K, True, 42)
    P = orc.protected_gemm(A, B, "i8", True)
    for i in range(M):
        for j in range(N):
            for bit in range(32):
                X = orc.flip(P.C_stored, i, j, bit)
                rf, cf, E, status, cc_obs, rc_obs = orc.check(P, X)
                exact_c, ring_c = orc.flags_int(cc_obs, P.cc_pred)
                assert np.array_equal(exact_c, ring_c)          # same for single flips
                assert status == orc.LOCALISED and E == [(i, j)]
                assert rf.sum() == 1 and cf.sum() == 1
                fixed = orc.correct(X, P.C_stored, E)
                assert np.array_equal(fixed, P.C_stored)


def test_flip_semantics():
    X = np.array([[5, -7]], dtype=np.int32)
    assert orc.flip(X, 0, 0, 1)[0, 0] == 7
    assert orc.flip(X, 0, 0, 31)[0, 0] == 5 - 2 ** 31
    assert orc.flip(X, 0, 1, 31)[0, 1] == -7 + 2 ** 31
    h = np.array([[0x3E00]], dtype=np.uint16)                    # fp16 1.5
    assert orc.decode(h, "f16")[0, 0] == 1.5
    y = orc.decode(orc.flip(h, 0, 0, 14), "f16")[0, 0]            # exponent all ones, mantissa != 0
    assert np.isnan(y)
    assert orc.decode(orc.flip(h, 0, 0, 9), "f16")[0, 0] == 1.0   # top mantissa bit cleared
    bb = np.array([[0x3FC0]], dtype=np.uint16)                    # bf16 1.5
    assert orc.decode(bb, "bf16")[0, 0] == 1.5
    assert orc.decode(orc.flip(bb, 0, 0, 7), "bf16")[0, 0] == 0.75  # lowest exponent bit cleared


def test_two_bit31_flips_in_one_column_escape_the_ring_check_only():
    # documented limit of mod-2^32 checksums: outside the single-error model
    A, B = _int_case(4, 3, 8, True, 9)
    P = orc.protected_gemm(A, B, "i8", True)
    X = orc.flip(orc.flip(P.C_stored, 0, 1, 31), 2, 1, 31)
    cc_obs, _, _ = orc.observe(orc.decode_stored(X, "i8"))
    exact, ring = orc.flags_int(cc_obs, P.cc_pred)
    d = int(cc_obs[1] - P.cc_pred[1])
    assert d % 2 ** 32 == 0 and exact[1] == (d != 0) and not ring[1]


# ---------------------------------------------------------------- P5: fp discrepancy equals the delta
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_fp_discrepancy_equals_injected_delta(dtype):
    M, N, K = 24, 40, 64
    A, B = gen.gen_operands(dtype, M, N, K, 21, 22, trans_b=True)
    P = orc.protected_gemm(A[0], B[0], dtype, True)
    # un-rounded product: identity holds to fp64 rounding
    cc0, rc0, s0 = orc.observe(P.C_ref)
    scale = np.max(np.abs(P.C_ref)) * max(M, N)
    assert np.max(np.abs(cc0 - P.cc_pred)) < 1e-12 * scale
    assert np.max(np.abs(rc0 - P.rc_pred)) < 1e-12 * scale
    assert abs(s0 - P.s_pred) < 1e-11 * scale
    # add delta to one element of the un-rounded product
    i, j, delta = 5, 17, 0.375
    X = P.C_ref.copy()
    X[i, j] += delta
    cc1, rc1, _ = orc.observe(X)
    dc, dr = cc1 - P.cc_pred, rc1 - P.rc_pred
    assert abs(dc[j] - delta) < 1e-10 and abs(dr[i] - delta) < 1e-10
    dc[j] = 0
    dr[i] = 0
    assert np.max(np.abs(dc)) < 1e-10 and np.max(np.abs(dr)) < 1e-10


def test_fp_flags_threshold_nan_and_localisation():
    dtype = "f16"
    M, N, K = 16, 24, 32
    A, B = gen.gen_operands(dtype, M, N, K, 31, 32, trans_b=True)
    P = orc.protected_gemm(A[0], B[0], dtype, True)
    want_tau = 1e-3 * K * np.max(np.abs(orc.decode(A[0], dtype))) * np.max(np.abs(orc.decode(B[0], dtype)))
    assert P.tau == pytest.approx(want_tau, rel=1e-15)
    rf, cf, E, status, _, _ = orc.check(P, P.C_stored)
    assert status == orc.CLEAN
    # exponent flip -> large delta or NaN/Inf: flagged in exactly one row and one column
    for bit in (14, 13):
        X = orc.flip(P.C_stored, 3, 7, bit)
        rf, cf, E, status, _, _ = orc.check(P, X)
        assert status == orc.LOCALISED and E == [(3, 7)]
    # flags_fp: boundary is inclusive, NaN and Inf flag
    obs = np.array([1.0, 1.5, np.nan, np.inf, -np.inf, 0.0])
    pred = np.array([0.5, 0.0, 0.0, 0.0, 0.0, 0.0])
    assert list(orc.flags_fp(obs, pred, 0.5)) == [False, True, True, True, True, False]


def test_one_sided_flags_mean_checksum_suspect():
    assert orc.localise(np.array([0, 1, 0], bool), np.array([0, 0], bool)) == ([], orc.CHECKSUM_SUSPECT)
    assert orc.localise(np.array([0, 0], bool), np.array([1, 0], bool)) == ([], orc.CHECKSUM_SUSPECT)
    E, st = orc.localise(np.array([0, 1, 1], bool), np.array([1, 0, 1], bool))
    assert st == orc.LOCALISED and E == [(1, 0), (1, 2), (2, 0), (2, 2)]


# ---------------------------------------------------------------- roundings against library conversions
def test_round_to_bf16_matches_torch_and_ties_to_even():
    g = np.random.default_rng(3)
    x32 = (g.standard_normal(20000) * np.exp(g.uniform(-30, 30, 20000))).astype(np.float32)
    got = orc.encode_bits(orc.round_to_format(x32.astype(np.float64), "bf16"), "bf16")
    want = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # hand-made ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even (1.0)
    assert orc.round_to_format(np.array([1 + 2.0 ** -8]), "bf16")[0] == 1.0
    assert orc.round_to_format(np.array([1 + 3 * 2.0 ** -8]), "bf16")[0] == 1 + 2.0 ** -6
    assert orc.round_to_format(np.array([1 + 2.0 ** -8 + 2.0 ** -40]), "bf16")[0] == 1 + 2.0 ** -7
    assert np.isinf(orc.round_to_format(np.array([3.4e38]), "bf16")[0])
    # generator's fp32 -> bf16 agrees with torch too (input preparation)
    assert np.array_equal(gen.f32_to_bf16_bits(x32), want)


def test_round_to_f16_matches_numpy_from_double():
    g = np.random.default_rng(4)
    x = g.standard_normal(20000) * np.exp(g.uniform(-20, 12, 20000))
    with np.errstate(over="ignore"):
        want = x.astype(np.float16)
    got = orc.round_to_format(x, "f16")
    assert np.array_equal(got, want.astype(np.float64))
    assert np.array_equal(orc.encode_bits(got, "f16"), want.view(np.uint16))
    assert np.isinf(orc.round_to_format(np.array([65520.0]), "f16")[0])
    assert orc.round_to_format(np.array([65519.9]), "f16")[0] == 65504.0
    assert orc.round_to_format(np.array([2.0 ** -25]), "f16")[0] == 0.0        # tie to even (0)
    assert orc.round_to_format(np.array([2.0 ** -25 * 1.01]), "f16")[0] == 2.0 ** -24


def test_store_int_range_guard_and_values():
    C = np.array([[2 ** 31 - 1, -(2 ** 31) + 1]], dtype=np.int64)
    assert orc.store(C, "i8").dtype == np.int32
    with pytest.raises(AssertionError):
        orc.store(np.array([[2 ** 31]], dtype=np.int64), "i8")


# ---------------------------------------------------------------- P7: what work is counted
def _paper_claims():
    import os
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_claims.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, vals, unit, where = [x.strip() for x in line.split("|")]
            assert where, name                                   # every figure carries its citation
            out[name] = [float(v) for v in vals.split()]
    return out


def test_operation_count_overhead_matches_papers_claim():
    claims = _paper_claims()
    # extra work of the method: encode MK + KN adds, predicted 2K(M+N), observed 2MN
    def ratio(M, N, K):
        return (2 * K * (M + N) + 2 * M * N + M * K + K * N) / (2 * M * N * K)
    assert ratio(12608, 3072, 768) == pytest.approx(0.0019, abs=1e-4)
    assert 100 * ratio(12608, 3072, 768) < claims["compute_overhead_max"][0]     # "< 0.2 %" (abstract)
    # the paper's own counts are consistent with its coverage claim
    missed, total = claims["missed_of_mismatching"]
    assert 100 * (1 - missed / total) > claims["coverage_min"][0]
    # the default tolerance is the one the benchmark spec fixes, 1e-3 K max|A| max|B| (the paper only
    # bounds its calibrated eps, "eps < 1e-3", a different quantity): a hand value and its scaling
    assert orc.tau(768, 5.25, 0.094) == pytest.approx(0.379008, rel=1e-12)
    assert orc.tau(2 * 768, 5.25, 0.094) == pytest.approx(2 * 0.379008, rel=1e-12)
    assert orc.tau(768, 10.5, 0.047) == pytest.approx(0.379008, rel=1e-12)
    assert claims["fixed_point_coverage"][0] == 100          # what the brute-force pin above demonstrates
    for (M, N, K) in [(6304, 2304, 768), (6304, 768, 768), (6304, 3072, 768), (6304, 768, 3072)]:
        assert 0.001 < ratio(M, N, K) < 0.0036


def test_tightened_storage_check_flags_exactly_the_flips_above_its_tolerance():
    """check_stored: a flip of stored C shows in its row and column sum with its full size delta
    (linearity, as in P5), so it must be flagged iff |delta| > 1e-2 tau (or non-finite), also
    where the plain check (tolerance tau) stays silent; the clean output never flags."""
    dtype = "bf16"
    M, N, K = 40, 48, 64
    A, B = gen.gen_operands(dtype, M, N, K, 41, 42, trans_b=True)
    P = orc.protected_gemm(A[0], B[0], dtype, True)
    rf, cf, E, status = orc.check_stored(P, P.C_stored)
    assert status == orc.CLEAN and not rf.any() and not cf.any()
    clean = orc.decode(P.C_stored, dtype)
    seen_small = seen_mid = 0
    for bit in range(15):
        for (i, j) in ((0, 0), (17, 5), (39, 47)):
            X = orc.flip(P.C_stored, i, j, bit)
            with np.errstate(all="ignore"):
                delta = abs(orc.decode(X, dtype)[i, j] - clean[i, j])
            rf, cf, E, status = orc.check_stored(P, X)
            rf0, cf0, _, status0, _, _ = orc.check(P, X)
            big = not (delta <= orc.STO_TOL_FACTOR * P.tau)
            if big:
                assert status == orc.LOCALISED and E == [(i, j)], (bit, i, j, delta)
            else:
                assert status == orc.CLEAN
                seen_small += 1
            if big and delta <= P.tau * 0.5:
                assert status0 == orc.CLEAN          # the plain check cannot see it
                seen_mid += 1
            assert (rf | rf0 == rf).all() and (cf | cf0 == cf).all()   # never weaker than the plain check
    assert seen_small > 0 and seen_mid > 0


def test_discrepancy_statistics_and_calibrated_threshold_closed_forms():
    """discrepancy_stats on a case with known discrepancies: shift the predictions of a clean
    protected GEMM by constants c_r, c_c; then d = (clean d) + c exactly, so sum, sum of squares
    and max follow in closed form from the unshifted statistics.  calibrated_tau on statistics
    built from a known mean and spread returns |mean| + z * std."""
    dtype = "f16"
    M, N, K = 24, 40, 32
    A, B = gen.gen_operands(dtype, M, N, K, 51, 52, trans_b=True)
    P = orc.protected_gemm(A[0], B[0], dtype, True)
    st0 = orc.discrepancy_stats(P, P.C_stored)
    assert st0["rows"][3] == M and st0["cols"][3] == N
    # clean discrepancies are the roundings of the stored values summed up: far below tau
    assert st0["rows"][2] < P.tau and st0["cols"][2] < P.tau
    cr, cc = 0.75, -1.25
    import copy
    Q = copy.copy(P)
    Q.rc_pred = P.rc_pred - cr
    Q.cc_pred = P.cc_pred - cc
    st1 = orc.discrepancy_stats(Q, P.C_stored)
    for name, c, n in (("rows", cr, M), ("cols", cc, N)):
        s0, q0, _, _ = st0[name]
        s1, q1, m1, n1 = st1[name]
        assert n1 == n
        assert s1 == pytest.approx(s0 + n * c, rel=1e-12, abs=1e-12)
        assert q1 == pytest.approx(q0 + 2 * c * s0 + n * c * c, rel=1e-12, abs=1e-12)
        assert abs(m1 - abs(c)) <= st0[name][2] + 1e-12
    # a population of n values mean mu, variance v: sum = n mu, sumsq = n (v + mu^2)
    mu, v, n = -0.02, 0.0009, 1000
    tau = orc.calibrated_tau([(n * mu, n * (v + mu * mu), 0.2, n)], z=4.0)
    assert tau == pytest.approx(0.02 + 4.0 * 0.03, rel=1e-12)
    # pooling two groups equals one group with the sums added
    t2 = orc.calibrated_tau([(1.0, 3.0, 1.0, 10), (-2.0, 5.0, 1.5, 30)], z=2.0)
    t1 = orc.calibrated_tau([(-1.0, 8.0, 1.5, 40)], z=2.0)
    assert t2 == pytest.approx(t1, rel=1e-15)



# ---------------------------------------------------------------- checksum-only correction
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 4, 5), (5, 7, 3)])
def test_checksum_only_correction_restores_every_single_bit_flip(M, N, K):
    """The truth it is pinned to is the clean output itself: for every element and every bit, the
    corrected matrix must be bit-identical to the undisturbed one (a wrong sign of d, a swapped
    row/column index or a missing wrap-around fails this)."""
    A, B = _int_case(M, N, K, True, 43)
    P = orc.protected_gemm(A, B, "i8", True)
    for i in range(M):
        for j in range(N):
            for bit in range(32):
                X = orc.flip(P.C_stored, i, j, bit)
                _, _, _, _, cc_obs, rc_obs = orc.check(P, X)
                Y, fixed = orc.correct_by_checksum(X, cc_obs, rc_obs, P.cc_pred, P.rc_pred)
                assert fixed == 1 and np.array_equal(Y, P.C_stored) and Y.dtype == np.int32


def test_checksum_only_correction_leaves_what_it_cannot_explain():
    A, B = _int_case(6, 5, 16, True, 44)
    P = orc.protected_gemm(A, B, "i8", True)
    # two errors in different rows and columns: two flags on each side
    X = orc.flip(orc.flip(P.C_stored, 1, 2, 5), 4, 0, 9)
    _, _, _, _, cc_obs, rc_obs = orc.check(P, X)
    Y, fixed = orc.correct_by_checksum(X, cc_obs, rc_obs, P.cc_pred, P.rc_pred)
    assert fixed == 0 and np.array_equal(Y, X)
    # one flagged row and column whose discrepancies disagree (a checksum word was hit as well)
    X = orc.flip(P.C_stored, 3, 3, 12)
    _, _, _, _, cc_obs, rc_obs = orc.check(P, X)
    cc_bad = cc_obs.copy()
    cc_bad[3] += 1
    Y, fixed = orc.correct_by_checksum(X, cc_bad, rc_obs, P.cc_pred, P.rc_pred)
    assert fixed == 0 and np.array_equal(Y, X)
    # clean
    _, _, _, _, cc_obs, rc_obs = orc.check(P, P.C_stored)
    Y, fixed = orc.correct_by_checksum(P.C_stored, cc_obs, rc_obs, P.cc_pred, P.rc_pred)
    assert fixed == 0 and np.array_equal(Y, P.C_stored)


# ---------------------------------------------------------------- a fault in the weight, after its checksum was taken
def test_weight_fault_after_encoding_shows_on_the_row_side_only():
    """b = B e is taken from the clean weight (the offline checksum of Sec. III-B.1, remark (2));
    then one element B[j, k] changes by delta.  Every row i of C moves by A[i, k] * delta in
    column j, so the row discrepancy is exactly A[i, k] * delta; the column prediction a B is
    formed from the weight as it is now and stays consistent with C: no column is flagged."""
    M, N, K = 9, 7, 12
    A, B = _int_case(M, N, K, True, 77)
    a, b_clean = orc.encode(A, B, True)
    j, k, bit = 3, 5, 6
    B2 = B.copy()
    B2[j, k] = np.int8(np.uint8(B2[j, k]) ^ np.uint8(1 << bit))
    delta = int(B2[j, k]) - int(B[j, k])
    C2 = orc.gemm(A, B2, True)
    cc_pred, rc_pred, _ = orc.predict(A, B2, a, b_clean, True)
    cc_obs, rc_obs, _ = orc.observe(C2)
    assert np.array_equal(cc_obs, cc_pred)
    assert np.array_equal(rc_obs - rc_pred, A[:, k].astype(np.int64) * delta)
    _, rf = orc.flags_int(rc_obs, rc_pred)
    _, cf = orc.flags_int(cc_obs, cc_pred)
    assert np.array_equal(rf, A[:, k] != 0) and not cf.any()
    E, status = orc.localise(rf, cf)
    assert E == [] and status == orc.CHECKSUM_SUSPECT


# ------------------------------------------------------------------ bias, operand flips, confidence levels
@pytest.mark.parametrize("dtype", ["i8", "bf16"])
def test_bias_moves_every_checksum_by_its_closed_form(dtype):
    """Sec. III-B.1 "Checksums": the checked product is adjusted by the layer bias.  Closed forms:
    a constant bias c moves every element by c, every column sum by M c, every row sum by N c
    and the scalar by M N c; a general bias moves column j by M bias[j] and every row by
    sum(bias); with A = 0 the output is the bias in every row; and the identity observed ==
    predicted still holds (exactly for integers)."""
    M, N, K = 9, 14, 24
    A, B = gen.gen_operands(dtype, M, N, K, 71, 72, trans_b=True)
    P0 = orc.protected_gemm(A[0], B[0], dtype, True)
    c = 3
    Pc = orc.protected_gemm(A[0], B[0], dtype, True, bias=np.full(N, c))
    assert np.array_equal(Pc.C_ref, P0.C_ref + c)
    assert np.allclose(Pc.cc_pred, P0.cc_pred + M * c, rtol=0, atol=1e-9)
    assert np.allclose(Pc.rc_pred, P0.rc_pred + N * c, rtol=0, atol=1e-9)
    assert abs(Pc.s_pred - (P0.s_pred + M * N * c)) <= 1e-9
    rng = np.random.default_rng(5)
    bias = rng.integers(-1000, 1000, N) if dtype == "i8" else rng.standard_normal(N).astype(np.float32)
    Pb = orc.protected_gemm(A[0], B[0], dtype, True, bias=bias)
    bw = np.asarray(bias, dtype=np.int64 if dtype == "i8" else np.float64)
    for j in range(N):
        assert np.allclose(Pb.C_ref[:, j], P0.C_ref[:, j] + bw[j], rtol=0, atol=1e-12)
    # library cross-check of the adjusted checksums and the identity on the product itself
    assert np.allclose(Pb.cc_pred, Pb.C_ref.sum(axis=0), rtol=1e-12, atol=1e-9)
    assert np.allclose(Pb.rc_pred, Pb.C_ref.sum(axis=1), rtol=1e-12, atol=1e-9)
    cc_obs, rc_obs, s_obs = orc.observe(Pb.C_ref)
    if dtype == "i8":
        assert np.array_equal(cc_obs, Pb.cc_pred) and np.array_equal(rc_obs, Pb.rc_pred) and s_obs == Pb.s_pred
        rf, cf, E, status, _, _ = orc.check(Pb, Pb.C_stored)
        assert status == orc.CLEAN and not rf.any() and not cf.any()
    # A = 0: the output is the bias, row by row
    Z = np.zeros_like(A[0])
    Pz = orc.protected_gemm(Z, B[0], dtype, True, bias=bias)
    assert np.array_equal(Pz.C_ref, np.tile(bw, (M, 1)))
    # a dropped bias term would be caught: the adjusted prediction differs from the plain one
    assert not np.allclose(Pb.rc_pred, P0.rc_pred) and not np.allclose(Pb.cc_pred, P0.cc_pred)


def test_operand_flips_move_one_row_or_one_column_of_the_product():
    """Flips in inputs and weights (the other injection sites of Sec. II-A / III-A).  Linearity:
    a flip of A[i,k] by delta moves row i of C by delta B[k,:] and nothing else; a flip of the
    stored weight W[n,k] by delta moves column n of C by delta A[:,k].  Against checksums taken
    before the flip: an A flip shows in the column check wherever delta B[k,j] != 0 and in row i
    iff delta b[k] != 0; a weight flip shows in the row check wherever delta A[i,k] != 0 and in
    column n iff delta a[k] != 0."""
    M, N, K = 7, 9, 16
    A, B = gen.gen_operands("i8", M, N, K, 81, 82, trans_b=True)
    A, B = A[0], B[0]
    P = orc.protected_gemm(A, B, "i8", True)
    rng = np.random.default_rng(9)
    for _ in range(20):
        i, k, n, bit = int(rng.integers(M)), int(rng.integers(K)), int(rng.integers(N)), int(rng.integers(8))
        A2 = orc.flip(A, i, k, bit)
        dA = int(A2[i, k]) - int(A[i, k])
        assert dA in (1 << bit, -(1 << bit)) or (bit == 7 and abs(dA) == 128)
        C2 = orc.gemm(A2, B, True)
        want = P.C_ref.copy()
        want[i, :] += dA * B[:, k].astype(np.int64)
        assert np.array_equal(C2, want)
        rf, cf, E, status, _, _ = orc.check(P, orc.store(C2, "i8"))
        assert np.array_equal(cf, dA * B[:, k].astype(np.int64) != 0)
        assert not rf.any() or rf[i]
        assert rf.sum() == (1 if dA * int(P.b[k]) != 0 else 0)
        B2 = orc.flip(B, n, k, bit)
        dB = int(B2[n, k]) - int(B[n, k])
        C3 = orc.gemm(A, B2, True)
        want = P.C_ref.copy()
        want[:, n] += dB * A[:, k].astype(np.int64)
        assert np.array_equal(C3, want)
        rf, cf, E, status, _, _ = orc.check(P, orc.store(C3, "i8"))
        assert np.array_equal(rf, dB * A[:, k].astype(np.int64) != 0)
        assert cf.sum() == (1 if dB * int(P.a[k]) != 0 else 0) and (not cf.any() or cf[n])
    # 16-bit operands: the flipped pattern decodes to the hand value
    X = np.array([[0x3FC0]], dtype=np.uint16)                    # bf16 1.5
    assert np.isnan(orc.decode(orc.flip(X, 0, 0, 14), "bf16")[0, 0])     # exponent all ones, mantissa not zero
    assert orc.decode(orc.flip(X, 0, 0, 7), "bf16")[0, 0] == 0.75
    assert orc.decode(orc.flip(X, 0, 0, 6), "bf16")[0, 0] == 1.0


def test_confidence_levels_and_separate_thresholds():
    """Eps generation at the paper's confidence levels: textbook normal quantiles (two-sided
    99.9 % -> 3.2905, 99.99 % -> 3.8906, 95 % -> 1.9600), and row / column thresholds fitted
    separately from pooled statistics in closed form."""
    assert orc.confidence_z(0.95) == pytest.approx(1.959964, abs=1e-5)
    assert orc.confidence_z(0.999) == pytest.approx(3.290527, abs=1e-5)
    assert orc.confidence_z(0.9999) == pytest.approx(3.890592, abs=1e-5)
    # rows: discrepancies {+1, -1} x 50 over two runs -> mean 0, std 1; columns: all equal 2 -> std 0
    rows = [(0.0, 50.0, 1.0, 50), (0.0, 50.0, 1.0, 50)]
    cols = [(40.0, 80.0, 2.0, 20)]
    tr, tc = orc.calibrated_thresholds(rows, cols, 0.999)
    assert tr == pytest.approx(3.290527, abs=1e-5)
    assert tc == pytest.approx(2.0, abs=1e-12)
    # pooling is over counts, not over runs: a run with ten times the entries weighs ten times
    rows2 = [(0.0, 0.0, 0.0, 900), (0.0, 100.0, 1.0, 100)]
    assert orc.calibrated_tau(rows2, 1.0) == pytest.approx(np.sqrt(0.1), rel=1e-12)
