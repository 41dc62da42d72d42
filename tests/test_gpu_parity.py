"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, element by
element on the same seeded inputs.

Bars: integer C, checksums (in Z/2^32), flags and counts bit-exact; bf16/fp16 C within 1e-2 of
max|C_ref| (and within one rounding of the storage type element-wise); fp32 checksums within a
small fraction of the tolerance tau = 1e-3 K max|A| max|B|; flags equal except for flips whose
|delta| lies within a factor two of tau."""
import numpy as np
import pytest
import torch

import abft_inputs as gen
import oracle as orc
import paper_2310_03841_amd as ab
from abft_harness import Run

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = ab.abft_create(max_rows=16384, max_cols=16384, max_depth=16384, max_batch=16)
    yield c
    ab.abft_destroy(c)


@pytest.fixture(scope="module")
def ctx_big():
    c = ab.abft_create(max_rows=12608, max_cols=3072, max_depth=3072, max_batch=1)
    yield c
    ab.abft_destroy(c)


def ring(x):
    return np.mod(np.asarray(x, dtype=np.int64), 2 ** 32).astype(np.uint32)


def oracle_items(dtype, A, B, trans_b):
    return [orc.protected_gemm(A[b], B[b], dtype, trans_b) for b in range(A.shape[0])]


def check_clean(run: Run, P, fused=True):
    """C, checksums, flags and counts of a clean protected GEMM against the oracle items P."""
    C = run.C()
    rf, cf = run.flags()
    cnt = run.cnt()
    a = run.ws(ab.ABFT_WS_A_SUM)
    b = run.ws(ab.ABFT_WS_B_SUM)
    ccp, rcp = run.ws(ab.ABFT_WS_CC_PRED), run.ws(ab.ABFT_WS_RC_PRED)
    cco, rco = run.ws(ab.ABFT_WS_CC_OBS), run.ws(ab.ABFT_WS_RC_OBS)
    sp = run.ws(ab.ABFT_WS_S_PRED)
    for bi, p in enumerate(P):
        if run.dtype == "i8":
            assert np.array_equal(C[bi], p.C_stored), f"C differs (batch {bi})"
            assert np.array_equal(a[bi].view(np.uint32), ring(p.a))
            assert np.array_equal(b[bi].view(np.uint32), ring(p.b))
            assert np.array_equal(ccp[bi].view(np.uint32), ring(p.cc_pred))
            assert np.array_equal(rcp[bi].view(np.uint32), ring(p.rc_pred))
            assert np.array_equal(cco[bi].view(np.uint32), ring(p.cc_pred))     # identity: obs == pred
            assert np.array_equal(rco[bi].view(np.uint32), ring(p.rc_pred))
            assert sp[bi, 0].view(np.uint32) == ring(p.s_pred)
        else:
            Cg = orc.decode(C[bi], run.dtype)
            scale = np.max(np.abs(p.C_ref))
            assert np.max(np.abs(Cg - p.C_ref)) <= 1e-2 * scale
            ulp = 2.0 ** -8 if run.dtype == "bf16" else 2.0 ** -11
            assert np.all(np.abs(Cg - p.C_ref) <= ulp * np.abs(p.C_ref) + 2e-6 * scale + 1e-7)
            # round-to-nearest-even from an fp32 accumulator: the stored bits equal the oracle's
            # rounding of the exact product except where fp32 noise crosses a rounding boundary
            assert np.sum(C[bi] != p.C_stored) <= max(2, 5e-3 * C[bi].size)     # small outputs: two crossings
            tol = 1e-2 * p.tau
            K = run.K
            assert np.max(np.abs(a[bi] - p.a)) <= 1e-5 * run.M * p.max_a
            assert np.max(np.abs(b[bi] - p.b)) <= 1e-5 * run.N * p.max_b
            assert np.max(np.abs(ccp[bi] - p.cc_pred)) <= tol * max(1.0, np.sqrt(run.M))
            assert np.max(np.abs(rcp[bi] - p.rc_pred)) <= tol * max(1.0, np.sqrt(run.N))
            cc0, rc0, _ = orc.observe(p.C_ref)
            assert np.max(np.abs(cco[bi] - cc0)) <= tol * max(1.0, np.sqrt(run.M))
            assert np.max(np.abs(rco[bi] - rc0)) <= tol * max(1.0, np.sqrt(run.N))
            assert abs(sp[bi, 0] - p.s_pred) <= 1e-4 * K * run.M * run.N * p.max_a * p.max_b
            tau_g = run.ws(ab.ABFT_WS_TAU)[bi, 0]
            assert tau_g == pytest.approx(p.tau, rel=1e-5)
    assert not rf.any() and not cf.any()
    assert cnt[0] == 0 and cnt[1] == 0 and cnt[2] == ab.ABFT_CLEAN


SHAPES = [
    # (M, N, K, batch, trans_b)
    (197, 768, 768, 1, True),      # ViT-B projection at batch 1 (the small configuration)
    (300, 200, 264, 1, True),      # several tiles, ragged M/N, ragged K slab
    (257, 130, 72, 2, True),
    (128, 128, 128, 1, True),      # tile-exact
    (1, 1, 1, 1, True),
    (197, 197, 64, 3, True),       # per-head Q K^T
    (197, 64, 197, 3, False),      # per-head attn V (B stored K x N)
    (150, 200, 136, 2, False),
    (777, 600, 192, 1, True),      # 256x256-tile path for 16-bit types (K a multiple of 64)
    (520, 1030, 256, 2, True),     # 256x256-tile path for all types, ragged both ways, batched
    (512, 512, 128, 1, True),      # tile-exact on the 256x256 path
    (520, 600, 4096, 1, True),     # deepest K of a protected GEMM: 16 / 32 slabs per workgroup to reduce
    (600, 512, 640, 1, True),      # two tile columns: a workgroup reduces every other slab of its tile row
    (520, 1300, 1152, 1, True),    # six tile columns, a ragged last one: owned slabs three (int8: one or two) apart
    (140, 90, 4096, 1, False),     # the same on the general kernel
]


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", SHAPES)
def test_clean_gemm_matches_oracle(ctx, dtype, M, N, K, batch, trans_b):
    _clean_case(ctx, dtype, M, N, K, batch, trans_b)


def _clean_case(ctx, dtype, M, N, K, batch, trans_b):
    a_kind = "softmax" if (not trans_b and dtype != "i8") else "act"
    A, B = gen.gen_operands(dtype, M, N, K, 101 + M, 202 + N, trans_b=trans_b, batch=batch,
                            a_kind=a_kind, b_kind="weight" if batch == 1 else "act")
    print(f"case dtype={dtype} M={M} N={N} K={K} batch={batch} trans_b={trans_b}", flush=True)
    run = Run(ctx, dtype, A, B, trans_b)
    P = oracle_items(dtype, A, B, trans_b)
    run.gemm(ab.ABFT_DETECT)
    check_clean(run, P)
    C_prot = run.C().copy()
    # unprotected mode: the same C, bit for bit
    run.dC.fill_(0)
    run.gemm(ab.ABFT_OFF)
    assert np.array_equal(run.C(), C_prot)
    # pad columns of C (between N and ldc) are never written
    if run.ldc != run.N:
        run.dC.fill_(0x1111)
        run.gemm(ab.ABFT_DETECT)
        pad = run.dC.cpu().numpy()[:, :, run.N:]
        assert np.all(pad == 0x1111)


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
def test_cached_b_checksum(ctx, dtype):
    M, N, K = 200, 136, 320
    A, B = gen.gen_operands(dtype, M, N, K, 7, 8, trans_b=True)
    A2, _ = gen.gen_operands(dtype, M, N, K, 9, 8, trans_b=True)
    run = Run(ctx, dtype, A, B, True)
    assert ab.abft_encode_b(ctx, run.dB, run.code, run.shape) == ab.ABFT_OK
    run.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)
    check_clean(run, oracle_items(dtype, A, B, True))
    run2 = Run(ctx, dtype, A2, B, True)
    run2.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)     # B encoding left by the previous call
    check_clean(run2, oracle_items(dtype, A2, B, True))


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(197, 768, 768, 1, True), (130, 70, 100, 2, False),
                                                  (600, 520, 256, 1, True)])
def test_stored_flip_verify_correct(ctx, dtype, M, N, K, batch, trans_b):
    A, B = gen.gen_operands(dtype, M, N, K, 31, 32, trans_b=trans_b, batch=batch)
    run = Run(ctx, dtype, A, B, trans_b)
    P = oracle_items(dtype, A, B, trans_b)
    run.gemm(ab.ABFT_DETECT)
    C_clean = run.C().copy()
    run.verify()
    rf, cf = run.flags()
    assert not rf.any() and not cf.any() and run.cnt()[2] == ab.ABFT_CLEAN
    flips = gen.gen_flips(40, M, N, dtype, 555, batch=batch)
    n_border = 0
    for (bi, i, j, bit) in flips:
        bi, i, j, bit = int(bi), int(i), int(j), int(bit)
        print(f"flip dtype={dtype} b={bi} i={i} j={j} bit={bit}", flush=True)
        run.inject(bi, i, j, bit)
        run.verify()
        rf, cf = run.flags()
        cnt = run.cnt()
        X = orc.flip(P[bi].C_stored, i, j, bit)
        orf, ocf, E, status, _, _ = orc.check(P[bi], X)
        if dtype == "i8":
            assert np.array_equal(run.C()[bi], X)
        else:
            with np.errstate(all="ignore"):
                delta = abs(orc.decode(X, dtype)[i, j] - orc.decode(P[bi].C_stored, dtype)[i, j])
            if P[bi].tau / 2 <= delta <= 2 * P[bi].tau:
                n_border += 1
                run.dC.copy_(torch.from_numpy(_with_ld(C_clean, run)).to("cuda"))
                continue
        want_rf = np.zeros((batch, M), bool)
        want_cf = np.zeros((batch, N), bool)
        want_rf[bi], want_cf[bi] = orf, ocf
        assert np.array_equal(rf, want_rf) and np.array_equal(cf, want_cf)
        assert cnt[0] == orf.sum() and cnt[1] == ocf.sum() and cnt[2] == status
        if dtype == "i8":
            assert status == orc.LOCALISED and E == [(i, j)]
        run.correct()
        rf, cf = run.flags()
        cnt = run.cnt()
        if status == orc.LOCALISED:
            assert cnt[3] == 1 and cnt[4] == ab.ABFT_LOCALISED
            assert np.array_equal(run.C(), C_clean), "C not restored"
            assert not rf.any() and not cf.any() and cnt[2] == ab.ABFT_CLEAN
        else:                                       # flip below tolerance: undetected, restore by hand
            assert status == orc.CLEAN and dtype != "i8" and cnt[3] == 0
            run.dC.copy_(torch.from_numpy(_with_ld(C_clean, run)).to("cuda"))
    assert n_border <= len(flips) // 2


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(600, 520, 256, 1, True), (197, 768, 768, 1, True),
                                                  (130, 70, 100, 2, False)])
def test_tightened_storage_check(ctx, dtype, M, N, K, batch, trans_b):
    _tightened_storage_case(ctx, dtype, M, N, K, batch, trans_b)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(70, 50, 40, 64, False), (100, 130, 72, 65, True),
                                                 (197, 197, 64, 64, True)])
def test_tightened_storage_check_item_kernel(ctx_items, dtype, M, N, K, batch, trans_b):
    _tightened_storage_case(ctx_items, dtype, M, N, K, batch, trans_b)


def _tightened_storage_case(ctx, dtype, M, N, K, batch, trans_b):
    """ABFT_STORED_SUMS: the epilogue's sums of the rounded values equal the oracle's sums of the
    stored clean C; verify then flags stored flips down to 1e-2 tau, as the oracle's check_stored."""
    A, B = gen.gen_operands(dtype, M, N, K, 61, 62, trans_b=trans_b, batch=batch)
    run = Run(ctx, dtype, A, B, trans_b)
    P = oracle_items(dtype, A, B, trans_b)
    run.gemm(ab.ABFT_DETECT | ab.ABFT_STORED_SUMS)
    assert run.cnt()[2] == ab.ABFT_CLEAN
    C_clean = run.C().copy()
    cc_sto, rc_sto = run.ws(ab.ABFT_WS_CC_STO), run.ws(ab.ABFT_WS_RC_STO)
    for bi in range(batch):
        # expected: the sums of the oracle's stored C.  The device's stored C may differ from it in
        # a few last-place roundings (fp32 noise on a rounding boundary): what those differences
        # add up to per column / row is allowed on top of the fp32 summation noise.
        Xo = orc.decode_stored(P[bi].C_stored, dtype)
        cc, rc, _ = orc.observe(Xo)
        miss = np.abs(orc.decode_stored(C_clean[bi], dtype) - Xo)
        assert np.count_nonzero(miss) <= 0.005 * miss.size
        tol = 1e-2 * orc.STO_TOL_FACTOR * P[bi].tau
        assert np.all(np.abs(cc_sto[bi] - cc) <= miss.sum(axis=0) + tol * np.sqrt(M))
        assert np.all(np.abs(rc_sto[bi] - rc) <= miss.sum(axis=1) + tol * np.sqrt(N))
    run.verify()
    rf, cf = run.flags()
    assert not rf.any() and not cf.any() and run.cnt()[2] == ab.ABFT_CLEAN
    flips = gen.gen_flips(40, M, N, dtype, 777, batch=batch)
    n_border = n_tight_only = 0
    for (bi, i, j, bit) in flips:
        bi, i, j, bit = int(bi), int(i), int(j), int(bit)
        print(f"flip dtype={dtype} b={bi} i={i} j={j} bit={bit}", flush=True)
        Xc = P[bi].C_stored
        X = orc.flip(Xc, i, j, bit)
        with np.errstate(all="ignore"):
            delta = abs(orc.decode(X, dtype)[i, j] - orc.decode(Xc, dtype)[i, j])
        orf, ocf, E, status = orc.check_stored(P[bi], X)
        t_sto = orc.STO_TOL_FACTOR * P[bi].tau
        if t_sto / 2 <= delta <= 2 * t_sto or P[bi].tau / 2 <= delta <= 2 * P[bi].tau:
            n_border += 1
            continue
        run.inject(bi, i, j, bit)
        run.verify()
        rf, cf = run.flags()
        cnt = run.cnt()
        big = status == orc.LOCALISED
        want_rf = np.zeros((batch, M), bool)
        want_cf = np.zeros((batch, N), bool)
        want_rf[bi], want_cf[bi] = orf, ocf
        if big:
            assert E == [(i, j)]
            n_tight_only += int(delta <= P[bi].tau / 2)
        assert np.array_equal(rf, want_rf) and np.array_equal(cf, want_cf), (bit, delta, t_sto)
        assert cnt[0] == orf.sum() and cnt[1] == ocf.sum() and cnt[2] == status
        run.correct()
        if big:
            cnt = run.cnt()
            assert cnt[3] == 1 and cnt[2] == ab.ABFT_CLEAN
            assert np.array_equal(run.C(), C_clean), "C not restored"
        else:
            run.dC.copy_(torch.from_numpy(_with_ld(C_clean, run)).to("cuda"))
    assert n_border <= len(flips) // 2 and n_tight_only > 0


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(600, 520, 256, 2, True), (197, 197, 64, 3, True)])
def test_discrepancy_statistics(ctx, dtype, M, N, K, batch, trans_b):
    """abft_discrepancy (source: re-sum of stored C) against the oracle's discrepancy_stats of its
    own stored C; a threshold calibrated from them flags nothing on the clean output."""
    A, B = gen.gen_operands(dtype, M, N, K, 91, 92, trans_b=trans_b, batch=batch)
    run = Run(ctx, dtype, A, B, trans_b)
    P = oracle_items(dtype, A, B, trans_b)
    stats = torch.zeros((batch, 8), dtype=torch.float32, device="cuda")
    run.gemm(ab.ABFT_DETECT)
    assert ab.abft_discrepancy(ctx, run.code, run.shape, ab.ABFT_DISC_STORED, stats) == ab.ABFT_ESTATE
    run.verify()
    assert ab.abft_discrepancy(ctx, run.code, run.shape, ab.ABFT_DISC_STORED, stats) == ab.ABFT_OK
    torch.cuda.synchronize()
    got = stats.cpu().numpy().astype(np.float64)
    C_dev = run.C()
    pooled = []
    for bi in range(batch):
        want = orc.discrepancy_stats(P[bi], P[bi].C_stored)
        # the device's stored C may differ from the oracle's in a few last-place roundings: their
        # total mass bounds how far the sums of d may drift; fp32 summation noise on top
        miss = np.abs(orc.decode_stored(C_dev[bi], dtype) - orc.decode_stored(P[bi].C_stored, dtype))
        assert np.count_nonzero(miss) <= 0.005 * miss.size
        drift = miss.sum() + 1e-3 * P[bi].tau
        for side, off in (("rows", 0), ("cols", 4)):
            s0, q0, m0, n0 = want[side]
            assert got[bi, off + 3] == n0
            assert abs(got[bi, off] - s0) <= drift
            rms_w, rms_g = np.sqrt(q0 / n0), np.sqrt(got[bi, off + 1] / n0)
            assert abs(rms_g - rms_w) <= 0.2 * rms_w + drift / n0
            slack = miss.max() * max(M, N) + 1e-3 * P[bi].tau
            assert m0 - slack <= got[bi, off + 2] <= m0 + slack
            pooled.append((got[bi, off], got[bi, off + 1], got[bi, off + 2], n0))
    # source FUSED: sums of the accumulators before rounding: fp32 noise only, far below the above
    assert ab.abft_discrepancy(ctx, run.code, run.shape, ab.ABFT_DISC_FUSED, stats) == ab.ABFT_OK
    torch.cuda.synchronize()
    fused = stats.cpu().numpy()
    assert np.all(fused[:, 2] < 1e-2 * P[0].tau) and np.all(fused[:, 6] < 1e-2 * P[0].tau)
    # a threshold at 6 standard deviations of the stored-side discrepancies covers every clean
    # discrepancy seen, and the clean output passes a verify under it
    tau_cal = orc.calibrated_tau(pooled, z=6.0)
    assert max(t[2] for t in pooled) < tau_cal
    if K >= 256:
        assert tau_cal < min(p.tau for p in P)      # deep K: tighter than the analytic tolerance
    run.tau = float(tau_cal)
    run.verify()
    assert run.cnt()[2] == ab.ABFT_CLEAN
    run.tau = 0.0
    i8 = ab.make_shape(64, 64, 64)
    assert ab.abft_discrepancy(ctx, ab.ABFT_I8, i8, ab.ABFT_DISC_FUSED, stats) == ab.ABFT_EINVAL


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_thresholds_calibrated_over_pooled_clean_runs(ctx, dtype):
    """Eps generation as the paper states it (Sec. III-B.1 "Eps Generation", Sec. IV-C): the
    discrepancies of fault-free seeded runs of one layer shape are pooled, rows and columns are
    fitted separately, and the thresholds are read off at a confidence level.  Pooled device
    statistics against the oracle's; then the two thresholds go into the checks: flips between the
    calibrated and the analytic tolerance are seen only under the calibrated ones, the row check
    and the column check each obey their own threshold, and clean outputs stay (nearly) clean."""
    M, N, K, runs = 300, 1030, 256, 12
    _, B = gen.gen_operands(dtype, M, N, K, 501, 502, trans_b=True)
    stats = torch.zeros((1, 8), dtype=torch.float32, device="cuda")
    rows_g, cols_g, rows_o, cols_o = [], [], [], []
    last = None
    for r in range(runs):
        A, _ = gen.gen_operands(dtype, M, N, K, 600 + r, 502, trans_b=True)
        run = Run(ctx, dtype, A, B, True)
        run.gemm(ab.ABFT_DETECT)
        run.verify()
        assert ab.abft_discrepancy(ctx, run.code, run.shape, ab.ABFT_DISC_STORED, stats) == ab.ABFT_OK
        torch.cuda.synchronize()
        g = stats.cpu().numpy().astype(np.float64)[0]
        rows_g.append(tuple(g[0:4]))
        cols_g.append(tuple(g[4:8]))
        P = orc.protected_gemm(A[0], B[0], dtype, True)
        want = orc.discrepancy_stats(P, P.C_stored)
        rows_o.append(want["rows"])
        cols_o.append(want["cols"])
        last = (run, P)
    for conf in (0.999, 0.9999):
        tr_g, tc_g = orc.calibrated_thresholds(rows_g, cols_g, conf)
        tr_o, tc_o = orc.calibrated_thresholds(rows_o, cols_o, conf)
        assert tr_g == pytest.approx(tr_o, rel=0.1) and tc_g == pytest.approx(tc_o, rel=0.1)
    run, P = last
    tr, tc = orc.calibrated_thresholds(rows_g, cols_g, 0.9999)
    assert tc < tr < P.tau                      # rows sum 1030 rounded values, columns 300: sqrt(N) against sqrt(M)
    # clean output under the calibrated thresholds: at 99.99 % at most a few of the 1330 checks flag
    run.tau, run.tau_cols = float(tr), float(tc)
    run.verify()
    assert run.cnt()[0] + run.cnt()[1] <= 2
    C_clean = run.dC.clone()
    Cd = orc.decode(P.C_stored, dtype)
    # a flip with tc < |delta| < tr is seen by the column check only; one above tr by both; both
    # are invisible to the analytic tolerance
    def flip_with_delta(lo, hi):
        for bit in range(9, 3, -1) if dtype == "f16" else range(6, 0, -1):
            for (i, j) in [(7, 11), (150, 500), (299, 1029), (33, 64), (200, 900)]:
                d = abs(orc.decode(orc.flip(P.C_stored, i, j, bit), dtype)[i, j] - Cd[i, j])
                if lo < d < hi:
                    return i, j, bit
        return None
    for lo, hi, want_row in ((1.5 * tc, tr / 1.5, False), (1.5 * tr, P.tau / 1.5, True)):
        pick = flip_with_delta(lo, hi)
        if pick is None:
            continue
        i, j, bit = pick
        run.tau, run.tau_cols = 0.0, 0.0
        run.inject(0, i, j, bit)
        run.verify()
        assert run.cnt()[2] == ab.ABFT_CLEAN                       # below the analytic tolerance
        run.tau, run.tau_cols = float(tr), float(tc)
        run.verify()
        rf, cf = run.flags()
        assert cf[0, j] and bool(rf[0, i]) == want_row
        run.dC.copy_(C_clean)
    run.tau, run.tau_cols = 0.0, 0.0


def _with_ld(C, run):
    full = np.zeros((run.batch, run.M, run.ldc), dtype=np.int32 if run.dtype == "i8" else np.int16)
    full[:, :, :run.N] = C.view(full.dtype)
    return full


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
def test_accumulator_flip_is_caught_by_the_fused_check(ctx, dtype):
    M, N, K = 197, 200, 256
    A, B = gen.gen_operands(dtype, M, N, K, 41, 42, trans_b=True)
    run = Run(ctx, dtype, A, B, True)
    run.gemm(ab.ABFT_DETECT)
    C_clean = run.C().copy()
    # fp32 accumulators: only the top exponent bit turns a value of order one into a delta
    # above tau for certain; integers: any bit does
    fp = dtype != "i8"
    for (i, j, bit) in [(0, 0, 30), (196, 199, 30 if fp else 27), (130, 129, 30 if fp else 0)]:
        print(f"acc flip dtype={dtype} i={i} j={j} bit={bit}", flush=True)
        run.inject(0, i, j, bit, ab.ABFT_INJECT_ACCUMULATOR)
        run.gemm(ab.ABFT_DETECT)
        rf, cf = run.flags()
        cnt = run.cnt()
        assert rf.sum() == 1 and cf.sum() == 1 and rf[0, i] and cf[0, j]
        assert cnt[0] == 1 and cnt[1] == 1 and cnt[2] == ab.ABFT_LOCALISED
        assert not np.array_equal(run.C(), C_clean)
        run.correct()
        assert np.array_equal(run.C(), C_clean)
        rf, cf = run.flags()
        assert not rf.any() and not cf.any() and run.cnt()[2] == ab.ABFT_CLEAN
        # one-shot: the next GEMM is clean again
        run.gemm(ab.ABFT_DETECT)
        assert run.cnt()[2] == ab.ABFT_CLEAN and np.array_equal(run.C(), C_clean)
    # DETECT_CORRECT does both in one call
    run.inject(0, 5, 7, 30, ab.ABFT_INJECT_ACCUMULATOR)
    run.gemm(ab.ABFT_DETECT_CORRECT)
    cnt = run.cnt()
    assert np.array_equal(run.C(), C_clean) and cnt[2] == ab.ABFT_CLEAN and cnt[3] == 1 and cnt[4] == ab.ABFT_LOCALISED


def test_corrupted_checksum_is_one_sided(ctx):
    # a fault in a predicted checksum entry (not in C) flags one side only: "checksum suspect"
    M, N, K = 64, 96, 128
    A, B = gen.gen_operands("i8", M, N, K, 51, 52, trans_b=True)
    run = Run(ctx, "i8", A, B, True)
    run.gemm(ab.ABFT_DETECT)
    ptr, n = ab.abft_workspace(ctx, ab.ABFT_WS_RC_PRED, run.shape)
    from abft_harness import _DevView
    t = torch.as_tensor(_DevView(ptr, n, "<i4"), device="cuda")
    t[10] += 1
    torch.cuda.synchronize()
    C_before = run.C().copy()
    run.verify()
    rf, cf = run.flags()
    assert rf.sum() == 1 and rf[0, 10] and not cf.any() and run.cnt()[2] == ab.ABFT_CHECKSUM_SUSPECT
    run.correct()                                   # nothing to recompute
    assert run.cnt()[3] == 0 and np.array_equal(run.C(), C_before)


@pytest.mark.gpu
def test_context_reuse_across_shapes_and_modes(ctx):
    """Protected calls alternate between two accumulate regions and each call's finish kernel
    clears the other one: whatever the order of shapes, dtypes and cached / uncached calls, a
    clean GEMM must come out clean, with exact integer checksums."""
    cases = [("i8", 300, 520, 256, True), ("bf16", 600, 640, 192, True), ("i8", 130, 70, 100, False),
             ("i8", 640, 520, 384, True)]
    runs = []
    for k, (dtype, M, N, K, tb) in enumerate(cases):
        A, B = gen.gen_operands(dtype, M, N, K, 71 + k, 81 + k, trans_b=tb)
        runs.append((Run(ctx, dtype, A, B, tb), oracle_items(dtype, A, B, tb)[0], dtype))
    order = [0, 1, 0, 0, 2, 3, 1, 3, 3, 2, 0]
    last = None
    for step_no, idx in enumerate(order):
        run, P, dtype = runs[idx]
        cached = (last == idx)                     # same B as the previous call: reuse its checksum
        run.gemm(ab.ABFT_DETECT | (ab.ABFT_B_CHECKSUM_CACHED if cached else 0))
        cnt = run.cnt()
        assert cnt[2] == ab.ABFT_CLEAN and cnt[0] == 0 and cnt[1] == 0, (step_no, idx, cnt)
        if dtype == "i8":
            ring = lambda v: (np.asarray(v, dtype=np.int64) & 0xFFFFFFFF).astype(np.uint32)
            for which, want in ((ab.ABFT_WS_CC_PRED, P.cc_pred), (ab.ABFT_WS_RC_PRED, P.rc_pred),
                                (ab.ABFT_WS_CC_OBS, P.cc_pred), (ab.ABFT_WS_RC_OBS, P.rc_pred),
                                (ab.ABFT_WS_A_SUM, P.a)):
                assert np.array_equal(run.ws(which)[0].view(np.uint32), ring(want)), (step_no, which)
        last = idx


def test_argument_errors(ctx):
    A, B = gen.gen_operands("bf16", 64, 64, 64, 1, 2, trans_b=True)
    run = Run(ctx, "bf16", A, B, True)
    s = run.shape
    r = run.result()
    assert ab.abft_gemm(ctx, None, run.dB, run.dC, run.code, ab.ABFT_DETECT, s, r) == ab.ABFT_EINVAL
    assert ab.abft_gemm(ctx, run.dA, run.dB, run.dC, 9, ab.ABFT_DETECT, s, r) == ab.ABFT_EINVAL
    assert ab.abft_gemm(ctx, run.dA, run.dB, run.dC, run.code, 7, s, r) == ab.ABFT_EINVAL
    assert ab.abft_gemm(ctx, run.dA, run.dB, run.dC, run.code, ab.ABFT_DETECT, s, None) == ab.ABFT_EINVAL
    bad = ab.make_shape(64, 64, 64, lda=68)
    assert ab.abft_gemm(ctx, run.dA, run.dB, run.dC, run.code, ab.ABFT_DETECT, bad, r) == ab.ABFT_EALIGN
    bad = ab.make_shape(64, 64, 64, lda=32)
    assert ab.abft_gemm(ctx, run.dA, run.dB, run.dC, run.code, ab.ABFT_DETECT, bad, r) == ab.ABFT_ESHAPE
    assert ab.abft_gemm(ctx, run.dA.data_ptr() + 2, run.dB, run.dC, run.code, ab.ABFT_DETECT, s, r) == ab.ABFT_EALIGN
    big = ab.make_shape(100000, 64, 64)
    assert ab.abft_gemm(ctx, run.dA, run.dB, run.dC, run.code, ab.ABFT_DETECT, big, r) == ab.ABFT_EWORKSPACE
    k17 = ab.make_shape(64, 64, 1 << 17)
    assert ab.abft_gemm(ctx, run.dA, run.dB, run.dC, ab.ABFT_I8, ab.ABFT_DETECT, k17, r) == ab.ABFT_ESHAPE
    fresh = ab.abft_create(1024, 1024, 1024, 1)
    try:
        assert ab.abft_verify(fresh, run.dC, run.code, s, r) == ab.ABFT_ESTATE
        assert ab.abft_gemm(fresh, run.dA, run.dB, run.dC, run.code,
                            ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED, s, r) == ab.ABFT_ESTATE
    finally:
        ab.abft_destroy(fresh)
    assert ab.abft_inject(ctx, run.dC, run.code, s, 0, 64, 0, 3) == ab.ABFT_EINVAL
    assert ab.abft_inject(ctx, run.dC, run.code, s, 0, 0, 0, 16) == ab.ABFT_EINVAL
    # nothing above may have disturbed the device
    run.gemm(ab.ABFT_DETECT)
    assert run.cnt()[2] == ab.ABFT_CLEAN


def _full_size_fp(ctx, dtype, M, N, K, seed_a, seed_b, sample_seed, edge_rows):
    """A floating-point GEMM at full size, in the launch configuration bench.py times: every element
    of C, all checksum vectors (the oracle computes all of it in a few seconds), clean flags; then
    seeded stored-C flips far above the tolerance are localised and repaired bit for bit, and with
    the stored-side sums also a mantissa flip far below it."""
    A, B = gen.gen_operands(dtype, M, N, K, seed_a, seed_b, trans_b=True)
    run = Run(ctx, dtype, A, B, True)
    run.gemm(ab.ABFT_DETECT)
    rf, cf = run.flags()
    cnt = run.cnt()
    assert not rf.any() and not cf.any() and cnt[2] == ab.ABFT_CLEAN
    Ad, Bd = orc.decode(A[0], dtype), orc.decode(B[0], dtype)
    a, b = orc.encode(Ad, Bd, True)
    cc, rc, s = orc.predict(Ad, Bd, a, b, True)
    ma, mb = np.max(np.abs(Ad)), np.max(np.abs(Bd))
    tau = orc.tau(K, ma, mb)
    assert run.ws(ab.ABFT_WS_TAU)[0, 0] == pytest.approx(tau, rel=1e-5)
    tol = 1e-2 * tau
    assert np.max(np.abs(run.ws(ab.ABFT_WS_A_SUM)[0] - a)) <= 1e-5 * M * ma
    assert np.max(np.abs(run.ws(ab.ABFT_WS_B_SUM)[0] - b)) <= 1e-5 * N * mb
    assert np.max(np.abs(run.ws(ab.ABFT_WS_CC_PRED)[0] - cc)) <= tol * np.sqrt(M)
    assert np.max(np.abs(run.ws(ab.ABFT_WS_RC_PRED)[0] - rc)) <= tol * np.sqrt(N)
    # observed sums equal the predictions up to fp32 noise (the identity, at full size)
    assert np.max(np.abs(run.ws(ab.ABFT_WS_CC_OBS)[0] - cc)) <= tol * np.sqrt(M)
    assert np.max(np.abs(run.ws(ab.ABFT_WS_RC_OBS)[0] - rc)) <= tol * np.sqrt(N)
    assert abs(run.ws(ab.ABFT_WS_S_PRED)[0, 0] - s) <= 1e-4 * K * M * N * ma * mb
    # the whole of C, element by element
    C = run.C()[0]
    ref = orc.gemm(Ad, Bd, True)
    got = orc.decode(C, dtype)
    scale = np.max(np.abs(ref))
    ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11
    err = np.abs(got - ref)
    assert np.max(err) <= 1e-2 * scale
    assert np.all(err <= ulp * np.abs(ref) + 2e-6 * scale + 1e-7)
    assert np.mean(C != orc.store(ref, dtype)) < 5e-3       # fp32 noise across a rounding boundary
    del err, got
    # stored flips at full size: an exponent flip of a small element is far above tau
    C_before = run.dC.clone()
    rng = np.random.default_rng(sample_seed)
    top = 14                                                 # bf16 and fp16: the top exponent bit
    ok = (np.abs(ref) > 0.05) & (np.abs(ref) < 0.5)         # setting bit 14 multiplies these by 2^16 or more
    cand = np.argwhere(ok)
    picks = [tuple(cand[k]) for k in rng.integers(0, len(cand), 4)] + \
            [(r, int(np.flatnonzero(ok[r])[-1])) for r in edge_rows]
    for (i, j) in picks:
        i, j = int(i), int(j)
        run.inject(0, i, j, top)
        run.verify()
        rf, cf = run.flags()
        assert rf.sum() == 1 and cf.sum() == 1 and rf[0, i] and cf[0, j] and run.cnt()[2] == ab.ABFT_LOCALISED
        run.correct()
        assert torch.equal(run.dC, C_before) and run.cnt()[2] == ab.ABFT_CLEAN and run.cnt()[3] == 1
    # with the stored-side sums a mantissa flip below tau is seen as well
    run.gemm(ab.ABFT_DETECT | ab.ABFT_STORED_SUMS)
    assert run.cnt()[2] == ab.ABFT_CLEAN and torch.equal(run.dC, C_before)
    i = int(rng.integers(0, M))
    j = int(np.argmax(np.abs(ref[i])))
    bit = 3 if dtype == "bf16" else 6                        # |delta| = |C| / 16
    assert tau / 100 < abs(ref[i, j]) / 16 < tau / 2
    run.inject(0, i, j, bit)
    run.verify()
    rf, cf = run.flags()
    assert rf.sum() == 1 and cf.sum() == 1 and rf[0, i] and cf[0, j]
    run.correct()
    assert torch.equal(run.dC, C_before) and run.cnt()[2] == ab.ABFT_CLEAN


def test_full_size_bench_workload(ctx_big):
    """The benchmark workload (ViT-B fc1, batch 64, bf16: 12608 x 3072 x 768)."""
    g = gen.CONFIGS[1]["gemms"][0]
    _full_size_fp(ctx_big, "bf16", g["M"], g["N"], g["K"], gen.seed_for(1, 0), gen.seed_for(1, 1), gen.seed_for(1, 7),
                  [0, 255, 256, 10751, 10752, 10880, g["M"] - 1])


def test_full_size_fp16_fc2(ctx_big):
    """The fp16 leg of the injection campaign (ViT-B fc2 at batch 32: 6304 x 768 x 3072)."""
    g = gen.CONFIGS[4]["gemms"][0]
    _full_size_fp(ctx_big, "f16", g["M"], g["N"], g["K"], gen.seed_for(4, 2), gen.seed_for(4, 3), gen.seed_for(4, 8),
                  [0, 127, 128, 6143, 6144, g["M"] - 1])


def test_full_size_int8_fc2(ctx_big):
    """ViT-B fc2 at batch 32 in int8 (the injection-campaign GEMM): every element of C bit-exact,
    exact checksums in Z/2^32 at full size, seeded flips detected, localised, repaired."""
    g = gen.CONFIGS[4]["gemms"][0]
    M, N, K = g["M"], g["N"], g["K"]
    A, B = gen.gen_operands("i8", M, N, K, gen.seed_for(4, 0), gen.seed_for(4, 1), trans_b=True)
    run = Run(ctx_big, "i8", A, B, True)
    run.gemm(ab.ABFT_DETECT)
    rf, cf = run.flags()
    assert not rf.any() and not cf.any() and run.cnt()[2] == ab.ABFT_CLEAN
    a, b = orc.encode(A[0], B[0], True)
    cc, rc, s = orc.predict(A[0], B[0], a, b, True)
    for which, want in ((ab.ABFT_WS_A_SUM, a), (ab.ABFT_WS_B_SUM, b), (ab.ABFT_WS_CC_PRED, cc),
                        (ab.ABFT_WS_RC_PRED, rc), (ab.ABFT_WS_CC_OBS, cc), (ab.ABFT_WS_RC_OBS, rc)):
        assert np.array_equal(run.ws(which)[0].view(np.uint32), ring(want)), which
    assert run.ws(ab.ABFT_WS_S_PRED)[0, 0].view(np.uint32) == ring(s)
    ref = orc.gemm(A[0], B[0], True)
    C = run.C()[0]
    assert np.array_equal(C, ref.astype(np.int32))
    C_before = run.dC.clone()
    for (_, i, j, bit) in gen.gen_flips(12, M, N, "i8", gen.seed_for(4, 9)):
        i, j, bit = int(i), int(j), int(bit)
        run.inject(0, i, j, bit)
        run.verify()
        rf, cf = run.flags()
        assert rf.sum() == 1 and cf.sum() == 1 and rf[0, i] and cf[0, j]
        run.correct()
        assert torch.equal(run.dC, C_before) and run.cnt()[2] == ab.ABFT_CLEAN


@pytest.fixture(scope="module")
def ctx_block():
    # one transformer block of ViT-L/16 at 384^2, batch 64: 1024 per-head GEMMs of 577 x 577
    c = ab.abft_create(max_rows=1024 * 577, max_cols=1024 * 577, max_depth=1024 * 640, max_batch=1024)
    yield c
    ab.abft_destroy(c)


def _block_cases():
    for cfg in (2, 3):
        for gi, g in enumerate(gen.CONFIGS[cfg]["gemms"]):
            yield pytest.param(cfg, gi, id=f"cfg{cfg + 1}-{g['name']}")


@pytest.mark.parametrize("cfg,gi", list(_block_cases()))
def test_transformer_block_gemms_full_size_sampled(ctx_block, cfg, gi):
    """Every GEMM class of one ViT-B/16 block (bf16, batch 32) and one ViT-L/16 block at 384^2
    (int8, batch 64) at full size.  The oracle gives all checksum vectors of every batch item
    (O(MK + KN + K(M+N)) work per item) and a seeded sample of full rows of C; the flags must be
    clean; one stored flip is localised and repaired."""
    dtype = gen.CONFIGS[cfg]["dtype"]
    g = gen.CONFIGS[cfg]["gemms"][gi]
    M, N, K, batch, tb = g["M"], g["N"], g["K"], g["batch"], g["trans_b"]
    A, B = gen.gen_operands(dtype, M, N, K, gen.seed_for(cfg, 10 + 2 * gi), gen.seed_for(cfg, 11 + 2 * gi),
                            trans_b=tb, batch=batch, a_kind=g["a_kind"], b_kind=g["b_kind"])
    run = Run(ctx_block, dtype, A, B, tb)
    run.gemm(ab.ABFT_DETECT)
    rf, cf = run.flags()
    cnt = run.cnt()
    assert not rf.any() and not cf.any() and cnt[0] == 0 and cnt[1] == 0 and cnt[2] == ab.ABFT_CLEAN
    got = {w: run.ws(w) for w in (ab.ABFT_WS_A_SUM, ab.ABFT_WS_B_SUM, ab.ABFT_WS_CC_PRED, ab.ABFT_WS_RC_PRED,
                                  ab.ABFT_WS_CC_OBS, ab.ABFT_WS_RC_OBS, ab.ABFT_WS_S_PRED)}
    tau_g = run.ws(ab.ABFT_WS_TAU)
    rng = np.random.default_rng(gen.seed_for(cfg, 40 + gi))
    items = np.unique(np.concatenate([rng.integers(0, batch, 5), [0, batch - 1]]))
    for bi in range(batch):
        Ad = A[bi] if dtype == "i8" else orc.decode(A[bi], dtype)
        Bd = B[bi] if dtype == "i8" else orc.decode(B[bi], dtype)
        a, b = orc.encode(Ad, Bd, tb)
        cc, rc, s = orc.predict(Ad, Bd, a, b, tb)
        if dtype == "i8":
            for w, want in ((ab.ABFT_WS_A_SUM, a), (ab.ABFT_WS_B_SUM, b), (ab.ABFT_WS_CC_PRED, cc),
                            (ab.ABFT_WS_RC_PRED, rc), (ab.ABFT_WS_CC_OBS, cc), (ab.ABFT_WS_RC_OBS, rc)):
                assert np.array_equal(got[w][bi].view(np.uint32), ring(want)), (bi, w)
            assert got[ab.ABFT_WS_S_PRED][bi, 0].view(np.uint32) == ring(s)
        else:
            ma, mb = np.max(np.abs(Ad)), np.max(np.abs(Bd))
            tau = orc.tau(K, ma, mb)
            assert tau_g[bi, 0] == pytest.approx(tau, rel=1e-5)
            tol = 1e-2 * tau
            assert np.max(np.abs(got[ab.ABFT_WS_A_SUM][bi] - a)) <= 1e-5 * M * ma
            assert np.max(np.abs(got[ab.ABFT_WS_B_SUM][bi] - b)) <= 1e-5 * N * mb
            assert np.max(np.abs(got[ab.ABFT_WS_CC_PRED][bi] - cc)) <= tol * np.sqrt(M)
            assert np.max(np.abs(got[ab.ABFT_WS_RC_PRED][bi] - rc)) <= tol * np.sqrt(N)
            assert np.max(np.abs(got[ab.ABFT_WS_CC_OBS][bi] - cc)) <= tol * np.sqrt(M)
            assert np.max(np.abs(got[ab.ABFT_WS_RC_OBS][bi] - rc)) <= tol * np.sqrt(N)
            assert abs(got[ab.ABFT_WS_S_PRED][bi, 0] - s) <= 1e-4 * K * M * N * ma * mb
        if bi in items:
            rows = np.unique(np.concatenate([rng.integers(0, M, 6), [0, M - 1]]))
            ref = orc.gemm(np.ascontiguousarray(Ad[rows]), Bd, tb)
            Cg = run.dC[bi][torch.as_tensor(rows, device="cuda")][:, :N].cpu().numpy()
            if dtype == "i8":
                assert np.array_equal(Cg, ref.astype(np.int32)), bi
            else:
                Cg = Cg.view(np.uint16)
                val = orc.decode(Cg, dtype)
                scale = np.max(np.abs(ref))
                assert np.max(np.abs(val - ref)) <= 1e-2 * scale
                assert np.all(np.abs(val - ref) <= 2.0 ** -8 * np.abs(ref) + 2e-6 * scale + 1e-7)
                assert np.mean(Cg != orc.store(ref, dtype)) < 5e-3
    # one stored flip (a high exponent bit for bf16, so that it is far above the tolerance)
    C_before = run.dC.clone()
    bi, i, j = int(items[-1]), int(rng.integers(0, M)), int(rng.integers(0, N))
    bit = int(rng.integers(0, 32)) if dtype == "i8" else 14
    run.inject(bi, i, j, bit)
    run.verify()
    rf, cf = run.flags()
    assert rf.sum() == 1 and cf.sum() == 1 and rf[bi, i] and cf[bi, j] and run.cnt()[2] == ab.ABFT_LOCALISED
    run.correct()
    assert torch.equal(run.dC, C_before) and run.cnt()[2] == ab.ABFT_CLEAN and run.cnt()[3] == 1
    del run, C_before
    torch.cuda.empty_cache()


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(197, 203, 256, 2, True), (600, 520, 128, 1, False)])
def test_correction_of_several_tiles_keeps_the_resummed_vectors(ctx, dtype, M, N, K, batch, trans_b):
    """Several corrupted elements at once, some sharing a tile row or a tile column, some in the
    ragged last tiles, some turned into Inf / NaN: after verify + correct the stored C is the clean
    one, every flag is down, and the re-summed vectors -- brought up to date for the rows and
    columns of the recomputed tiles only -- are the sums of the clean stored C."""
    A, B = gen.gen_operands(dtype, M, N, K, 411, 412, trans_b=trans_b, batch=batch)
    P = oracle_items(dtype, A, B, trans_b)
    run = Run(ctx, dtype, A, B, trans_b)
    run.gemm(ab.ABFT_DETECT)
    clean = np.stack([p.C_stored for p in P])
    if dtype == "i8":
        assert np.array_equal(run.C(), clean)
    C_clean = run.C().copy()
    # integers: a different bit per element, so that two errors in one column cannot cancel mod 2^32
    bits = [30, 29, 28, 27, 26, 25] if dtype == "i8" else [14] * 6
    spots = [(0, 0, 0), (0, 0, 40), (0, 70, 5), (0, M - 1, N - 1), (0, M - 1, 40)]
    tiles = 3 * 3                                           # tile rows {0, 2, last} x tile columns {0, 1, last}
    if batch > 1:
        spots.append((1, 33, N - 1))
        tiles += 1
    run.verify()
    for (bi, i, j), bit in zip(spots, bits):
        run.inject(bi, i, j, bit)
    run.verify()
    rf, cf = run.flags()
    for (bi, i, j) in spots:
        assert rf[bi, i] and cf[bi, j]
    assert rf.sum() == (3 if batch == 1 else 4) and cf.sum() == (4 if batch == 1 else 5)
    run.correct()
    assert np.array_equal(run.C(), C_clean), "C not restored"
    rf, cf = run.flags()
    cnt = run.cnt()
    assert not rf.any() and not cf.any()
    assert cnt[0] == 0 and cnt[1] == 0 and cnt[2] == ab.ABFT_CLEAN and cnt[3] == tiles
    cc_v, rc_v = run.ws(ab.ABFT_WS_CC_VOBS), run.ws(ab.ABFT_WS_RC_VOBS)
    for bi in range(batch):
        _, _, _, _, cc_obs, rc_obs = orc.check(P[bi], C_clean[bi])
        if dtype == "i8":
            assert np.array_equal(cc_v[bi].view(np.uint32), (np.asarray(cc_obs) & 0xFFFFFFFF).astype(np.uint32))
            assert np.array_equal(rc_v[bi].view(np.uint32), (np.asarray(rc_obs) & 0xFFFFFFFF).astype(np.uint32))
        else:
            assert np.max(np.abs(cc_v[bi] - cc_obs)) <= 1e-2 * P[bi].tau
            assert np.max(np.abs(rc_v[bi] - rc_obs)) <= 1e-2 * P[bi].tau
    run.correct()                                           # nothing left to repair
    cnt = run.cnt()
    assert cnt[2] == ab.ABFT_CLEAN and cnt[3] == 0 and np.array_equal(run.C(), C_clean)
    run.verify()                                            # the full re-sum agrees
    rf, cf = run.flags()
    assert not rf.any() and not cf.any() and run.cnt()[2] == ab.ABFT_CLEAN


@pytest.mark.parametrize("M,N,K,batch,trans_b", [(197, 768, 768, 1, True), (130, 70, 100, 3, False),
                                                 (520, 1030, 256, 2, True)])
def test_checksum_only_correction_int8(ctx, M, N, K, batch, trans_b):
    """Single stored flips repaired from the checksums alone (no operand read, no recompute):
    the result must be what the oracle's checksum-only correction gives, i.e. the clean C bit
    for bit; patterns the scheme cannot explain are left for the tile recompute."""
    A, B = gen.gen_operands("i8", M, N, K, 311, 312, trans_b=trans_b, batch=batch)
    P = oracle_items("i8", A, B, trans_b)
    run = Run(ctx, "i8", A, B, trans_b)
    run.gemm(ab.ABFT_DETECT)
    # before any verify there is no re-summed C to work from
    assert ab.abft_correct_checksum(ctx, run.dC, run.code, run.shape, run.result()) == ab.ABFT_ESTATE
    clean = np.stack([p.C_stored for p in P])
    assert np.array_equal(run.C(), clean)
    for (bi, i, j, bit) in gen.gen_flips(10, M, N, "i8", 313, batch=batch):
        bi, i, j, bit = int(bi), int(i), int(j), int(bit)
        run.inject(bi, i, j, bit)
        run.verify()
        X = run.C()
        rf, cf = run.flags()
        assert rf.sum() == 1 and cf.sum() == 1 and rf[bi, i] and cf[bi, j]
        _, _, _, _, cc_obs, rc_obs = orc.check(P[bi], X[bi])
        want, fixed = orc.correct_by_checksum(X[bi], cc_obs, rc_obs, P[bi].cc_pred, P[bi].rc_pred)
        assert fixed == 1
        run.correct_checksum()
        got = run.C()
        assert np.array_equal(got[bi], want) and np.array_equal(got, clean)
        cnt = run.cnt()
        assert cnt[0] == 0 and cnt[1] == 0 and cnt[2] == ab.ABFT_CLEAN and cnt[3] == 1 and cnt[4] == ab.ABFT_LOCALISED
        rf, cf = run.flags()
        assert not rf.any() and not cf.any()
        # the re-summed vectors were updated with the repair: they equal the predictions again
        assert np.array_equal(run.ws(ab.ABFT_WS_CC_VOBS), run.ws(ab.ABFT_WS_CC_PRED))
        assert np.array_equal(run.ws(ab.ABFT_WS_RC_VOBS), run.ws(ab.ABFT_WS_RC_PRED))
        run.verify()
        assert run.cnt()[2] == ab.ABFT_CLEAN
    # two errors in one item (two flags on each side): untouched, left for the recompute;
    # a single error in another item of the same call is still repaired
    run.inject(0, 1, 2, 5)
    run.inject(0, M - 1, N - 1, 30)
    if batch > 1:
        run.inject(batch - 1, 3, 4, 31)
    run.verify()
    X = run.C()
    run.correct_checksum()
    got = run.C()
    for bi in range(batch):
        _, _, _, _, cc_obs, rc_obs = orc.check(P[bi], X[bi])
        want, _ = orc.correct_by_checksum(X[bi], cc_obs, rc_obs, P[bi].cc_pred, P[bi].rc_pred)
        assert np.array_equal(got[bi], want), bi
    assert np.array_equal(got[0], X[0]) and not np.array_equal(got[0], clean[0])
    cnt = run.cnt()
    assert cnt[0] == 2 and cnt[1] == 2 and cnt[2] == ab.ABFT_LOCALISED and cnt[3] == (1 if batch > 1 else 0)
    run.correct()
    assert np.array_equal(run.C(), clean) and run.cnt()[2] == ab.ABFT_CLEAN
    # floating point is refused
    Af, Bf = gen.gen_operands("bf16", 64, 64, 64, 1, 2, trans_b=True)
    rf16 = Run(ctx, "bf16", Af, Bf, True)
    rf16.gemm(ab.ABFT_DETECT)
    rf16.verify()
    assert ab.abft_correct_checksum(ctx, rf16.dC, rf16.code, rf16.shape, rf16.result()) == ab.ABFT_EINVAL


# ---------------------------------------------------------------- batches of small problems
@pytest.fixture(scope="module")
def ctx_items():
    c = ab.abft_create(max_rows=66 * 640, max_cols=66 * 640, max_depth=66 * 640, max_batch=66)
    yield c
    ab.abft_destroy(c)


ITEM_SHAPES = [
    # (M, N, K, batch, trans_b): from 64 items on, one workgroup takes a whole item
    (70, 50, 40, 64, True),        # N <= 64: 2 x 2 waves, 64-row blocks
    (70, 50, 40, 64, False),
    (130, 64, 197, 64, False),     # attn V shape with several slabs of K
    (100, 130, 72, 65, True),      # N <= 256: 1 x 4 waves, two column blocks per wave at most
    (45, 200, 100, 66, False),
    (197, 197, 64, 64, True),      # per-head Q K^T
    (60, 300, 24, 64, True),       # N <= 640: five column blocks per wave at most
    (33, 577, 64, 64, False),
    (1, 1, 1, 64, True),
    (193, 1, 236, 66, False),      # a single column: one 32-column block, 31 of them padding
    (1, 300, 100, 64, True),       # a single row
]


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", ITEM_SHAPES)
def test_item_kernel_clean_matches_oracle(ctx_items, dtype, M, N, K, batch, trans_b):
    s = ab.make_shape(M, N, K, batch=batch, lda=K, ldb=K if trans_b else N, ldc=N, transB=trans_b)
    assert ab.abft_tile_shape(ab.DTYPE_CODE[dtype], s) == (M, N)      # the whole item per workgroup
    _clean_case(ctx_items, dtype, M, N, K, batch, trans_b)


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(70, 50, 40, 64, False), (100, 130, 72, 65, True)])
def test_item_kernel_flips_cached_b_and_correction(ctx_items, dtype, M, N, K, batch, trans_b):
    ctx = ctx_items
    A, B = gen.gen_operands(dtype, M, N, K, 61, 62, trans_b=trans_b, batch=batch, b_kind="act")
    P = oracle_items(dtype, A, B, trans_b)
    run = Run(ctx, dtype, A, B, trans_b)
    run.gemm(ab.ABFT_DETECT)
    check_clean(run, P)
    C_clean = run.C().copy()
    # the encoding of B left by that call serves a second one; so does abft_encode_b's
    run.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)
    check_clean(run, P)
    assert ab.abft_encode_b(ctx, run.dB, run.code, run.shape) == ab.ABFT_OK
    run.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)
    check_clean(run, P)
    # armed accumulator flips: caught by the check inside the kernel, at the element
    fp = dtype != "i8"
    for (bi, i, j, bit) in [(0, 0, 0, 30), (batch - 1, M - 1, N - 1, 30 if fp else 27), (7, M // 2, N // 2, 30 if fp else 0)]:
        run.inject(bi, i, j, bit, ab.ABFT_INJECT_ACCUMULATOR)
        run.gemm(ab.ABFT_DETECT)
        rf, cf = run.flags()
        cnt = run.cnt()
        assert rf.sum() == 1 and cf.sum() == 1 and rf[bi, i] and cf[bi, j]
        assert cnt[0] == 1 and cnt[1] == 1 and cnt[2] == ab.ABFT_LOCALISED
        run.correct()
        assert np.array_equal(run.C(), C_clean) and run.cnt()[2] == ab.ABFT_CLEAN
        run.gemm(ab.ABFT_DETECT)
        assert run.cnt()[2] == ab.ABFT_CLEAN and np.array_equal(run.C(), C_clean)
    run.inject(3, 5, 7, 30, ab.ABFT_INJECT_ACCUMULATOR)
    run.gemm(ab.ABFT_DETECT_CORRECT)
    cnt = run.cnt()
    assert np.array_equal(run.C(), C_clean) and cnt[2] == ab.ABFT_CLEAN and cnt[3] == 1 and cnt[4] == ab.ABFT_LOCALISED
    # stored flips: verify works from the vectors the kernel left
    for (bi, i, j, bit) in gen.gen_flips(8, M, N, dtype, 63, batch=batch):
        bi, i, j, bit = int(bi), int(i), int(j), int(bit)
        X = orc.flip(P[bi].C_stored, i, j, bit)
        if dtype != "i8":
            with np.errstate(all="ignore"):
                delta = abs(orc.decode(X, dtype)[i, j] - orc.decode(P[bi].C_stored, dtype)[i, j])
            if not (delta > 2 * P[bi].tau):            # below or near the tolerance: covered elsewhere
                continue
        run.inject(bi, i, j, bit)
        run.verify()
        rf, cf = run.flags()
        assert rf.sum() == 1 and cf.sum() == 1 and rf[bi, i] and cf[bi, j] and run.cnt()[2] == ab.ABFT_LOCALISED
        run.correct()
        assert np.array_equal(run.C(), C_clean) and run.cnt()[2] == ab.ABFT_CLEAN
    # a tiled-kernel call after item calls on the same context (the regions they share)
    A1, B1 = gen.gen_operands(dtype, 300, 200, 264, 64, 65, trans_b=True)
    r1 = Run(ctx, dtype, A1, B1, True)
    r1.gemm(ab.ABFT_DETECT)
    check_clean(r1, oracle_items(dtype, A1, B1, True))
    run.gemm(ab.ABFT_DETECT)
    check_clean(run, P)
    r1.gemm(ab.ABFT_DETECT)
    check_clean(r1, oracle_items(dtype, A1, B1, True))


@pytest.mark.parametrize("dtype", ["i8", "bf16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(197, 130, 72, 3, True), (150, 70, 100, 2, False),
                                                 (600, 520, 256, 2, True),       # 256-row tiles
                                                 (70, 50, 40, 64, False), (100, 130, 72, 65, True)])
def test_leading_dimensions_and_batch_strides(ctx_items, dtype, M, N, K, batch, trans_b):
    """Operands and C embedded in larger allocations: leading dimensions wider than the rows,
    batch strides longer than an item.  Everything outside the M x N items of C must stay as it
    was; everything outside the operands is filled with a pattern that must never be used."""
    ctx = ctx_items
    es, osz = (1, 4) if dtype == "i8" else (2, 2)
    A, B = gen.gen_operands(dtype, M, N, K, 71, 72, trans_b=trans_b, batch=batch)
    P = oracle_items(dtype, A, B, trans_b)

    def embed(arr, extra_rows, extra_cols, fill, tdt):
        b, r, c = arr.shape
        ld = (c + extra_cols + 16 // arr.dtype.itemsize - 1) // (16 // arr.dtype.itemsize) * (16 // arr.dtype.itemsize)
        big = np.full((b, r + extra_rows, ld), fill, dtype=arr.dtype)
        big[:, :r, :c] = arr
        t = torch.from_numpy(big.view(np.int16) if arr.dtype == np.uint16 else big).to("cuda").view(tdt)
        return t, ld, (r + extra_rows) * ld

    in_t = torch.int8 if dtype == "i8" else torch.int16
    pat = 0x55 if dtype == "i8" else 0x7F55            # bf16/f16: a large finite value (f16: NaN pattern 0x7F55)
    dA, lda, sA = embed(A, 3, 40, pat, in_t)
    dB, ldb, sB = embed(B, 2, 24, pat, in_t)
    out_np = np.int32 if dtype == "i8" else np.uint16
    Cbig = np.full((batch, M + 4, N), 0, dtype=out_np)
    dC, ldc, sC = embed(Cbig, 0, 20, 0, torch.int32 if dtype == "i8" else torch.int16)
    dC.fill_(0x1234)
    shape = ab.make_shape(M, N, K, batch=batch, lda=lda, ldb=ldb, ldc=ldc, strideA=sA, strideB=sB, strideC=sC,
                          transB=trans_b)
    rf = torch.full((batch * M,), 7, dtype=torch.uint8, device="cuda")
    cf = torch.full((batch * N,), 7, dtype=torch.uint8, device="cuda")
    cnt = torch.full((8,), 99, dtype=torch.int32, device="cuda")
    res = ab.make_result(rf, cf, cnt, 0.0)
    code = ab.DTYPE_CODE[dtype]
    for mode in (ab.ABFT_DETECT, ab.ABFT_OFF):
        dC.fill_(0x1234)
        rc = ab.abft_gemm(ctx, dA, dB, dC, code, mode, shape, None if mode == ab.ABFT_OFF else res)
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
        torch.cuda.synchronize()
        Ch = dC.cpu().numpy()
        got = Ch[:, :M, :N]
        for bi, p in enumerate(P):
            if dtype == "i8":
                assert np.array_equal(got[bi], p.C_stored), (mode, bi)
            else:
                val = orc.decode(got[bi].view(np.uint16), dtype)
                scale = np.max(np.abs(p.C_ref))
                assert np.max(np.abs(val - p.C_ref)) <= 1e-2 * scale
                assert np.mean(got[bi].view(np.uint16) != p.C_stored) < 5e-3
        assert np.all(Ch[:, M:, :] == 0x1234) and np.all(Ch[:, :, N:] == 0x1234), "wrote outside C"
    c = cnt.cpu().numpy()
    assert not rf.cpu().numpy().any() and not cf.cpu().numpy().any() and c[0] == 0 and c[1] == 0 and c[2] == ab.ABFT_CLEAN
    from abft_harness import read_ws
    kind = "i" if dtype == "i8" else "f"
    ccp = read_ws(ctx, ab.ABFT_WS_CC_PRED, shape, kind).reshape(batch, -1)
    rcp = read_ws(ctx, ab.ABFT_WS_RC_PRED, shape, kind).reshape(batch, -1)
    for bi, p in enumerate(P):
        if dtype == "i8":
            assert np.array_equal(ccp[bi].view(np.uint32), ring(p.cc_pred))
            assert np.array_equal(rcp[bi].view(np.uint32), ring(p.rc_pred))
        else:
            assert np.max(np.abs(ccp[bi] - p.cc_pred)) <= 1e-2 * p.tau * max(1.0, np.sqrt(M))
            assert np.max(np.abs(rcp[bi] - p.rc_pred)) <= 1e-2 * p.tau * max(1.0, np.sqrt(N))
    # a flip, verify and the tile recompute on the embedded C
    C_before = dC.clone()
    bi, i, j, bit = batch - 1, M - 1, N - 1, 30 if dtype == "i8" else 14
    assert ab.abft_inject(ctx, dC, code, shape, bi, i, j, bit, ab.ABFT_INJECT_STORED_C) == ab.ABFT_OK
    # (the last call above ran unprotected: the predictions of the protected one before it still stand)
    assert ab.abft_verify(ctx, dC, code, shape, res) == ab.ABFT_OK
    torch.cuda.synchronize()
    f_r, f_c = rf.cpu().numpy().reshape(batch, M), cf.cpu().numpy().reshape(batch, N)
    assert f_r.sum() == 1 and f_c.sum() == 1 and f_r[bi, i] and f_c[bi, j]
    assert ab.abft_correct(ctx, dA, dB, dC, code, shape, res) == ab.ABFT_OK
    torch.cuda.synchronize()
    assert torch.equal(dC, C_before) and cnt.cpu().numpy()[2] == ab.ABFT_CLEAN


@pytest.mark.parametrize("M,N,K", [(197, 768, 768), (600, 520, 256)])
def test_faults_in_the_operands(ctx, M, N, K):
    """Other injection sites (Sec. III-A: inputs and weights as well as outputs).  A flip in the
    weight after its checksum was encoded moves a whole column of C: the row checks catch it in
    every row whose A[i, k] is non-zero, the column check (whose prediction reads the weight as
    it is) stays silent, and the status says that C itself is not the suspect.  A flip in A
    before the call is outside what a GEMM's own checksums can see: they are taken from the
    operands as given, so the call is clean and C is the product of what it was given."""
    A, B = gen.gen_operands("i8", M, N, K, 81, 82, trans_b=True)
    run = Run(ctx, "i8", A, B, True)
    assert ab.abft_encode_b(ctx, run.dB, run.code, run.shape) == ab.ABFT_OK
    j, k, bit = N // 2, K // 3, 5
    B2 = B.copy()
    B2[0, j, k] = np.int8(np.uint8(B2[0, j, k]) ^ np.uint8(1 << bit))
    run.dB[0, j, k] = int(B2[0, j, k])
    run.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)
    a, b_clean = orc.encode(A[0], B[0], True)
    C2 = orc.gemm(A[0], B2[0], True)
    cc_pred, rc_pred, _ = orc.predict(A[0], B2[0], a, b_clean, True)
    cc_obs, rc_obs, _ = orc.observe(C2)
    _, want_rf = orc.flags_int(rc_obs, rc_pred)
    _, want_cf = orc.flags_int(cc_obs, cc_pred)
    rf, cf = run.flags()
    cnt = run.cnt()
    assert np.array_equal(run.C()[0], C2.astype(np.int32))
    assert np.array_equal(rf[0], want_rf) and np.array_equal(cf[0], want_cf) and not want_cf.any()
    assert cnt[0] == want_rf.sum() and cnt[1] == 0 and cnt[2] == ab.ABFT_CHECKSUM_SUSPECT
    # re-encoding the weight as it is now makes the call consistent again (the fault is then part of the input)
    run.gemm(ab.ABFT_DETECT)
    assert run.cnt()[2] == ab.ABFT_CLEAN
    # a flip in A before the call
    A2 = A.copy()
    A2[0, M // 2, K // 2] = np.int8(np.uint8(A2[0, M // 2, K // 2]) ^ np.uint8(1 << 7))
    run.dA[0, M // 2, K // 2] = int(A2[0, M // 2, K // 2])
    run.gemm(ab.ABFT_DETECT)
    assert run.cnt()[2] == ab.ABFT_CLEAN
    assert np.array_equal(run.C()[0], orc.gemm(A2[0], B2[0], True).astype(np.int32))


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(777, 600, 192, 1, True), (300, 200, 264, 2, True), (150, 200, 136, 2, False),
                                                 (197, 64, 197, 3, False), (100, 130, 72, 65, True), (520, 1030, 256, 1, True)])
def test_gemm_with_layer_bias(ctx_items, dtype, M, N, K, batch, trans_b):
    """C = A B + bias (Sec. III-B.1 "Checksums": the checked product is adjusted by the layer
    bias): C, both predictions, both observed sums, the scalar, clean flags, the unprotected mode,
    and a stored flip localised and repaired by a tile recompute that adds the bias again -- on the
    256-wide tiles, the general kernel, both layouts of B, batches, and a batch the bias-free call
    would hand to the one-workgroup-per-item kernel."""
    ctx = ctx_items
    A, B = gen.gen_operands(dtype, M, N, K, 301 + M, 302 + N, trans_b=trans_b, batch=batch,
                            b_kind="weight" if batch == 1 else "act")
    rng = np.random.default_rng(77 + N)
    if dtype == "i8":
        bias = rng.integers(-100000, 100000, N).astype(np.int32)
        d_bias = torch.from_numpy(bias).to("cuda")
    else:
        # of the size of the product's entries: the tolerance 1e-3 K max|A| max|B| knows nothing of
        # the bias, and the rounding of a stored row grows with the magnitude of its entries
        bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
        d_bias = torch.from_numpy(bias).to("cuda")
    P = [orc.protected_gemm(A[b], B[b], dtype, trans_b, bias=bias) for b in range(batch)]
    run = Run(ctx, dtype, A, B, trans_b)
    run.gemm_bias(d_bias, ab.ABFT_DETECT)
    check_clean(run, P)
    C_prot = run.C().copy()
    run.dC.fill_(0)
    run.gemm_bias(d_bias, ab.ABFT_OFF)
    assert np.array_equal(run.C(), C_prot)
    # the plain call on the same operands is the product without the bias
    run.gemm(ab.ABFT_DETECT)
    check_clean(run, oracle_items(dtype, A, B, trans_b))
    # stored flip: verify against the biased predictions, repair by recompute
    run.gemm_bias(d_bias, ab.ABFT_DETECT | (ab.ABFT_STORED_SUMS if dtype != "i8" else 0))
    assert np.array_equal(run.C(), C_prot)
    run.verify()
    assert run.cnt()[2] == ab.ABFT_CLEAN
    bi, i = batch - 1, M // 2
    mag = np.abs(P[bi].C_ref[i])
    mid = np.flatnonzero((mag > 0.05) & (mag < 0.5))         # top exponent bit clear: setting it multiplies by 2^16 or more
    j = int(mid[0]) if mid.size else int(np.argmin(mag))
    run.inject(bi, i, j, 30 if dtype == "i8" else 14)
    run.verify()
    rf, cf = run.flags()
    assert rf.sum() == 1 and cf.sum() == 1 and rf[bi, i] and cf[bi, j]
    run.correct()
    assert np.array_equal(run.C(), C_prot) and run.cnt()[2] == ab.ABFT_CLEAN and run.cnt()[3] == 1
    # DETECT_CORRECT with a fault in the accumulators
    acc0 = np.abs(P[0].C_ref - np.asarray(bias, dtype=P[0].C_ref.dtype)[None, :])      # the accumulator: the product alone
    ai, aj = (M - 1, N - 1) if dtype == "i8" else tuple(int(x) for x in np.argwhere(acc0 < 1.0)[-1])
    run.inject(0, ai, aj, 30, ab.ABFT_INJECT_ACCUMULATOR)    # |acc| < 2: bit 30 set makes it huge
    run.gemm_bias(d_bias, ab.ABFT_DETECT_CORRECT)
    cnt = run.cnt()
    assert cnt[2] == ab.ABFT_CLEAN and cnt[3] == 1 and cnt[4] == ab.ABFT_LOCALISED
    assert np.array_equal(run.C(), C_prot)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M,N1,N2,K1", [(600, 512, 520, 256), (197, 768, 264, 128)])
def test_input_checksum_carried_over_from_the_producer(ctx, dtype, M, N1, N2, K1):
    """Sec. V "Optimizations" (2): the checksum of a tensor is generated while it is produced.
    Producer C1 = A1 W1^T with the stored-side sums; consumer C2 = C1 W2^T takes e^T C1 and
    max|C1| from the producer (abft_supply_a + ABFT_A_CHECKSUM_GIVEN) instead of forming them.
    Clean: the consumer's vectors match the oracle's for the stored C1.  A bit of C1 flipped between
    the two calls is outside the consumer's own view of its input (its row prediction is formed from
    the flipped tensor) but disagrees with the carried checksum: the column check flags exactly the
    columns the oracle names, the row check stays silent."""
    A1, W1 = gen.gen_operands(dtype, M, N1, K1, 701, 702, trans_b=True)
    _, W2 = gen.gen_operands(dtype, M, N2, N1, 703, 704, trans_b=True)
    prod = Run(ctx, dtype, A1, W1, True)
    prod.gemm(ab.ABFT_DETECT | ab.ABFT_STORED_SUMS)
    assert prod.cnt()[2] == ab.ABFT_CLEAN
    C1 = prod.C()                                               # (1, M, N1) bits as stored
    a_ptr, na = ab.abft_workspace(ctx, ab.ABFT_WS_CC_STO, prod.shape)
    m_ptr, _ = ab.abft_workspace(ctx, ab.ABFT_WS_C_MAX, prod.shape)
    assert na == N1
    # the producer's side of the hand-over against the oracle: column sums and max of the stored C1
    C1d = orc.decode(C1[0], dtype)
    assert np.max(np.abs(prod.ws(ab.ABFT_WS_CC_STO)[0] - C1d.sum(axis=0))) <= 1e-5 * M * np.max(np.abs(C1d))
    assert prod.ws(ab.ABFT_WS_C_MAX)[0, 0] == np.float32(np.max(np.abs(C1d)))
    # keep the carried vectors: the consumer's call reuses the context's regions
    from abft_harness import _DevView
    a_dev = torch.as_tensor(_DevView(a_ptr, N1, "<u4"), device="cuda").clone()
    m_dev = torch.as_tensor(_DevView(m_ptr, 1, "<u4"), device="cuda").clone()
    cons = Run(ctx, dtype, C1, W2, True)
    P2 = orc.protected_gemm(C1[0], W2[0], dtype, True)

    def consumer():
        assert ab.abft_supply_a(ctx, a_dev, m_dev) == ab.ABFT_OK
        cons.gemm(ab.ABFT_DETECT | ab.ABFT_A_CHECKSUM_GIVEN)
    consumer()
    rf, cf = cons.flags()
    assert not rf.any() and not cf.any() and cons.cnt()[2] == ab.ABFT_CLEAN
    tol = 1e-2 * P2.tau
    assert cons.ws(ab.ABFT_WS_TAU)[0, 0] == pytest.approx(P2.tau, rel=1e-5)
    assert np.max(np.abs(cons.ws(ab.ABFT_WS_CC_PRED)[0] - P2.cc_pred)) <= tol * np.sqrt(M)
    assert np.max(np.abs(cons.ws(ab.ABFT_WS_RC_PRED)[0] - P2.rc_pred)) <= tol * np.sqrt(N2)
    cc0, rc0, _ = orc.observe(P2.C_ref)
    assert np.max(np.abs(cons.ws(ab.ABFT_WS_CC_OBS)[0] - cc0)) <= tol * np.sqrt(M)
    assert np.max(np.abs(cons.ws(ab.ABFT_WS_RC_OBS)[0] - rc0)) <= tol * np.sqrt(N2)
    assert np.max(np.abs(orc.decode(cons.C()[0], dtype) - P2.C_ref)) <= 1e-2 * np.max(np.abs(P2.C_ref))
    # the mode bit without a supplied vector is refused (the pointers are consumed by the call)
    assert ab.abft_gemm(ctx, cons.dA, cons.dB, cons.dC, cons.code, ab.ABFT_DETECT | ab.ABFT_A_CHECKSUM_GIVEN,
                        cons.shape, cons.result()) == ab.ABFT_ESTATE
    # a flip of C1 between producer and consumer
    i, k, bit = M // 3, N1 // 5, 14
    small = np.flatnonzero(np.abs(C1d[i]) < 1.0)
    k = int(small[len(small) // 2])                            # below 2: bit 14 set makes it huge
    cons.inject_operand("A", 0, i, k, bit)
    consumer()
    rf, cf = cons.flags()
    A2f = orc.flip(C1[0], i, k, bit)
    with np.errstate(all="ignore"):
        delta = orc.decode(A2f, dtype)[i, k] - C1d[i, k]
        shift = np.abs(delta * orc.decode(W2[0], dtype)[:, k])                 # what column j of C2 moved by
    sure, quiet = ~(shift <= 2 * P2.tau), shift < P2.tau / 2
    assert cf[0][sure].all() and not cf[0][quiet].any() and sure.any()
    assert not rf.any() and cons.cnt()[2] == ab.ABFT_CHECKSUM_SUSPECT


def test_input_checksum_given_int8(ctx):
    """The same mode on the integer path: the caller's a = e^T A (here the oracle's, in Z/2^32);
    an input flipped after its checksum was taken flags exactly the columns j with B[k,j] != 0."""
    M, N, K = 300, 264, 256
    A, B = gen.gen_operands("i8", M, N, K, 711, 712, trans_b=True)
    P = orc.protected_gemm(A[0], B[0], "i8", True)
    a_dev = torch.from_numpy(ring(P.a).view(np.int32)).to("cuda")
    run = Run(ctx, "i8", A, B, True)
    assert ab.abft_supply_a(ctx, a_dev, None) == ab.ABFT_OK
    run.gemm(ab.ABFT_DETECT | ab.ABFT_A_CHECKSUM_GIVEN)
    assert run.cnt()[2] == ab.ABFT_CLEAN
    assert np.array_equal(run.C()[0], P.C_stored)
    assert np.array_equal(run.ws(ab.ABFT_WS_CC_PRED)[0].view(np.uint32), ring(P.cc_pred))
    assert np.array_equal(run.ws(ab.ABFT_WS_RC_PRED)[0].view(np.uint32), ring(P.rc_pred))
    i, k, bit = 123, 45, 6
    run.inject_operand("A", 0, i, k, bit)
    assert ab.abft_supply_a(ctx, a_dev, None) == ab.ABFT_OK
    run.gemm(ab.ABFT_DETECT | ab.ABFT_A_CHECKSUM_GIVEN)
    rf, cf = run.flags()
    A2 = orc.flip(A[0], i, k, bit)
    P2 = orc.protected_gemm(A2, B[0], "i8", True)
    _, ocf, _, _, _, _ = orc.check(P, P2.C_stored)             # the old checksums against the new product
    assert np.array_equal(cf[0], ocf) and not rf.any() and run.cnt()[2] == ab.ABFT_CHECKSUM_SUSPECT
    assert np.array_equal(run.C()[0], P2.C_stored)


@pytest.mark.parametrize("dtype", ["i8", "bf16"])
def test_operand_injection_sites(ctx, dtype):
    """Flips in inputs and weights (Sec. II-A / III-A) through abft_inject: the bit lands where the
    oracle's flip puts it; a weight flipped after its offline encoding shows as row flags in
    exactly the rows the oracle names and in no column (the column prediction reads the weight as
    it is); a flip before the call is part of the operands the call encodes: clean, and C is the
    product of the flipped operands."""
    M, N, K = 197, 264, 128
    A, B = gen.gen_operands(dtype, M, N, K, 401, 402, trans_b=True)
    run = Run(ctx, dtype, A, B, True)
    assert ab.abft_encode_b(ctx, run.dB, run.code, run.shape) == ab.ABFT_OK
    P = orc.protected_gemm(A[0], B[0], dtype, True)
    n, k, bit = 33, 77, 6 if dtype == "i8" else 13
    run.inject_operand("B", 0, n, k, bit)
    B2 = orc.flip(B[0], n, k, bit)
    assert np.array_equal(run.dB.cpu().numpy()[0, :, :K].view(B2.dtype), B2)
    run.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)
    rf, cf = run.flags()
    P2 = orc.protected_gemm(A[0], B2, dtype, True)
    orf, ocf, _, status, _, _ = orc.check(P, P2.C_stored if dtype == "i8" else orc.store(P2.C_ref, dtype))
    if dtype == "i8":
        assert np.array_equal(rf[0], orf) and not cf.any() and run.cnt()[2] == ab.ABFT_CHECKSUM_SUSPECT
        assert np.array_equal(run.C()[0], P2.C_stored)
    else:
        d = np.abs((orc.decode(B2, dtype)[n, k] - orc.decode(B[0], dtype)[n, k]) * orc.decode(A[0], dtype)[:, k])
        sure = d > 2 * P.tau
        quiet = d < P.tau / 2
        assert rf[0][sure].all() and not rf[0][quiet].any() and not cf.any()
    # an input flipped before the call: consistent, hence silent
    i, ka = 100, 5
    run.inject_operand("A", 0, i, ka, bit)
    A2 = orc.flip(A[0], i, ka, bit)
    assert np.array_equal(run.dA.cpu().numpy()[0, :, :K].view(A2.dtype), A2)
    run.gemm(ab.ABFT_DETECT)
    assert run.cnt()[2] == ab.ABFT_CLEAN
    check_clean(run, [orc.protected_gemm(A2, B2, dtype, True)])
    # argument checks
    s = run.shape
    assert ab.abft_inject(ctx, run.dA, run.code, s, 0, M, 0, 0, ab.ABFT_INJECT_OPERAND_A) == ab.ABFT_EINVAL
    assert ab.abft_inject(ctx, run.dA, run.code, s, 0, 0, K, 0, ab.ABFT_INJECT_OPERAND_A) == ab.ABFT_EINVAL
    assert ab.abft_inject(ctx, run.dB, run.code, s, 0, N, 0, 0, ab.ABFT_INJECT_OPERAND_B) == ab.ABFT_EINVAL
    assert ab.abft_inject(ctx, run.dB, run.code, s, 0, 0, 0, 8 if dtype == "i8" else 16, ab.ABFT_INJECT_OPERAND_B) == ab.ABFT_EINVAL


@pytest.mark.parametrize("dtype", ["i8", "bf16"])
@pytest.mark.parametrize("M,N,K,batch,trans_b", [(40, 50, 64, 1100, True), (70, 40, 100, 1030, False),
                                                 (36, 300, 128, 1040, True)])
def test_item_kernel_more_items_than_workgroups(dtype, M, N, K, batch, trans_b):
    """More batch items than the kernel launches workgroups (1024): a workgroup takes several items
    in turn, reusing its LDS, and the flagged counts of all its items meet in one ticket.
    (K is kept at 64 or more: the re-check after a correction sums the stored, rounded C of every
    item, and with a much smaller K the tolerance 1e-3 K max|A| max|B| comes within reach of the
    rounding of a row of bf16 values.)"""
    c = ab.abft_create(max_rows=batch * M, max_cols=batch * N, max_depth=batch * 128, max_batch=batch)
    try:
        A, B = gen.gen_operands(dtype, M, N, K, 91, 92, trans_b=trans_b, batch=batch, b_kind="act")
        P = oracle_items(dtype, A, B, trans_b)
        run = Run(c, dtype, A, B, trans_b)
        assert ab.abft_tile_shape(run.code, run.shape) == (M, N)
        run.gemm(ab.ABFT_DETECT)
        check_clean(run, P)
        C_clean = run.C().copy()
        # armed flips in an item of the first turn and in one of the second turn of a workgroup
        bit = 27 if dtype == "i8" else 30
        for bi in (5, 1024 + 5, batch - 1):
            run.inject(bi, M - 1, N - 1, bit, ab.ABFT_INJECT_ACCUMULATOR)
            run.gemm(ab.ABFT_DETECT)
            rf, cf = run.flags()
            cnt = run.cnt()
            assert rf.sum() == 1 and cf.sum() == 1 and rf[bi, M - 1] and cf[bi, N - 1]
            assert cnt[0] == 1 and cnt[1] == 1 and cnt[2] == ab.ABFT_LOCALISED
            run.correct()
            assert np.array_equal(run.C(), C_clean) and run.cnt()[2] == ab.ABFT_CLEAN
        run.dC.fill_(0)
        run.gemm(ab.ABFT_OFF)
        assert np.array_equal(run.C(), C_clean)
    finally:
        ab.abft_destroy(c)


@pytest.mark.parametrize("dtype,M,N,K,batch,trans_b", [("i8", 197, 768, 768, 1, True), ("bf16", 600, 520, 256, 2, True),
                                                       ("bf16", 100, 130, 72, 65, True), ("i8", 70, 50, 40, 64, False)])
def test_calls_can_be_captured_in_a_graph(dtype, M, N, K, batch, trans_b):
    """The hot calls only enqueue kernels (no allocation, no copy, no synchronisation, no memset
    node): a protected GEMM followed by a verify is captured once and replayed several times, with
    eager calls on the same context in between -- a verify of a flipped C, which must flag exactly
    the flipped element, and a protected GEMM with nothing cached, which must give the eager
    vectors -- and every replay must give the eager result again."""
    ctx = ab.abft_create(max_rows=70 * 256, max_cols=70 * 256, max_depth=70 * 128, max_batch=70)
    try:
        A, B = gen.gen_operands(dtype, M, N, K, 95, 96, trans_b=trans_b, batch=batch, b_kind="act" if batch > 1 else "weight")
        run = Run(ctx, dtype, A, B, trans_b)
        res = run.result()
        WS = (ab.ABFT_WS_B_SUM, ab.ABFT_WS_A_SUM, ab.ABFT_WS_CC_PRED, ab.ABFT_WS_RC_PRED, ab.ABFT_WS_CC_OBS, ab.ABFT_WS_RC_OBS)
        run.gemm(ab.ABFT_DETECT)                     # warm-up: kernel attributes are set on first use
        run.verify()
        C_eager = run.dC.clone()
        C_host = run.C().copy()
        vec_eager = [run.ws(w).copy() for w in WS]
        assert run.cnt()[2] == ab.ABFT_CLEAN

        def same_vectors(tag):
            for w, want in zip(WS, vec_eager):
                got = run.ws(w)
                if dtype == "i8":
                    assert np.array_equal(got, want), (tag, w)
                else:       # fp32 atomics: the order of the additions is not fixed
                    assert np.allclose(got, want, rtol=0, atol=1e-3 * max(1.0, float(np.max(np.abs(want))))), (tag, w)

        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                rc1 = ab.abft_gemm(ctx, run.dA, run.dB, run.dC, run.code, ab.ABFT_DETECT, run.shape, res)
                rc2 = ab.abft_verify(ctx, run.dC, run.code, run.shape, res)
        assert rc1 == ab.ABFT_OK and rc2 == ab.ABFT_OK
        torch.cuda.current_stream().wait_stream(side)
        bit = 5 if dtype == "i8" else 14
        for rep in range(4):
            run.dC.fill_(0)
            run.counts.fill_(99)
            run.row_flag.fill_(7)
            run.col_flag.fill_(7)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(run.dC[:, :, :N], C_eager[:, :, :N]), rep
            rf, cf = run.flags()
            assert not rf.any() and not cf.any() and run.cnt()[2] == ab.ABFT_CLEAN, rep
            same_vectors(("replay", rep))
            # eager calls between the replays, on the same context
            bi = rep % batch
            fi, fj = 1, 2
            if dtype != "i8":                        # an element below 2: setting bit 14 makes it huge
                small = np.argwhere(np.abs(orc.decode(C_host[bi], dtype)) < 1.0)
                fi, fj = int(small[rep][0]), int(small[rep][1])
            run.inject(bi, fi, fj, bit)
            run.verify()
            rf, cf = run.flags()
            cnt = run.cnt()
            assert rf.sum() == 1 and cf.sum() == 1 and rf[bi, fi] and cf[bi, fj], rep
            assert cnt[0] == 1 and cnt[1] == 1 and cnt[2] == ab.ABFT_LOCALISED, rep
            if rep % 2:
                run.correct()
                assert run.cnt()[2] == ab.ABFT_CLEAN and torch.equal(run.dC[:, :, :N], C_eager[:, :, :N]), rep
            run.dC.fill_(0)
            run.gemm(ab.ABFT_DETECT)                 # nothing cached: pass over B, GEMM, finish
            assert torch.equal(run.dC[:, :, :N], C_eager[:, :, :N]), rep
            rf, cf = run.flags()
            assert not rf.any() and not cf.any() and run.cnt()[2] == ab.ABFT_CLEAN, rep
            same_vectors(("eager", rep))
        del graph
    finally:
        ab.abft_destroy(ctx)


@pytest.mark.parametrize("dtype,M,N,K", [("bf16", 600, 520, 256), ("f16", 197, 768, 768)])
def test_fault_before_the_stored_sums_is_corrected_to_clean(ctx, dtype, M, N, K):
    """A fault that is in the accumulators when the epilogue sums the values it stores is part of
    those sums.  After abft_correct has recomputed the tile, the sums of its rows and columns are
    the fresh ones: the call ends CLEAN, and so does a later abft_verify."""
    A, B = gen.gen_operands(dtype, M, N, K, 61, 62, trans_b=True)
    run = Run(ctx, dtype, A, B, True)
    run.gemm(ab.ABFT_DETECT | ab.ABFT_STORED_SUMS)
    C_clean = run.C().copy()
    assert run.cnt()[2] == ab.ABFT_CLEAN
    for (i, j, bit) in [(5, 7, 30), (M - 1, N - 1, 30), (300, 33, 30)]:     # |C| < 2: bit 30 set makes it huge
        i = min(i, M - 1)
        run.inject(0, i, j, bit, ab.ABFT_INJECT_ACCUMULATOR)
        run.gemm(ab.ABFT_DETECT | ab.ABFT_STORED_SUMS)
        rf, cf = run.flags()
        assert rf.sum() == 1 and cf.sum() == 1 and rf[0, i] and cf[0, j]
        run.correct()
        cnt = run.cnt()
        assert cnt[2] == ab.ABFT_CLEAN and cnt[3] == 1 and cnt[4] == ab.ABFT_LOCALISED
        assert np.array_equal(run.C(), C_clean)
        run.verify()
        rf, cf = run.flags()
        assert not rf.any() and not cf.any() and run.cnt()[2] == ab.ABFT_CLEAN
        # the tight storage check is still armed: a flip far below tau is seen
        jm = int(np.argmax(np.abs(orc.decode(C_clean[0, 2], dtype))))     # |delta| = |C| / 16: between tau / 100 and tau
        run.inject(0, 2, jm, 3 if dtype == "bf16" else 6)
        run.verify()
        rf, cf = run.flags()
        assert rf[0, 2] and cf[0, jm] and rf.sum() == 1 and cf.sum() == 1
        run.correct()
        assert run.cnt()[2] == ab.ABFT_CLEAN and np.array_equal(run.C(), C_clean)


def _random_shapes():
    rng = np.random.default_rng(20231003)
    out = []
    for _ in range(24):                     # the tiled kernels: up to a few tiles, ragged everywhere
        M, N = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        K = int(rng.choice([1, 7, 16, 31, 64, 100, 128, 129, 200, 256, 384, 512, 640]))
        out.append((M, N, K, int(rng.integers(1, 4)), bool(rng.integers(0, 2))))
    for _ in range(24):                     # the item kernel: every tile configuration, several slabs
        N = int(rng.choice([rng.integers(1, 65), rng.integers(65, 257), rng.integers(257, 641)]))
        M = int(rng.integers(1, 260))
        K = int(rng.integers(1, 130 if N > 256 else (190 if N > 64 else 320)))
        out.append((M, N, K, int(rng.integers(64, 70)), bool(rng.integers(0, 2))))
    return out


@pytest.fixture(scope="module")
def ctx_random():
    c = ab.abft_create(max_rows=70 * 700, max_cols=70 * 700, max_depth=70 * 640, max_batch=70)
    yield c
    ab.abft_destroy(c)


@pytest.mark.parametrize("M,N,K,batch,trans_b", _random_shapes())
def test_seeded_random_shapes(ctx_random, M, N, K, batch, trans_b):
    """Seeded shapes nobody chose by hand, int8 and bf16 alternating (fp16 shares the bf16 code
    but for the conversion): C, every checksum vector, flags, unprotected mode, C's padding."""
    dtype = "i8" if (M + N + K) % 2 else "bf16"
    _clean_case(ctx_random, dtype, M, N, K, batch, trans_b)


def test_two_contexts_on_two_streams():
    """Two contexts, each on its own stream, interleaved call by call: no state is shared between
    contexts, so each stream's results are those of its own problem."""
    c1 = ab.abft_create(max_rows=4096, max_cols=4096, max_depth=4096, max_batch=70)
    c2 = ab.abft_create(max_rows=70 * 256, max_cols=70 * 256, max_depth=70 * 128, max_batch=70)
    try:
        A1, B1 = gen.gen_operands("i8", 600, 520, 256, 101, 102, trans_b=True)
        A2, B2 = gen.gen_operands("bf16", 100, 130, 72, 103, 104, trans_b=True, batch=65, b_kind="act")
        r1, r2 = Run(c1, "i8", A1, B1, True), Run(c2, "bf16", A2, B2, True)
        P1, P2 = oracle_items("i8", A1, B1, True), oracle_items("bf16", A2, B2, True)
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        for _ in range(5):
            with torch.cuda.stream(s1):
                assert ab.abft_gemm(c1, r1.dA, r1.dB, r1.dC, r1.code, ab.ABFT_DETECT, r1.shape, r1.result()) == ab.ABFT_OK
            with torch.cuda.stream(s2):
                assert ab.abft_gemm(c2, r2.dA, r2.dB, r2.dC, r2.code, ab.ABFT_DETECT, r2.shape, r2.result()) == ab.ABFT_OK
            with torch.cuda.stream(s1):
                assert ab.abft_verify(c1, r1.dC, r1.code, r1.shape, r1.result()) == ab.ABFT_OK
            with torch.cuda.stream(s2):
                assert ab.abft_verify(c2, r2.dC, r2.code, r2.shape, r2.result()) == ab.ABFT_OK
        torch.cuda.synchronize()
        check_clean(r1, P1)
        check_clean(r2, P2)
    finally:
        ab.abft_destroy(c1)
        ab.abft_destroy(c2)


def test_two_streams_half_a_step_apart():
    """Two independent batches of one Linear layer, each with a context and a stream of its own,
    the weight shared: every context records an event behind its GEMM kernel
    (abft_gemm_done_event) and the second stream's first call waits for the first stream's GEMM.
    Results must be those of each batch's own problem, in every mode, and the events must have
    been recorded."""
    M, N, K = 1100, 768, 256
    ctxs = [ab.abft_create(max_rows=M, max_cols=N, max_depth=K, max_batch=1) for _ in range(2)]
    try:
        A0, B = gen.gen_operands("bf16", M, N, K, 301, 302, trans_b=True)
        A1, _ = gen.gen_operands("bf16", M, N, K, 303, 302, trans_b=True)
        runs = [Run(ctxs[0], "bf16", A0, B, True), Run(ctxs[1], "bf16", A1, B, True)]
        runs[1].dB = runs[0].dB                                  # one weight tensor for both
        Ps = [oracle_items("bf16", A0, B, True), oracle_items("bf16", A1, B, True)]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        events = []
        for c, st in zip(ctxs, streams):
            ev = torch.cuda.Event()
            ev.record(st)
            assert ab.abft_gemm_done_event(c, ev.cuda_event) == ab.ABFT_OK
            events.append(ev)
        torch.cuda.synchronize()
        for mode in (ab.ABFT_DETECT, ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED, ab.ABFT_OFF, ab.ABFT_DETECT):
            print(f"two streams mode={mode}", flush=True)
            for k in range(6):
                i = k & 1
                r = runs[i]
                if k == 1:
                    streams[1].wait_event(events[0])
                rc = ab.abft_gemm(ctxs[i], r.dA, r.dB, r.dC, r.code, mode, r.shape,
                                  None if mode == ab.ABFT_OFF else r.result(), streams[i].cuda_stream)
                assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
            torch.cuda.synchronize()
            assert events[0].query() and events[1].query()
            if mode != ab.ABFT_OFF:
                check_clean(runs[0], Ps[0])
                check_clean(runs[1], Ps[1])
        assert ab.abft_gemm_done_event(ctxs[0], None) == ab.ABFT_OK
        runs[0].gemm(ab.ABFT_DETECT)
        check_clean(runs[0], Ps[0])
    finally:
        for c in ctxs:
            ab.abft_destroy(c)


@pytest.mark.parametrize("dtype", ["i8", "bf16"])
def test_detect_correct_on_clean_input_leaves_the_fused_verdict(ctx, dtype):
    """A clean DETECT_CORRECT call recomputes nothing and does not re-sum the stored C: flags,
    counts and C are those of a DETECT call; a stored flip afterwards is still found and repaired
    (the correction then sums the stored C itself)."""
    M, N, K = 700, 520, 192
    A, B = gen.gen_operands(dtype, M, N, K, 311, 312, trans_b=True)
    run = Run(ctx, dtype, A, B, True)
    P = oracle_items(dtype, A, B, True)
    run.gemm(ab.ABFT_DETECT)
    C_clean = run.C().copy()
    for rep in range(3):
        run.gemm(ab.ABFT_DETECT_CORRECT)
        cnt = run.cnt()
        rf, cf = run.flags()
        assert not rf.any() and not cf.any()
        assert cnt[0] == 0 and cnt[1] == 0 and cnt[2] == ab.ABFT_CLEAN and cnt[3] == 0 and cnt[4] == ab.ABFT_CLEAN
        assert np.array_equal(run.C(), C_clean)
    check_clean(run, P)
    run.inject(0, 321, 123, 30 if dtype == "i8" else 14)
    run.verify()
    rf, cf = run.flags()
    assert rf[0, 321] and cf[0, 123]
    run.correct()
    assert np.array_equal(run.C(), C_clean) and run.cnt()[2] == ab.ABFT_CLEAN
    # and a fault inside a DETECT_CORRECT call is repaired by that call, clean calls before and after
    run.inject(0, 5, 7, 30, ab.ABFT_INJECT_ACCUMULATOR)
    run.gemm(ab.ABFT_DETECT_CORRECT)
    cnt = run.cnt()
    assert np.array_equal(run.C(), C_clean) and cnt[2] == ab.ABFT_CLEAN and cnt[3] == 1 and cnt[4] == ab.ABFT_LOCALISED
    run.gemm(ab.ABFT_DETECT_CORRECT)
    cnt = run.cnt()
    assert np.array_equal(run.C(), C_clean) and cnt[2] == ab.ABFT_CLEAN and cnt[3] == 0
