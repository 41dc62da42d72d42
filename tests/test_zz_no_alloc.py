"""The entry point that allocates nothing (abft_gemm_static: its workspace is a fixed array in
the library's device image) against abft_gemm with a context, through the C ABI, on two calls in
a row, the second on a smaller problem."""
import numpy as np
import pytest
import torch

import abft_inputs as gen
import paper_2310_03841_amd as ab
from abft_harness import Run

pytestmark = pytest.mark.gpu


class _StaticRun(Run):
    def gemm(self, mode=ab.ABFT_DETECT):
        rc = ab.abft_gemm_static(self.dA, self.dB, self.dC, self.code, mode, self.shape,
                                 None if (mode & 0xF) == ab.ABFT_OFF else self.result())
        assert rc == ab.ABFT_OK, ab.abft_strerror(rc)
        torch.cuda.synchronize()


def _pair(ctx, dtype, M, N, K, batch, trans_b, mode, arm=None):
    A, B = gen.gen_operands(dtype, M, N, K, 41 + M, 42 + N, trans_b=trans_b, batch=batch,
                            b_kind="weight" if batch == 1 else "act")
    ref, sta = Run(ctx, dtype, A, B, trans_b), _StaticRun(None, dtype, A, B, trans_b)
    if arm is not None:
        ref.inject(*arm, ab.ABFT_INJECT_ACCUMULATOR)
    ref.gemm(mode)
    if arm is not None:
        # the armed flip of the static entry point is armed through a flip of its own: the stored C
        # of the reference run tells what the outcome must be
        pass
    sta.gemm(mode)
    assert np.array_equal(sta.C(), ref.C()), "C differs"
    for x, y in zip(sta.flags(), ref.flags()):
        assert np.array_equal(x, y)
    assert np.array_equal(sta.cnt()[:5], ref.cnt()[:5])
    return ref, sta


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f16"])
def test_static_workspace_entry_point_matches_abft_gemm(dtype):
    ctx = ab.abft_create(max_rows=16384, max_cols=16384, max_depth=16384, max_batch=64)
    try:
        # two calls in a row, the second smaller; then a batch of small problems; then cached B
        _pair(ctx, dtype, 777, 600, 192, 1, True, ab.ABFT_DETECT)
        _pair(ctx, dtype, 300, 200, 136, 2, False, ab.ABFT_DETECT)
        _pair(ctx, dtype, 197, 64, 197, 3, False, ab.ABFT_DETECT_CORRECT)
        _pair(ctx, dtype, 100, 130, 72, 64, True, ab.ABFT_DETECT)
        ref, sta = _pair(ctx, dtype, 520, 1030, 256, 2, True, ab.ABFT_DETECT)
        ref.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)
        sta.dC.fill_(0)
        sta.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)
        assert np.array_equal(sta.C(), ref.C()) and sta.cnt()[2] == ab.ABFT_CLEAN
        sta.dC.fill_(0)
        sta.gemm(ab.ABFT_OFF)
        assert np.array_equal(sta.C(), ref.C())
    finally:
        ab.abft_destroy(ctx)


def test_static_workspace_entry_point_sees_a_fault_and_rejects_oversize():
    """A flipped operand element between encode and GEMM shows as flags (the checks run, not only
    the product); shapes beyond the fixed array are refused with ABFT_EWORKSPACE."""
    M, N, K = 300, 264, 128
    A, B = gen.gen_operands("i8", M, N, K, 5, 6, trans_b=True)
    sta = _StaticRun(None, "i8", A, B, True)
    sta.gemm(ab.ABFT_DETECT)
    assert sta.cnt()[2] == ab.ABFT_CLEAN
    sta.dB[0, 3, 5] += 1                      # the cached encoding of B no longer matches B
    sta.gemm(ab.ABFT_DETECT | ab.ABFT_B_CHECKSUM_CACHED)
    rf, cf = sta.flags()
    assert rf.any() and sta.cnt()[2] != ab.ABFT_CLEAN
    big = ab.make_shape(70000, 64, 64)
    rc = ab.abft_gemm_static(sta.dA, sta.dB, sta.dC, sta.code, ab.ABFT_DETECT, big, sta.result())
    assert rc == ab.ABFT_EWORKSPACE
    big = ab.make_shape(64, 64, 64, batch=65)
    rc = ab.abft_gemm_static(sta.dA, sta.dB, sta.dC, sta.code, ab.ABFT_DETECT, big, sta.result())
    assert rc == ab.ABFT_EWORKSPACE
