"""Shared comparison rules for the GPU parity tests."""
import numpy as np

REL_TOL = 2.0 ** -10     # max relative error of an fp16 output against the oracle's fp32 epilogue value
SUBNORMAL_STEP = 2.0 ** -24
FP16_MIN_NORMAL = 2.0 ** -14


def assert_fp16_close(out_gpu_f16, y32, acc=None, what=""):
    """|O - y32| <= 2^-10 |y32| in the fp16 normal range, one subnormal step below it;
    where the integer sum is zero the output must be (signed) zero."""
    o = np.asarray(out_gpu_f16).astype(np.float64)
    y = np.asarray(y32).astype(np.float64)
    assert o.shape == y.shape, (what, o.shape, y.shape)
    finite = np.abs(y) < 65520.0
    assert np.all(np.isfinite(o[finite])), what
    assert np.all(np.isinf(o[~finite])), what
    err = np.abs(o - y)
    normal = finite & (np.abs(y) >= FP16_MIN_NORMAL)
    small = finite & ~normal
    bad = (normal & (err > REL_TOL * np.abs(y))) | (small & (err > SUBNORMAL_STEP))
    if bad.any():
        i = np.argwhere(bad)[0]
        raise AssertionError(f"{what}: {bad.sum()} outputs out of tolerance, first at {tuple(i)}: "
                             f"gpu {o[tuple(i)]!r} oracle {y[tuple(i)]!r}")
    if acc is not None:
        z = np.asarray(acc) == 0
        assert not o[z].any(), what


def assert_equal_bits(a, b, what=""):
    a = np.asarray(a)
    b = np.asarray(b)
    assert a.shape == b.shape and a.dtype == b.dtype, (what, a.shape, b.shape, a.dtype, b.dtype)
    if not np.array_equal(a, b):
        i = np.argwhere(a != b)
        raise AssertionError(f"{what}: {len(i)} mismatches, first at {tuple(i[0])}: gpu {a[tuple(i[0])]} oracle {b[tuple(i[0])]}")
