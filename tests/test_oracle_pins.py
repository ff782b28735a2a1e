"""Pins of the CPU oracle against things other than itself: values the paper
prints, exact integer / rational arithmetic, closed forms, invariants and
library routines.  All CPU-only."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2311_09550_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- helpers

def fp32_round(fr: Fraction) -> Fraction:
    """Exact round-half-to-even of a rational to the nearest fp32 (normal range only)."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = 0
    while a >= Fraction(2) ** (e + 24):
        e += 1
    while a < Fraction(2) ** (e + 23):
        e -= 1
    assert -149 <= e <= 104
    scaled = a / Fraction(2) ** e  # in [2^23, 2^24)
    q = scaled.numerator // scaled.denominator
    rem = scaled - q
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and q % 2 == 1):
        q += 1
    return sign * q * Fraction(2) ** e


def rne_int(fr: Fraction) -> int:
    q = math.floor(fr)
    rem = fr - q
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and q % 2 == 1):
        q += 1
    return q


def exact_quantize_row(vals, qmax, qmin, denom):
    """Eq. (2) with z = 0 in exact rational arithmetic with explicit fp32 roundings."""
    fr = [Fraction(float(v)) for v in vals]
    amax = max(abs(v) for v in fr)
    if amax == 0:
        return [0] * len(fr), Fraction(0)
    scale = fp32_round(amax / denom)
    codes = []
    for v in fr:
        q = fp32_round(v / scale)
        codes.append(int(min(qmax, max(qmin, rne_int(q)))))
    return codes, scale


# -------------------------------------------------------------------- fp16

def test_half_to_float_all_bit_patterns_match_numpy(oracle):
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.half_to_float(h)
    want = h.view(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(want)], want.view(np.uint32)[~np.isnan(want)])
    assert np.all(np.isnan(got[np.isnan(want)]))


def test_float_to_half_matches_numpy_rne(oracle):
    g = synth.rng(900)
    # every fp16 value, every midpoint between neighbours, and points just off the midpoints
    h = np.arange(0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mids = (h[:-1] + h[1:]) / 2
    pts = np.concatenate([h, mids, np.nextafter(mids.astype(np.float32), np.float32(np.inf)).astype(np.float64),
                          np.nextafter(mids.astype(np.float32), np.float32(-np.inf)).astype(np.float64),
                          [65504.0, 65519.99, 65520.0, 65536.0, 1e6, 2.0 ** -25, 2.0 ** -24, 1.5 * 2.0 ** -24]])
    pts = np.concatenate([pts, -pts]).astype(np.float32)
    rnd = (g.standard_normal(200000) * np.exp(g.uniform(-20, 12, 200000))).astype(np.float32)
    f = np.concatenate([pts, rnd])
    got = oracle.float_to_half(f)
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want)


def test_double_to_half_single_rounding(oracle):
    # 1 + 2^-11 + 2^-30 lies just above a tie: direct rounding goes up, double rounding via fp32 would tie to even (down)
    d = np.array([1.0 + 2.0 ** -11 + 2.0 ** -30, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11], np.float64)
    got = oracle.double_to_half(d).view(np.float16).astype(np.float64)
    assert list(got) == [1.0 + 2.0 ** -10, 1.0, 1.0 + 2 * 2.0 ** -10]


# -------------------------------------------------------------- pack/unpack

def test_paper_worked_example_minus_seven(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "sint4_worked_example.txt")) if l.strip() and l[0] != "#"]
    assert rows
    for value, twos, nibble, byte_hi, as_int8, _uint4 in rows:
        value, nib, as_int8 = int(value), int(nibble, 2), int(as_int8)
        assert format(value & 0xFF, "08b") == twos
        wp = oracle.pack_w4(np.array([[value, 0]], np.int8))
        assert wp[0, 0] & 15 == nib                      # the low four bits of the two's complement are packed
        assert oracle.unpack_w4(wp)[0, 0] == value
        assert format(nib << 4, "08b") == byte_hi
        assert oracle.nibble_in_high_half_as_int8(nib) == as_int8 == 16 * value
        assert as_int8 >> 4 == value                     # dividing by 16 restores the value


def test_all_nibbles_high_half_is_times_16(oracle):
    for v in range(-8, 8):
        nib = v & 15
        assert oracle.nibble_in_high_half_as_int8(nib) == 16 * v


def test_pack_layout_and_roundtrip_all_bytes(oracle):
    # every byte value: low nibble is k even, high nibble is k odd
    b = np.arange(256, dtype=np.uint8).reshape(1, 256)
    wq = oracle.unpack_w4(b)
    assert wq.shape == (1, 512)
    for byte in range(256):
        lo, hi = byte & 15, byte >> 4
        assert wq[0, 2 * byte] == (lo - 16 if lo >= 8 else lo)
        assert wq[0, 2 * byte + 1] == (hi - 16 if hi >= 8 else hi)
    assert np.array_equal(oracle.pack_w4(wq), b)
    # all 16 x 16 ordered pairs of values
    pairs = np.array([[a, c] for a in range(-8, 8) for c in range(-8, 8)], np.int8).reshape(1, -1)
    assert np.array_equal(oracle.unpack_w4(oracle.pack_w4(pairs)), pairs)


def test_pack_rejects_out_of_range(oracle):
    with pytest.raises(ValueError):
        oracle.pack_w4(np.array([[8, 0]], np.int8))
    with pytest.raises(ValueError):
        oracle.pack_w4(np.array([[0, -9]], np.int8))


# --------------------------------------------------------------------- acc

@pytest.mark.parametrize("M,N,K", [(1, 1, 2), (3, 5, 6), (8, 7, 64), (2, 3, 34)])
def test_acc_vs_int64_brute_force(oracle, M, N, K):
    g = synth.rng(901, M, N, K)
    xq = g.integers(-128, 128, size=(M, K), dtype=np.int8)
    wq = g.integers(-8, 8, size=(N, K), dtype=np.int8)
    # extremes in the corners
    xq[0, :] = -128
    wq[0, :] = -8
    if M > 1:
        xq[1, :] = 127
    if N > 1:
        wq[1, :] = 7
    acc = oracle.gemm_acc_i32(xq, oracle.pack_w4(wq))
    for m in range(M):
        for n in range(N):
            s = 0
            for k in range(K):
                s += int(xq[m, k]) * int(wq[n, k])
            assert int(acc[m, n]) == s


def test_acc_vs_float64_blas(oracle):
    # every partial sum is an integer far below 2^53, so dgemm is exact
    xq, wq, _, _ = synth.uniform_codes(8, 1024, 1024)
    acc = oracle.gemm_acc_i32(xq, oracle.pack_w4(wq))
    want = xq.astype(np.float64) @ wq.astype(np.float64).T
    assert np.array_equal(acc.astype(np.float64), want)


def test_acc_closed_forms_and_no_overflow(oracle):
    K = 28672  # largest K of the workloads
    xq = np.full((2, K), 127, np.int8)
    xq[1, :] = -128
    wq = np.full((2, K), -8, np.int8)
    wq[1, :] = 7
    acc = oracle.gemm_acc_i32(xq, oracle.pack_w4(wq))
    assert acc[0, 0] == 127 * -8 * K == -29130752
    assert acc[1, 0] == -128 * -8 * K
    assert acc[0, 1] == 127 * 7 * K
    # the sixteen-fold accumulator of the sign-bit trick still fits int32 (Sec. 5.3: no overflow)
    assert abs(16 * int(acc[1, 0])) < 2 ** 31 and 16 * int(acc[0, 0]) == -466092032


def test_acc_invariants(oracle):
    g = synth.rng(902)
    M, N, K = 5, 12, 96
    xq = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    # zero weights give zero output
    assert not oracle.gemm_acc_i32(xq, np.zeros((N, K // 2), np.uint8)).any()
    # a single +-1 weight selects (or negates) one activation column
    wq = np.zeros((N, K), np.int8)
    ks = g.integers(0, K, size=N)
    sg = g.choice([-1, 1], size=N).astype(np.int8)
    wq[np.arange(N), ks] = sg
    acc = oracle.gemm_acc_i32(xq, oracle.pack_w4(wq))
    assert np.array_equal(acc, xq[:, ks].astype(np.int32) * sg.astype(np.int32))
    # the same permutation of k applied to both operands leaves acc unchanged
    wq = g.integers(-8, 8, size=(N, K), dtype=np.int8)
    perm = g.permutation(K)
    a0 = oracle.gemm_acc_i32(xq, oracle.pack_w4(wq))
    a1 = oracle.gemm_acc_i32(np.ascontiguousarray(xq[:, perm]), oracle.pack_w4(np.ascontiguousarray(wq[:, perm])))
    assert np.array_equal(a0, a1)
    # transposed operands are not interchangeable: X W^T, not W X^T (N != M here)
    assert a0.shape == (M, N)
    # additivity over a split of K
    h = K // 2
    left = oracle.gemm_acc_i32(np.ascontiguousarray(xq[:, :h]), oracle.pack_w4(np.ascontiguousarray(wq[:, :h])))
    right = oracle.gemm_acc_i32(np.ascontiguousarray(xq[:, h:]), oracle.pack_w4(np.ascontiguousarray(wq[:, h:])))
    assert np.array_equal(a0, left + right)


# ---------------------------------------------------------------- epilogue

def test_epilogue_unit_scales_are_exact(oracle):
    acc = np.arange(-2048, 2049, dtype=np.int32).reshape(1, -1)
    y32, out = oracle.epilogue(acc, np.ones(1, np.float32), np.ones(acc.shape[1], np.float32))
    assert np.array_equal(y32, acc.astype(np.float32))
    assert np.array_equal(out.astype(np.int32), acc)      # |acc| <= 2048 is exact in fp16


def test_epilogue_linear_in_scales(oracle):
    xq, wq, s_a, s_w = synth.uniform_codes(8, 256, 128)
    acc = oracle.gemm_acc_i32(xq, oracle.pack_w4(wq))
    y, o = oracle.epilogue(acc, s_a, s_w)
    y2, o2 = oracle.epilogue(acc, 2 * s_a, s_w)
    y3, o3 = oracle.epilogue(acc, s_a, 4 * s_w)
    assert np.array_equal(y2, 2 * y) and np.array_equal(y3, 4 * y)
    assert np.array_equal(o2.astype(np.float32), 2 * o.astype(np.float32))
    assert np.array_equal(o3.astype(np.float32), 4 * o.astype(np.float32))
    # s_a indexes rows, s_w indexes columns
    s_a1 = s_a.copy(); s_a1[3] *= 2
    y4, _ = oracle.epilogue(acc, s_a1, s_w)
    assert np.array_equal(y4[3], 2 * y[3]) and np.array_equal(np.delete(y4, 3, 0), np.delete(y, 3, 0))
    s_w1 = s_w.copy(); s_w1[17] *= 2
    y5, _ = oracle.epilogue(acc, s_a, s_w1)
    assert np.array_equal(y5[:, 17], 2 * y[:, 17]) and np.array_equal(np.delete(y5, 17, 1), np.delete(y, 17, 1))


def test_epilogue_closed_form_exact_rational(oracle):
    # Eq. (6),(7): y = fp32( fp32(acc) * fp32(s_a * s_w) ), then one rounding to fp16
    acc = np.array([[16777217, -29130752, 3, 0], [-1, 123456789, 2 ** 24 + 3, 7]], np.int32)
    s_a = np.array([0.0037, 0.0091], np.float32)
    s_w = np.array([0.0012, 0.0055, 0.00999, 1e-3], np.float32)
    y32, out = oracle.epilogue(acc, s_a, s_w)
    for m in range(2):
        for n in range(4):
            s = fp32_round(Fraction(float(s_a[m])) * Fraction(float(s_w[n])))
            a = fp32_round(Fraction(int(acc[m, n])))
            y = fp32_round(a * s)
            assert Fraction(float(y32[m, n])) == y
            with np.errstate(over="ignore"):
                assert out[m, n] == np.float32(float(y)).astype(np.float16) or (
                    np.isinf(out[m, n]) and abs(y) >= 65520)


def test_epilogue_zero_acc_gives_zero(oracle):
    acc = np.zeros((2, 3), np.int32)
    y32, out = oracle.epilogue(acc, np.array([0.5, 0.0], np.float32), np.ones(3, np.float32))
    assert not y32.any() and not out.astype(np.float32).any()


# --------------------------------------------------------------- quantiser

def test_quantizer_exact_rational_small_rows(oracle):
    g = synth.rng(903)
    rows = [g.standard_normal(64).astype(np.float16) * np.float16(s) for s in (1.0, 0.01, 37.0, 300.0)]
    rows.append(np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5] + [0.0] * 56, np.float16))  # ties, s_a = 1
    x = np.stack(rows)
    xq, s_a = oracle.quantize_act(x)
    for r in range(x.shape[0]):
        codes, scale = exact_quantize_row(x[r], 127, -127, 127)
        assert Fraction(float(s_a[r])) == scale
        assert list(xq[r]) == codes


def test_quantizer_ties_round_half_to_even(oracle):
    x = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 126.5, -126.5]], np.float16)
    xq, s_a = oracle.quantize_act(x)
    assert s_a[0] == 1.0
    assert list(xq[0]) == [127, 0, 2, 2, 0, -2, -2, 4, 126, -126]


def test_quantizer_properties(oracle):
    x = synth.activations_fp16(16, 512, tag=5)
    xq, s_a = oracle.quantize_act(x)
    xf = x.astype(np.float64)
    amax = np.abs(xf).max(axis=1)
    assert np.array_equal(s_a, (amax.astype(np.float32) / np.float32(127.0)))
    # the row maximum maps to +-127 and nothing exceeds it
    assert np.array_equal(np.abs(xq).max(axis=1), np.full(16, 127))
    am = np.abs(xf).argmax(axis=1)
    assert np.array_equal(xq[np.arange(16), am], (127 * np.sign(xf[np.arange(16), am])).astype(np.int8))
    # reconstruction error at most half a step (plus fp32 rounding of the quotient)
    err = np.abs(xf - xq.astype(np.float64) * s_a[:, None].astype(np.float64))
    assert np.all(err <= 0.5 * s_a[:, None].astype(np.float64) * (1 + 2.0 ** -20))
    # sign symmetry and invariance of the codes under a power-of-two rescale of the row
    xq_neg, s_neg = oracle.quantize_act(-x)
    assert np.array_equal(xq_neg, -xq) and np.array_equal(s_neg, s_a)
    xq2, s2 = oracle.quantize_act((x.astype(np.float32) * 2).astype(np.float16))
    assert np.array_equal(xq2, xq) and np.array_equal(s2, 2 * s_a)


def test_quantizer_zero_row_and_row_independence(oracle):
    x = synth.activations_fp16(4, 128, tag=6)
    x[2, :] = 0
    xq, s_a = oracle.quantize_act(x)
    assert s_a[2] == 0.0 and not xq[2].any() and np.all(np.isfinite(s_a))
    # each token has its own scale: changing one row leaves the others alone
    y = x.copy(); y[0, 3] = np.float16(1000.0)
    yq, t_a = oracle.quantize_act(y)
    assert np.array_equal(yq[1:], xq[1:]) and np.array_equal(t_a[1:], s_a[1:]) and t_a[0] != s_a[0]


def test_quantizer_division_not_reciprocal_multiply(oracle):
    """Eq. (2) divides by the scale.  Find inputs where x * (1/s) or x * (127/amax) would give a
    different int8 code, and check the oracle agrees with exact division there."""
    g = synth.rng(904)
    found = 0
    for _ in range(400):
        x = (g.standard_normal(256) * g.uniform(0.1, 30)).astype(np.float16)
        xf = x.astype(np.float32)
        amax = np.abs(xf).max()
        s = np.float32(amax / np.float32(127.0))
        by_div = np.rint(xf / s)
        by_rcp = np.rint(xf * (np.float32(1.0) / s))
        by_inv = np.rint(xf * (np.float32(127.0) / amax))
        differs = (by_div != by_rcp) | (by_div != by_inv)
        if differs.any():
            found += 1
            xq, _ = oracle.quantize_act(x[None, :])
            codes, _ = exact_quantize_row(x, 127, -127, 127)
            assert list(xq[0]) == codes
    assert found >= 3  # such inputs exist, so the distinction is tested


# -------------------------------------------------------------- weight RTN

def test_weight_rtn_eq8_eq9(oracle):
    w = synth.weights_fp16(32, 256)
    w[5, :] = 0
    w[6, 0] = np.float16(-1.0)          # negative extreme sets the scale
    wq, s_w = oracle.quantize_weights_rtn(w)
    wf = w.astype(np.float64)
    top = np.maximum(np.abs(wf.max(axis=1)), np.abs(wf.min(axis=1)))
    assert np.array_equal(s_w, top.astype(np.float32) / np.float32(7.0))
    assert wq.min() >= -7 and wq.max() <= 7        # with gamma = beta = 1 plain RTN never reaches -8
    nz = top > 0
    assert np.array_equal(np.abs(wq[nz]).max(axis=1), np.full(nz.sum(), 7))
    assert wq[6, 0] == -7 and s_w[5] == 0 and not wq[5].any()
    err = np.abs(wf - wq * s_w[:, None].astype(np.float64))
    assert np.all(err <= 0.5 * s_w[:, None] * (1 + 2.0 ** -20))
    for r in (0, 6, 31):
        codes, scale = exact_quantize_row(w[r], 7, -8, 7)
        assert list(wq[r]) == codes and Fraction(float(s_w[r])) == scale


def test_weight_clipping_eq8_eq9_with_strengths(oracle):
    """Eq. (8),(9) with clipping strengths gamma, beta per channel."""
    # without strengths it is the plain RTN, bit for bit
    w = synth.weights_fp16(24, 128)
    a, sa = oracle.quantize_weights_clip(w)
    b, sb = oracle.quantize_weights_rtn(w)
    assert np.array_equal(a, b) and np.array_equal(sa.view(np.uint32), sb.view(np.uint32))
    ones = np.ones(24, np.float32)
    c, sc = oracle.quantize_weights_clip(w, ones, ones)
    assert np.array_equal(c, b) and np.array_equal(sc.view(np.uint32), sb.view(np.uint32))

    # hand-worked row, every value, the scale and every quotient exact: max 1.75, min -3.5, gamma = 1/2, beta = 1/4
    # => S = max(|0.5 * 1.75|, |0.25 * -3.5|) / 7 = 0.875 / 7 = 1/8; codes = clamp(rne(8 w), -8, 7)
    row = np.array([[1.75, -3.5, 0.875, 0.4375, -0.4375, 0.0, 0.1875, -0.1875, 0.3125, -0.3125, -0.875, -1.0625, 0.9375,
                     0.0625]], np.float16)
    wq, s = oracle.quantize_weights_clip(row, np.float32([0.5]), np.float32([0.25]))
    assert float(s[0]) == 0.125
    # 8 w =      14   -28  7  3.5  -3.5 0  1.5 -1.5  2.5 -2.5  -7  -8.5  7.5  0.5   (ties go to the even integer)
    assert list(wq[0]) == [7, -8, 7, 4, -4, 0, 2, -2, 2, -2, -7, -8, 7, 0]

    # the paper's illustration: a range (-0.4, 0.2) narrowed to about (-0.2, 0.2) by halving beta
    row = np.array([[-0.4, 0.2, -0.1, 0.1, 0.05, -0.2, -0.3]], np.float16)
    wq, s = oracle.quantize_weights_clip(row, None, np.float32([0.5]))
    codes, scale = exact_quantize_row(np.array([0.2], np.float16), 7, -8, 7)      # S = fp16(0.2) / 7
    assert Fraction(float(s[0])) == scale and codes == [7]
    assert wq[0, 0] == -8 and wq[0, 1] == 7 and wq[0, 6] == -8 and wq[0, 5] == -7
    lo, hi = -8 * float(s[0]), 7 * float(s[0])
    assert -0.23 < lo < -0.22 and abs(hi - 0.2) < 1e-3

    # properties on random rows: saturation outside the clipped range, half-step error inside, exact rational codes
    g = synth.rng(906)
    w = synth.weights_fp16(16, 256, config_id=7)
    gamma = g.uniform(0.3, 1.0, 16).astype(np.float32)
    beta = g.uniform(0.3, 1.0, 16).astype(np.float32)
    wq, s = oracle.quantize_weights_clip(w, gamma, beta)
    wf = w.astype(np.float64)
    assert wq.min() == -8 and wq.max() == 7
    inside = (wf >= -8.5 * s[:, None]) & (wf <= 7.5 * s[:, None])
    err = np.abs(wf - wq * s[:, None].astype(np.float64))
    assert np.all(err[inside] <= 0.5 * np.broadcast_to(s[:, None], wf.shape)[inside] * (1 + 2.0 ** -20))
    assert np.all(wq[wf > 7.5 * s[:, None]] == 7) and np.all(wq[wf < -8.5 * s[:, None]] == -8)
    for r in (0, 9):
        fr = [Fraction(float(v)) for v in w[r]]
        up = abs(fp32_round(Fraction(float(gamma[r])) * max(fr)))
        down = abs(fp32_round(Fraction(float(beta[r])) * min(fr)))
        scale = fp32_round(max(up, down) / 7)
        assert Fraction(float(s[r])) == scale
        assert list(wq[r]) == [int(min(7, max(-8, rne_int(fp32_round(v / scale))))) for v in fr]


# ------------------------------------------------- vanilla unsigned storage

def test_u4_paper_worked_example_and_equivalence_with_signed_storage(oracle):
    """App. A.1: -7 plus 8 is stored as 0000 0001; subtracting 8 on the device gives the signed code back, so the sum
    over unsigned nibbles equals the sum over the signed format of the same codes."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "sint4_worked_example.txt")) if l.strip() and l[0] != "#"]
    for value, _twos, _nibble, _hi, _as_int8, uint4 in rows:
        value, u = int(value), int(uint4, 2)
        assert u == value + 8 and oracle.pack_u4(np.array([[u, 8]]))[0, 0] == (u | (8 << 4))
        x = np.array([[3, 5]], np.int8)
        assert oracle.gemm_acc_i32_u4(x, oracle.pack_u4(np.array([[u, 8]])))[0, 0] == 3 * value
    g = synth.rng(909)
    xq = g.integers(-128, 128, size=(6, 192), dtype=np.int8)
    wq = g.integers(-8, 8, size=(20, 192), dtype=np.int8)
    wq[0, :] = -8
    wq[1, :] = 7
    acc_u = oracle.gemm_acc_i32_u4(xq, oracle.pack_u4(wq.astype(np.int16) + 8))
    assert np.array_equal(acc_u, oracle.gemm_acc_i32(xq, oracle.pack_w4(wq)))
    # int64 brute force and the closed form sum x*u - 8*sum x
    u = (wq.astype(np.int64) + 8)
    want = xq.astype(np.int64) @ u.T - 8 * xq.astype(np.int64).sum(axis=1, keepdims=True)
    assert np.array_equal(acc_u.astype(np.int64), want)
    for m in range(2):
        for n in range(3):
            assert int(acc_u[m, n]) == sum(int(xq[m, k]) * (int(u[n, k]) - 8) for k in range(192))
    with pytest.raises(ValueError):
        oracle.pack_u4(np.array([[16, 0]]))


# --------------------------------------------------------------------- W8A8

@pytest.mark.parametrize("M,N,K", [(1, 1, 2), (3, 5, 6), (8, 7, 64), (2, 3, 34)])
def test_w8_acc_vs_int64_brute_force(oracle, M, N, K):
    g = synth.rng(907, M, N, K)
    xq = g.integers(-128, 128, size=(M, K), dtype=np.int8)
    w8 = g.integers(-128, 128, size=(N, K), dtype=np.int8)
    xq[0, :] = -128
    w8[0, :] = -128
    if N > 1:
        w8[1, :] = 127
    acc = oracle.gemm_acc_i32_w8(xq, w8)
    for m in range(M):
        for n in range(N):
            assert int(acc[m, n]) == sum(int(xq[m, k]) * int(w8[n, k]) for k in range(K))


def test_w8_acc_blas_closed_forms_and_the_int4_special_case(oracle):
    g = synth.rng(908)
    xq = g.integers(-127, 128, size=(8, 1024), dtype=np.int8)
    w8 = g.integers(-128, 128, size=(96, 1024), dtype=np.int8)
    acc = oracle.gemm_acc_i32_w8(xq, w8)
    assert np.array_equal(acc.astype(np.float64), xq.astype(np.float64) @ w8.astype(np.float64).T)   # exact in dgemm
    # largest magnitude at the largest K of the contract stays inside int32
    K = 65536
    a = oracle.gemm_acc_i32_w8(np.full((1, K), -128, np.int8), np.stack([np.full(K, -128, np.int8), np.full(K, 127, np.int8)]))
    assert a[0, 0] == 128 * 128 * K == 2 ** 30 and a[0, 1] == -128 * 127 * K
    # codes that fit four bits: the W8A8 sum is the W4A8 sum of the same codes (two independent loops agree)
    w4 = g.integers(-8, 8, size=(40, 1024), dtype=np.int8)
    assert np.array_equal(oracle.gemm_acc_i32_w8(xq, w4), oracle.gemm_acc_i32(xq, oracle.pack_w4(w4)))
    # a single +-1 weight selects (or negates) an activation column; permuting k in both operands changes nothing
    sel = np.zeros((2, 1024), np.int8)
    sel[0, 77] = 1
    sel[1, 1000] = -1
    s = oracle.gemm_acc_i32_w8(xq, sel)
    assert np.array_equal(s[:, 0], xq[:, 77].astype(np.int32)) and np.array_equal(s[:, 1], -xq[:, 1000].astype(np.int32))
    perm = g.permutation(1024)
    assert np.array_equal(oracle.gemm_acc_i32_w8(xq[:, perm], w8[:, perm]), acc)


def test_w8_weight_rtn_eq8_eq9_eight_bits(oracle):
    w = synth.weights_fp16(24, 256, config_id=9)
    w[5, :] = 0
    w[6, 0] = np.float16(-1.0)
    wq, s_w = oracle.quantize_weights_rtn8(w)
    wf = w.astype(np.float64)
    top = np.abs(wf).max(axis=1)
    assert np.array_equal(s_w, top.astype(np.float32) / np.float32(127.0))
    assert wq.min() >= -127 and wq.max() <= 127
    nz = top > 0
    assert np.array_equal(np.abs(wq[nz].astype(np.int32)).max(axis=1), np.full(nz.sum(), 127))
    assert wq[6, 0] == -127 and s_w[5] == 0 and not wq[5].any()
    err = np.abs(wf - wq * s_w[:, None].astype(np.float64))
    assert np.all(err <= 0.5 * s_w[:, None] * (1 + 2.0 ** -20))
    for r in (0, 6, 23):
        codes, scale = exact_quantize_row(w[r], 127, -128, 127)
        assert list(wq[r]) == codes and Fraction(float(s_w[r])) == scale
    # it is the per-token activation quantiser applied to weight rows (same formula, same rounding)
    xq, s_a = oracle.quantize_act(w)
    assert np.array_equal(xq, wq) and np.array_equal(s_a.view(np.uint32), s_w.view(np.uint32))


# --------------------------------------------------------------------- glue

def test_silu_mul_vs_library_and_identities(oracle):
    torch = pytest.importorskip("torch")
    g = synth.rng(905)
    I = 96
    gu = (g.standard_normal((4, 2 * I)) * 3).astype(np.float16)
    gu[0, 0] = 0.0
    y64, h = oracle.silu_mul(gu)
    gate = torch.from_numpy(gu[:, :I].astype(np.float64))
    up = torch.from_numpy(gu[:, I:].astype(np.float64))
    want = (torch.nn.functional.silu(gate) * up).numpy()
    assert np.allclose(y64, want, rtol=1e-14, atol=0)
    assert y64[0, 0] == 0.0
    # silu(x) - silu(-x) = x
    gneg = gu.copy(); gneg[:, :I] = -gu[:, :I]
    y64n, _ = oracle.silu_mul(gneg)
    assert np.allclose(y64 - y64n, gu[:, :I].astype(np.float64) * gu[:, I:].astype(np.float64), rtol=1e-13, atol=1e-300)
    assert np.array_equal(h, y64.astype(np.float16))


# --------------------------------------------------------------- end to end

def test_w4a8_linear_tracks_the_fp_matmul(oracle):
    """Loose statistical check, not a parity criterion: the quantised linear approximates X W^T."""
    M, N, K = 8, 256, 1024
    x = synth.activations_fp16(M, K, tag=7)
    w = synth.weights_fp16(N, K)
    xq, s_a = oracle.quantize_act(x)
    wq, s_w = oracle.quantize_weights_rtn(w)
    _, y32, out = oracle.gemm(xq, s_a, oracle.pack_w4(wq), s_w)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    rel = np.linalg.norm(y32 - ref) / np.linalg.norm(ref)
    assert rel < 0.25
    assert np.corrcoef(y32.ravel(), ref.ravel())[0, 1] > 0.97
    assert np.allclose(out.astype(np.float32), y32, rtol=2.0 ** -10, atol=2.0 ** -24)


# ------------------------------------------------ fine-grained comparison

def test_fine_grained_hand_worked_example(oracle):
    """Two groups of 128, two channels with different scales (a transposed scale array would swap them):
    channel 0: 128 * 1 * 0.5 + 128 * (-2) * 0.125 = 64 - 32 = 32, times s_a = 2 -> 64;
    channel 1: 128 * 3 * 0.25 + 128 * (-1) * 1.0 = 96 - 128 = -32, times 2 -> -64."""
    xq = np.ones((1, 256), np.int8)
    wq = np.empty((2, 256), np.int8)
    wq[0, :128], wq[0, 128:] = 1, -2
    wq[1, :128], wq[1, 128:] = 3, -1
    s_g = np.array([[0.5, 0.25], [0.125, 1.0]], np.float32)   # [group][channel]
    y64, y32, out, mag = oracle.gemm_fine_grained(xq, np.array([2.0], np.float32), oracle.pack_w4(wq), s_g)
    assert y64.tolist() == [[64.0, -64.0]] and y32.tolist() == [[64.0, -64.0]]
    assert out.astype(np.float64).tolist() == [[64.0, -64.0]]
    assert mag.tolist() == [[192.0, 448.0]]


def test_fine_grained_equals_dequantise_first_matmul(oracle):
    """Scaling each group's integer sum equals multiplying by weights dequantised group-wise beforehand
    (the W4A16-shaped Eq. (4)): checked against a float64 library matmul."""
    M, N, K = 9, 37, 640
    xq, wq, s_a, _ = synth.uniform_codes(M, N, K, config_id=60)
    s_g = synth.group_scales(N, K, 128, config_id=60)
    y64, y32, out, mag = oracle.gemm_fine_grained(xq, s_a, oracle.pack_w4(wq), s_g)
    w_deq = wq.astype(np.float64) * np.repeat(s_g.astype(np.float64).T, 128, axis=1)   # [N][K]
    ref = s_a.astype(np.float64)[:, None] * (xq.astype(np.float64) @ w_deq.T)
    assert np.all(np.abs(y64 - ref) <= 1e-13 * mag + 1e-300)
    # fp32 chain: one rounding per group term plus the final product
    assert np.all(np.abs(y32.astype(np.float64) - y64) <= (K // 128 + 2) * 2.0 ** -24 * mag)
    assert np.all(np.abs(out.astype(np.float64) - y32.astype(np.float64)) <= 2.0 ** -11 * np.abs(y32) + 2.0 ** -25)
    assert np.all(mag >= np.abs(y64))
    # other group sizes follow the same definition
    for group in (32, 64, 320, 640):
        sg = synth.group_scales(N, K, group, config_id=61)
        y = oracle.gemm_fine_grained(xq, s_a, oracle.pack_w4(wq), sg, group)[0]
        wd = wq.astype(np.float64) * np.repeat(sg.astype(np.float64).T, group, axis=1)
        ref = s_a.astype(np.float64)[:, None] * (xq.astype(np.float64) @ wd.T)
        assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_fine_grained_reduces_to_per_channel(oracle):
    """With the same scale in every group of a channel, and with one group spanning all of K, Eq. (5) is Eq. (6)."""
    M, N, K = 7, 21, 512
    xq, wq, s_a, s_w = synth.uniform_codes(M, N, K, config_id=62)
    wp = oracle.pack_w4(wq)
    acc = oracle.gemm_acc_i32(xq, wp)
    exact = acc.astype(np.float64) * s_a.astype(np.float64)[:, None] * s_w.astype(np.float64)[None, :]
    y64 = oracle.gemm_fine_grained(xq, s_a, wp, np.tile(s_w, (4, 1)))[0]
    assert np.allclose(y64, exact, rtol=1e-14, atol=0)
    y64, y32, _, _ = oracle.gemm_fine_grained(xq, s_a, wp, s_w.reshape(1, N), group=K)
    assert np.allclose(y64, exact, rtol=1e-15, atol=0)
    # a single group: fma(float(acc), s, 0) * s_a, two fp32 roundings, in exact rational arithmetic
    for m in range(M):
        for n in range(0, N, 5):
            want = fp32_round(fp32_round(Fraction(int(acc[m, n])) * Fraction(float(s_w[n]))) * Fraction(float(s_a[m])))
            assert Fraction(float(y32[m, n])) == want


def test_fine_grained_fp32_chain_in_exact_rational_arithmetic(oracle):
    """The fp32 result is a chain of fused multiply-adds in ascending group order (one rounding each), then one
    product with s_a: replayed with exact rationals and explicit roundings on small inputs."""
    M, N, K, group = 3, 4, 384, 64
    xq, wq, s_a, _ = synth.uniform_codes(M, N, K, config_id=63)
    s_g = synth.group_scales(N, K, group, config_id=63)
    _, y32, out, _ = oracle.gemm_fine_grained(xq, s_a, oracle.pack_w4(wq), s_g, group)
    differs_from_unfused = 0
    for m in range(M):
        for n in range(N):
            f = Fraction(0)
            unfused = Fraction(0)
            for g in range(K // group):
                s = int(np.dot(xq[m, g * group:(g + 1) * group].astype(np.int64), wq[n, g * group:(g + 1) * group].astype(np.int64)))
                f = fp32_round(Fraction(s) * Fraction(float(s_g[g, n])) + f)
                unfused = fp32_round(fp32_round(Fraction(s) * Fraction(float(s_g[g, n]))) + unfused)
            want = fp32_round(f * Fraction(float(s_a[m])))
            assert Fraction(float(y32[m, n])) == want
            assert float(out[m, n]) == float(np.float32(float(want)).astype(np.float16))
            differs_from_unfused += fp32_round(unfused * Fraction(float(s_a[m]))) != want
    assert differs_from_unfused > 0   # the check above tells a fused chain from a multiply-then-add one


def test_group_weight_quantiser(oracle):
    """Group-wise round-to-nearest: with one group per channel it is the per-channel quantiser; every non-zero group
    reaches code magnitude 7; the reconstruction error is at most half a step of the group's own scale."""
    N, K = 12, 512
    w = synth.weights_fp16(N, K, config_id=64)
    w[3, 128:256] = 0
    wq1, s1 = oracle.quantize_weights_groups(w, group=K)
    wq0, s0 = oracle.quantize_weights_rtn(w)
    assert np.array_equal(wq1, wq0) and np.array_equal(s1.reshape(-1), s0)
    wq, s_g = oracle.quantize_weights_groups(w, group=128)
    assert s_g.shape == (4, N) and s_g[1, 3] == 0 and not wq[3, 128:256].any()
    blocks = np.abs(wq.astype(np.int32)).reshape(N, 4, 128).max(axis=2)
    assert np.all((blocks == 7) | (s_g.T == 0))
    top = np.abs(w.astype(np.float64)).reshape(N, 4, 128).max(axis=2)
    assert np.allclose(s_g.T, (top / 7).astype(np.float32), rtol=2.0 ** -23)
    rec = wq.astype(np.float64) * np.repeat(s_g.astype(np.float64).T, 128, axis=1)
    assert np.all(np.abs(rec - w.astype(np.float64)) <= 0.5000001 * np.repeat(s_g.astype(np.float64).T, 128, axis=1))
    # finer groups never reconstruct worse in the maximum norm of a group than the channel-wide scale allows
    assert np.all(s_g.T <= s0[:, None] * (1 + 2.0 ** -22))
