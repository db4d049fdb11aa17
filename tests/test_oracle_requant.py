"""Pins for the oracle's requantise-to-u8 step: an exact-rational re-derivation of
s32 -> binary32 -> one binary32 multiply -> ties-to-even integer -> +zc -> clamp."""
from fractions import Fraction

import numpy as np


def rne_to_binary32(x: Fraction) -> Fraction:
    """Nearest binary32 (normal range only), ties to even, in exact arithmetic."""
    if x == 0:
        return x
    mag = abs(x)
    e = 0
    while mag >= (1 << 24):
        mag /= 2
        e += 1
    while mag < (1 << 23):
        mag *= 2
        e -= 1
    assert -149 <= e <= 104, "outside the normal range this helper covers"
    m = round(mag)                  # Python rounds a Fraction half to even
    out = Fraction(m) * (Fraction(2) ** e)
    return out if x > 0 else -out


def requant_exact(c: int, scale32: np.float32, zc: int) -> int:
    f = rne_to_binary32(Fraction(c))
    g = rne_to_binary32(f * Fraction(float(scale32)))   # float(scale32) is exact
    r = round(g)                                        # half to even
    return min(255, max(0, r + zc))


def check(oracle, cs, scale, zc):
    cs = np.asarray(cs, dtype=np.int64)
    C = cs.astype(np.int32).reshape(1, -1)
    s32 = np.float32(scale)
    got = oracle.requant_s32u8(C, s32, zc)[0]
    want = [requant_exact(int(c), s32, zc) for c in cs]
    assert got.tolist() == want


def test_ties_to_even(oracle):
    check(oracle, np.arange(-41, 42), 0.5, 20)          # odd c gives exact .5
    check(oracle, np.arange(-1001, 1001, 2), 0.25, 128)
    # explicit hand values: 0.5*{1,3,5,-1,-3} -> {0,2,2,-0,-2}
    C = np.array([[1, 3, 5, -1, -3]], np.int32)
    assert oracle.requant_s32u8(C, 0.5, 10).tolist() == [[10, 12, 12, 10, 8]]


def test_clamp_edges(oracle):
    C = np.array([[-2, -1, 0, 1, 254, 255, 256, 257]], np.int32)
    assert oracle.requant_s32u8(C, 1.0, 0).tolist() == [[0, 0, 0, 1, 254, 255, 255, 255]]
    assert oracle.requant_s32u8(C, 1.0, 1).tolist() == [[0, 0, 1, 2, 255, 255, 255, 255]]
    check(oracle, [-2**31, -2**31 + 1, 2**31 - 1, 2**31 - 64, 2**31 - 65], 2.0**-23, 128)
    check(oracle, [-2**31, 2**31 - 1], 2.0**-30, 0)
    check(oracle, [-2**31, 2**31 - 1, 3, -3], 2.0**30, -5)


def test_extreme_output_zero_points(oracle):
    """zc at both ends of the int32 range and next to them, with a scale of 2^30 (r up to 2^61)
    and with scales that bring r + zc back into [0, 255]: the sum r + zc is exact (no 32-bit
    wrap, no float rounding), checked against the exact-rational helper."""
    cs = [-2**31, -2**31 + 1, -2**31 + 300, -3, -1, 0, 1, 2, 3, 255, 2**31 - 300, 2**31 - 2, 2**31 - 1]
    for zc in (-2**31, -2**31 + 300, 2**31 - 1, 2**31 - 300, -2**31 + 1):
        for scale in (2.0**30, 1.0, 2.0**-30, 0.75, 2.0**-7):
            check(oracle, cs, scale, zc)
    # sums that land inside [0, 255] only because zc is huge: c * 1.0 + zc
    check(oracle, [2**31 - 1, 2**31 - 100, 2**31 - 255, 2**31 - 256], 1.0, -2**31 + 300)
    check(oracle, [-2**31, -2**31 + 100, -2**31 + 254, -2**31 + 300], 1.0, 2**31 - 1)


def test_extreme_output_zero_points_channel_form_with_relu(oracle):
    """The same extremes through the per-column form, with and without the ReLU floor at zc."""
    rng = np.random.default_rng(44)
    M, N, K = 5, 6, 40
    A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    bias = np.array([2**31 - 1, -2**31, 12345, -2**31 + 300, 2**31 - 300, 0], dtype=np.int64).astype(np.int32)
    scale = np.array([2.0**30, 1.0, 2.0**-30, 0.75, 2.0**30, 1.0], np.float32)
    for zc in (-2**31, -2**31 + 300, 2**31 - 1):
        for relu in (False, True):
            got = oracle.gemm_u8s8u8_requant_channel(A, B, 100, 3, scale, zc, bias=bias, relu=relu)
            for i in range(M):
                for j in range(N):
                    c = sum((int(A[i, k]) - 100) * (int(B[j, k]) - 3) for k in range(K)) + int(bias[j])
                    c = (c + 2**31) % 2**32 - 2**31              # the bias add wraps in 32 bits
                    g = rne_to_binary32(rne_to_binary32(Fraction(c)) * Fraction(float(scale[j])))
                    q = round(g) + zc
                    if relu:
                        q = max(q, zc)
                    assert int(got[i, j]) == min(255, max(0, q)), (i, j, zc, relu)


def test_above_2_pow_24_conversion_rounds(oracle):
    base = 1 << 24
    cs = [base + d for d in range(-4, 40)] + [-(base + d) for d in range(-4, 40)]
    cs += [(1 << 27) + d for d in range(0, 64)]
    check(oracle, cs, 2.0**-17, 128)
    check(oracle, cs, 7.62939453125e-06 * 1.000001, 7)


def test_random_against_exact(oracle):
    rng = np.random.default_rng(31)
    for scale in (0.00096, 0.00048, 0.0123, 1.7, 3.1e-7, 2.0**-30, 123.456):
        cs = np.concatenate([rng.integers(-2**31, 2**31, size=600),
                             rng.integers(-400000, 400000, size=600)])
        check(oracle, cs, scale, int(rng.integers(-300, 300)))


def test_fused_equals_two_step(oracle):
    rng = np.random.default_rng(32)
    A = np.clip(np.rint(rng.normal(128, 40, size=(33, 300))), 0, 255).astype(np.uint8)
    B = np.clip(np.rint(rng.normal(0, 30, size=(29, 300))), -127, 127).astype(np.int8)
    C32 = oracle.gemm_u8s8s32(A, B, 128, 0)
    two = oracle.requant_s32u8(C32, 0.00096, 128)
    one = oracle.gemm_u8s8u8_requant(A, B, 128, 0, 0.00096, 128)
    assert np.array_equal(one, two)
    assert 20 < len(np.unique(one)) and one.min() >= 0      # spreads over the u8 range
    want = [[requant_exact(int(c), np.float32(0.00096), 128) for c in row] for row in C32]
    assert one.tolist() == want


# ---- per-column ("per-channel") epilogue ---------------------------------------------------


def test_channel_form_reduces_to_per_tensor(oracle):
    rng = np.random.default_rng(41)
    A = rng.integers(0, 256, size=(19, 150), dtype=np.uint8)
    B = rng.integers(-128, 128, size=(23, 150), dtype=np.int8)
    s = np.float32(0.0021)
    want = oracle.gemm_u8s8u8_requant(A, B, 77, -4, s, 99)
    got = oracle.gemm_u8s8u8_requant_channel(A, B, 77, -4, np.full(23, s, np.float32), 99,
                                             zb_vec=np.full(23, -4, np.int32), bias=np.zeros(23, np.int32))
    assert np.array_equal(got, want)
    assert np.array_equal(oracle.gemm_u8s8u8_requant_channel(A, B, 77, -4, np.full(23, s, np.float32), 99), want)


def test_channel_form_against_exact_arithmetic(oracle):
    """Python-integer sums with a different zero-point, scale and bias per column, the exact
    binary32 rounding helper above, ReLU applied as max(q, zc) before the clamp."""
    rng = np.random.default_rng(42)
    M, N, K = 7, 11, 60
    A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
    za, zc = 131, 20
    zbv = rng.integers(-128, 128, size=N).astype(np.int32)
    bias = rng.integers(-50000, 50000, size=N).astype(np.int32)
    scale = (10.0 ** rng.uniform(-5, -2, size=N)).astype(np.float32)
    for relu in (False, True):
        got = oracle.gemm_u8s8u8_requant_channel(A, B, za, 0, scale, zc, zb_vec=zbv, bias=bias, relu=relu)
        for i in range(M):
            for j in range(N):
                c = sum((int(A[i, k]) - za) * (int(B[j, k]) - int(zbv[j])) for k in range(K)) + int(bias[j])
                f = rne_to_binary32(Fraction(c))
                g = rne_to_binary32(f * Fraction(float(scale[j])))
                q = round(g) + zc
                if relu:
                    q = max(q, zc)
                assert int(got[i, j]) == min(255, max(0, q)), (i, j, relu)


def test_channel_bias_is_an_accumulator_shift_and_relu_is_a_floor(oracle):
    rng = np.random.default_rng(43)
    A = rng.integers(0, 256, size=(9, 80), dtype=np.uint8)
    B = rng.integers(-100, 100, size=(13, 80), dtype=np.int8)
    bias = rng.integers(-30000, 30000, size=13).astype(np.int32)
    scale = np.full(13, 0.0015, np.float32)
    C32 = oracle.gemm_u8s8s32(A, B, 128, 0)
    shifted = (C32.astype(np.int64) + bias[None, :]).astype(np.int32)
    want = oracle.requant_s32u8(shifted, np.float32(0.0015), 128)
    plain = oracle.gemm_u8s8u8_requant_channel(A, B, 128, 0, scale, 128, bias=bias)
    assert np.array_equal(plain, want)
    relu = oracle.gemm_u8s8u8_requant_channel(A, B, 128, 0, scale, 128, bias=bias, relu=True)
    assert np.array_equal(relu, np.maximum(plain, 128))
    assert (plain < 128).any() and (plain > 128).any()
