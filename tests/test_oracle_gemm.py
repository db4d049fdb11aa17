"""Pins for the CPU oracle's integer GEMM: each test fixes it to something other
than itself (Python big integers, closed forms, structural identities), chosen
so a dropped term, wrong sign, wrong index or transposed operand fails."""
import itertools
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def brute(A, B, za, zb):
    """Python-integer evaluation of sum_k (A[i][k]-za)(B[j][k]-zb), wrapped to 32 bits."""
    M, K = A.shape
    N = B.shape[0]
    a = A.tolist()
    b = B.tolist()
    out = [[0] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            s = 0
            for k in range(K):
                s += (a[i][k] - za) * (b[j][k] - zb)
            s &= 0xFFFFFFFF
            out[i][j] = s - (1 << 32) if s >= (1 << 31) else s
    return np.array(out, dtype=np.int64).reshape(M, N)


def rand_ab(rng, M, N, K):
    return (rng.integers(0, 256, size=(M, K), dtype=np.uint8),
            rng.integers(-128, 128, size=(N, K), dtype=np.int8))


def test_brute_force_all_tiny_shapes(oracle):
    rng = np.random.default_rng(11)
    dims = (1, 2, 3, 4, 5, 7, 8, 9)
    for M, N, K in itertools.product(dims, dims, dims):
        A, B = rand_ab(rng, M, N, K)
        za = int(rng.integers(0, 256))
        zb = int(rng.integers(-128, 128))
        got = oracle.gemm_u8s8s32(A, B, za, zb)
        assert np.array_equal(got.astype(np.int64), brute(A, B, za, zb)), (M, N, K, za, zb)


def test_brute_force_random_shapes_with_leading_dims(oracle):
    rng = np.random.default_rng(12)
    for _ in range(40):
        M, N, K = (int(x) for x in rng.integers(1, 34, size=3))
        pa, pb, pc = (int(x) for x in rng.integers(0, 5, size=3))
        Abig = rng.integers(0, 256, size=(M, K + pa), dtype=np.uint8)
        Bbig = rng.integers(-128, 128, size=(N, K + pb), dtype=np.int8)
        Cbig = np.full((M, N + pc), -777, dtype=np.int32)
        A, B, C = Abig[:, :K], Bbig[:, :K], Cbig[:, :N]
        za, zb = int(rng.integers(0, 256)), int(rng.integers(-128, 128))
        oracle.gemm_u8s8s32(A, B, za, zb, out=C)
        assert np.array_equal(C.astype(np.int64), brute(A, B, za, zb))
        assert np.all(Cbig[:, N:] == -777)          # gap of the leading dimension untouched


def test_numpy_int64_matmul_agrees(oracle):
    rng = np.random.default_rng(13)
    for (M, N, K) in ((17, 33, 129), (64, 64, 256), (5, 300, 77)):
        A, B = rand_ab(rng, M, N, K)
        za, zb = 131, -5
        ref = (A.astype(np.int64) - za) @ (B.astype(np.int64) - zb).T
        assert np.array_equal(oracle.gemm_u8s8s32(A, B, za, zb).astype(np.int64), ref)
        assert np.array_equal(oracle.gemm_u8s8s64(A, B, za, zb), ref)


def test_identity_operand(oracle):
    rng = np.random.default_rng(14)
    K = 37
    A = rng.integers(0, 256, size=(9, K), dtype=np.uint8)
    eye = np.eye(K, dtype=np.int8)                      # B = I  (N = K)
    for za in (0, 7, 128, 255):
        assert np.array_equal(oracle.gemm_u8s8s32(A, eye, za, 0), A.astype(np.int32) - za)
    # A = identity in u8: rows of C are the columns of the K x N operand, i.e. C[i][j] = B[j][i]
    B = rng.integers(-128, 128, size=(21, K), dtype=np.int8)
    assert np.array_equal(oracle.gemm_u8s8s32(np.eye(K, dtype=np.uint8), B, 0, 0), B.T.astype(np.int32))


def test_zero_operands(oracle):
    rng = np.random.default_rng(15)
    A, B = rand_ab(rng, 6, 10, 50)
    assert not oracle.gemm_u8s8s32(np.full_like(A, 93), B, 93, -4).any()      # A == za
    assert not oracle.gemm_u8s8s32(A, np.full_like(B, -17), 3, -17).any()     # B == zb
    assert not oracle.gemm_u8s8s32(np.zeros_like(A), B, 0, 0).any()


def test_one_hot_pins_layout(oracle):
    """A single non-zero in A and in B gives one product at exactly (i, j):
    pins row-major A, column-major B and the leading dimensions."""
    M, N, K = 5, 7, 11
    for (i, ka, j, kb) in ((0, 0, 0, 0), (4, 10, 6, 10), (2, 3, 5, 3), (2, 3, 5, 4), (3, 9, 1, 9)):
        A = np.zeros((M, K + 3), dtype=np.uint8)[:, :K]
        B = np.zeros((N, K + 2), dtype=np.int8)[:, :K]
        A[i, ka] = 200
        B[j, kb] = -100
        C = oracle.gemm_u8s8s32(A, B)
        want = np.zeros((M, N), dtype=np.int32)
        if ka == kb:
            want[i, j] = -20000
        assert np.array_equal(C, want)


def test_closed_forms(oracle):
    M, N, K = 40, 50, 123
    for (a, b, za, zb) in ((255, -128, 0, 0), (255, 127, 0, 0), (10, 3, 200, -8), (0, -128, 255, 127)):
        C = oracle.gemm_u8s8s32(np.full((M, K), a, np.uint8), np.full((N, K), b, np.int8), za, zb)
        assert np.all(C == K * (a - za) * (b - zb))
    i = np.arange(300)[:, None] % 256
    j = np.arange(200)[:, None] % 128
    A = np.broadcast_to(i, (300, K)).astype(np.uint8)
    B = np.broadcast_to(j, (200, K)).astype(np.int8)
    assert np.array_equal(oracle.gemm_u8s8s32(A, B), (K * i * j.T).astype(np.int32))


def test_four_term_partial_dot_products(oracle):
    """Sec. 2.1 four-term sums and the Sec. 3.1 broadcast form, hand-evaluated fixture."""
    rows = []
    with open(os.path.join(HERE, "golden", "four_term_dot.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            a, b, e = line.split("|")
            rows.append(([int(x) for x in a.split()], [int(x) for x in b.split()], int(e)))
    for a, b, e in rows:
        C = oracle.gemm_u8s8s32(np.array([a], np.uint8), np.array([b], np.int8))
        assert C.shape == (1, 1) and int(C[0, 0]) == e
    # broadcast form: v rows of the packed operand against one shared 4-byte b
    A = np.array([r[0] for r in rows], np.uint8)
    b = np.array([[5, -6, 7, -8]], np.int8)
    want = [sum(x * y for x, y in zip(r[0], [5, -6, 7, -8])) for r in rows]
    assert oracle.gemm_u8s8s32(A, b)[:, 0].tolist() == want


def test_no_16bit_saturation(oracle):
    """Adjacent-pair extremes exceed the s16 range; the result is the exact sum."""
    A = np.full((1, 2), 255, np.uint8)
    assert int(oracle.gemm_u8s8s32(A, np.full((1, 2), 127, np.int8))[0, 0]) == 64770
    assert int(oracle.gemm_u8s8s32(A, np.full((1, 2), -128, np.int8))[0, 0]) == -65280


def test_zero_point_expansion_identity(oracle):
    rng = np.random.default_rng(16)
    A, B = rand_ab(rng, 23, 31, 211)
    A64, B64 = A.astype(np.int64), B.astype(np.int64)
    for za, zb in ((0, 0), (128, 0), (0, 5), (77, -8), (255, 127), (1, -128)):
        raw = np.array([[int(np.dot(A64[i], B64[j])) for j in range(31)] for i in range(23)])
        want = raw - za * B64.sum(1)[None, :] - zb * A64.sum(1)[:, None] + 211 * za * zb
        assert np.array_equal(oracle.gemm_u8s8s32(A, B, za, zb).astype(np.int64), want)


def test_shift_form_identity(oracle):
    """The signed-shift form the GPU path relies on: sum (A-128) B + 128 colsum(B) == sum A B,
    and (a xor 0x80) read as s8 equals a - 128 for every byte."""
    a = np.arange(256, dtype=np.uint8)
    assert np.array_equal((a ^ 0x80).view(np.int8).astype(np.int32), a.astype(np.int32) - 128)
    rng = np.random.default_rng(17)
    A, B = rand_ab(rng, 12, 19, 333)
    shifted = oracle.gemm_u8s8s32(A, B, 128, 0).astype(np.int64)
    assert np.array_equal(shifted + 128 * B.astype(np.int64).sum(1)[None, :],
                          oracle.gemm_u8s8s32(A, B).astype(np.int64))


def test_linearity_in_b(oracle):
    rng = np.random.default_rng(18)
    A = rng.integers(0, 256, size=(8, 90), dtype=np.uint8)
    B1 = rng.integers(-60, 60, size=(13, 90), dtype=np.int8)
    B2 = rng.integers(-60, 60, size=(13, 90), dtype=np.int8)
    lhs = oracle.gemm_u8s8s32(A, (B1 + B2).astype(np.int8))
    assert np.array_equal(lhs, oracle.gemm_u8s8s32(A, B1) + oracle.gemm_u8s8s32(A, B2))


def test_k_permutation_invariance(oracle):
    """Sec. 2.1: the reduction order along K does not change the integers."""
    rng = np.random.default_rng(19)
    A, B = rand_ab(rng, 10, 14, 257)
    p = rng.permutation(257)
    assert np.array_equal(oracle.gemm_u8s8s32(A, B, 9, -3),
                          oracle.gemm_u8s8s32(np.ascontiguousarray(A[:, p]),
                                              np.ascontiguousarray(B[:, p]), 9, -3))


def test_k_split_additivity_through_the_wrap(oracle):
    """Sec. 2.1: partial sums over parts of K add up to the whole sum in the ring of integers mod 2^32,
    zero-points included and also where the whole sum wraps (what a K split over workgroups with
    atomic adds relies on)."""
    rng = np.random.default_rng(23)
    A, B = rand_ab(rng, 7, 9, 300)
    cuts = (0, 1, 64, 65, 256, 299, 300)
    whole = oracle.gemm_u8s8s32(A, B, 200, -100).astype(np.uint32)
    parts = np.zeros_like(whole)
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        parts += oracle.gemm_u8s8s32(np.ascontiguousarray(A[:, lo:hi]), np.ascontiguousarray(B[:, lo:hi]), 200, -100).astype(np.uint32)
    assert np.array_equal(parts, whole)
    K = 66000                                           # 66000 * 255 * 128 > 2^31: the whole sum wraps
    A = np.full((2, K), 255, dtype=np.uint8)
    B = np.full((3, K), -128, dtype=np.int8)
    whole = oracle.gemm_u8s8s32(A, B).astype(np.uint32)
    assert int(whole[0, 0]) == (-K * 32640) % 2**32
    halves = sum(oracle.gemm_u8s8s32(A[:, lo:hi].copy(), B[:, lo:hi].copy()).astype(np.uint32)
                 for lo, hi in ((0, 30000), (30000, K)))
    assert np.array_equal(halves.astype(np.uint32), whole)


@pytest.mark.parametrize("K,b,want32", [
    (65793, -128, -65793 * 32640),                  # last K whose negative extreme still fits (-2147483520)
    (65794, -128, (-65794 * 32640) + 2**32),        # one more wraps to +2147451136
    (66311, 127, 66311 * 32385),                    # last exact K at the positive extreme
    (66312, 127, 66312 * 32385 - 2**32),            # one more wraps negative
])
def test_overflow_bounds(oracle, K, b, want32):
    A = np.full((1, K), 255, np.uint8)
    B = np.full((1, K), b, np.int8)
    assert int(oracle.gemm_u8s8s64(A, B)[0, 0]) == K * 255 * b
    assert int(oracle.gemm_u8s8s32(A, B)[0, 0]) == want32
    assert -2**31 <= want32 < 2**31


def test_sampled_matches_full(oracle):
    rng = np.random.default_rng(20)
    A, B = rand_ab(rng, 30, 41, 100)
    full = oracle.gemm_u8s8s32(A, B, 5, -2)
    rows = rng.integers(0, 30, size=200)
    cols = rng.integers(0, 41, size=200)
    assert np.array_equal(oracle.gemm_u8s8s32_sampled(A, B, rows, cols, 5, -2), full[rows, cols])
    ref = (A.astype(np.int64) - 5) @ (B.astype(np.int64) + 2).T
    assert np.array_equal(full.astype(np.int64), ref)


def test_k_zero_gives_zeros(oracle):
    A = np.zeros((3, 0), np.uint8)
    B = np.zeros((4, 0), np.int8)
    assert np.array_equal(oracle.gemm_u8s8s32(A, B, 9, 9), np.zeros((3, 4), np.int32))


def test_signed_variant_brute_force_and_relation_to_unsigned(oracle):
    """s8 x s8: Python-integer brute force on small shapes, numpy on a larger one, and the
    identity C_s8(A - 128, za - 128) == C_u8(A, za) that ties it to the unsigned form."""
    rng = np.random.default_rng(51)
    for _ in range(30):
        M, N, K = (int(x) for x in rng.integers(1, 12, size=3))
        A = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
        B = rng.integers(-128, 128, size=(N, K), dtype=np.int8)
        za, zb = int(rng.integers(-128, 128)), int(rng.integers(-128, 128))
        want = [[sum((int(A[i, k]) - za) * (int(B[j, k]) - zb) for k in range(K)) for j in range(N)] for i in range(M)]
        assert oracle.gemm_s8s8s32(A, B, za, zb).tolist() == want
    A = rng.integers(-128, 128, size=(37, 300), dtype=np.int8)
    B = rng.integers(-128, 128, size=(29, 300), dtype=np.int8)
    ref = (A.astype(np.int64) + 7) @ (B.astype(np.int64) - 5).T
    assert np.array_equal(oracle.gemm_s8s8s32(A, B, -7, 5).astype(np.int64), ref)
    Au = (A.astype(np.int16) + 128).astype(np.uint8)
    assert np.array_equal(oracle.gemm_u8s8s32(Au, B, 121, 5), oracle.gemm_s8s8s32(A, B, -7, 5))
    assert int(oracle.gemm_s8s8s32(np.full((1, 4), -128, np.int8), np.full((1, 4), -128, np.int8))[0, 0]) == 65536


def test_unsigned_weight_variant_brute_force_and_relation_to_signed(oracle):
    """u8 x u8: Python-integer brute force, a numpy product, the wrap at the largest products
    (255 * 255 * K passes 2^31 at K = 33026) and C_u8u8(B, zb) == C_u8s8(B - 128, zb - 128)."""
    rng = np.random.default_rng(52)
    for _ in range(30):
        M, N, K = (int(x) for x in rng.integers(1, 12, size=3))
        A = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        B = rng.integers(0, 256, size=(N, K), dtype=np.uint8)
        za, zb = int(rng.integers(0, 256)), int(rng.integers(0, 256))
        want = [[sum((int(A[i, k]) - za) * (int(B[j, k]) - zb) for k in range(K)) for j in range(N)] for i in range(M)]
        assert oracle.gemm_u8u8s32(A, B, za, zb).tolist() == want
    A = rng.integers(0, 256, size=(37, 300), dtype=np.uint8)
    B = rng.integers(0, 256, size=(29, 300), dtype=np.uint8)
    ref = (A.astype(np.int64) - 7) @ (B.astype(np.int64) - 200).T
    assert np.array_equal(oracle.gemm_u8u8s32(A, B, 7, 200).astype(np.int64), ref)
    Bs = (B.astype(np.int16) - 128).astype(np.int8)
    assert np.array_equal(oracle.gemm_u8u8s32(A, B, 7, 200), oracle.gemm_u8s8s32(A, Bs, 7, 72))
    full = lambda K: int(oracle.gemm_u8u8s32(np.full((1, K), 255, np.uint8), np.full((1, K), 255, np.uint8))[0, 0])
    assert full(33025) == 33025 * 65025 == 2147450625
    assert full(33026) == 33026 * 65025 - 2**32


def test_16bit_variant(oracle):
    """s16 x s16: Python-integer brute force with zero-points over the int16 range, a numpy product,
    wrap at the extremes (32768^2 * 2 = 2^31 wraps to -2^31), leading dimensions, and agreement
    with the 8-bit sum when the values fit 8 bits."""
    rng = np.random.default_rng(53)
    for _ in range(30):
        M, N, K = (int(x) for x in rng.integers(1, 12, size=3))
        A = rng.integers(-32768, 32768, size=(M, K), dtype=np.int16)
        B = rng.integers(-32768, 32768, size=(N, K), dtype=np.int16)
        za, zb = int(rng.integers(-32768, 32768)), int(rng.integers(-32768, 32768))
        want = [[((sum((int(A[i, k]) - za) * (int(B[j, k]) - zb) for k in range(K)) + 2**31) % 2**32) - 2**31
                 for j in range(N)] for i in range(M)]
        assert oracle.gemm_s16s16s32(A, B, za, zb).tolist() == want
    A = rng.integers(-3000, 3000, size=(37, 300), dtype=np.int16)
    B = rng.integers(-200, 200, size=(29, 300), dtype=np.int16)
    ref = (A.astype(np.int64) - 11) @ (B.astype(np.int64) + 7).T          # fits int32: no wrap
    assert np.array_equal(oracle.gemm_s16s16s32(A, B, 11, -7).astype(np.int64), ref)
    lo = np.full((1, 2), -32768, np.int16)
    assert int(oracle.gemm_s16s16s32(lo, lo)[0, 0]) == -2**31            # 2 * 2^30 = 2^31 wraps
    assert int(oracle.gemm_s16s16s32(lo[:, :1], lo[:, :1])[0, 0]) == 2**30
    hi = np.full((1, 3), 32767, np.int16)
    assert int(oracle.gemm_s16s16s32(hi, hi)[0, 0]) == (3 * 32767 * 32767 + 2**31) % 2**32 - 2**31
    # padded rows (leading dimension > K) are not read
    Ap = np.full((5, 40), 12345, np.int16); Ap[:, :33] = rng.integers(-32768, 32768, size=(5, 33))
    Bp = np.full((4, 50), -321, np.int16); Bp[:, :33] = rng.integers(-32768, 32768, size=(4, 33))
    assert np.array_equal(oracle.gemm_s16s16s32(Ap[:, :33], Bp[:, :33], 5, 6),
                          oracle.gemm_s16s16s32(np.ascontiguousarray(Ap[:, :33]), np.ascontiguousarray(Bp[:, :33]), 5, 6))
    # 8-bit values: the same sum as the signed 8-bit variant
    A8 = rng.integers(-128, 128, size=(9, 70), dtype=np.int8)
    B8 = rng.integers(-128, 128, size=(6, 70), dtype=np.int8)
    assert np.array_equal(oracle.gemm_s16s16s32(A8.astype(np.int16), B8.astype(np.int16), -3, 9),
                          oracle.gemm_s8s8s32(A8, B8, -3, 9))
