/*
 * CPU oracle for the low-precision integer GEMM  C_s32 = A_u8 x B_s8.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product path never does.
 * It shares no source, header, table or helper with the HIP path.
 *
 * What it follows (paper sections, not a listing):
 *  - Problem statement, Sec. 2.1 "Conventional Approach": an unsigned 8-bit
 *    matrix times a signed 8-bit matrix gives a 32-bit result matrix; each
 *    element is the dot product of a row of one operand with a K-long vector
 *    of the other.  The operand stored as [N x K] in the paper is, here, the
 *    column-major K x N matrix B (column j = K contiguous bytes).
 *  - Sec. 2.1 closing remark and Sec. 3.1: the reordered reductions (phases
 *    1-3 of the conventional scheme, phases 1-2 of NGEMM) produce the same
 *    integers as the plain sum unless 32-bit overflow occurs.  So the oracle
 *    is the plain sum, accumulated in 64 bits, and the 32-bit result is the
 *    low 32 bits (two's complement) of that sum: exact whenever it fits,
 *    the wrapped value otherwise.
 *  - Sec. 3.1.1: zero padding of the packed operand is internal and never
 *    visible; the result has exactly M x N elements.
 *  - Sec. 4 "operation fusion": the paper names fusion of post-GEMM operations
 *    but gives no formula.  The zero-point form sum_k (A-za)(B-zb) and the
 *    requantisation sequence below are this build's reading, fixed as:
 *        f = (float)c          (binary32, round to nearest even)
 *        g = f * scale         (one binary32 multiply, no fused multiply-add)
 *        r = nearbyintf(g)     (ties to even)
 *        q = clamp((int64)r + zc, 0, 255)
 *
 * Parity pins (tests/test_oracle_*.py): brute force with Python integers on
 * tiny shapes, identity / zero / one-hot operands, closed forms for constant
 * and ramp operands, the four-term partial dot product of Sec. 2.1, the
 * zero-point expansion identity, linearity, K-permutation invariance, wrap
 * behaviour at the overflow bounds, and an integer-only re-derivation of the
 * requantisation.  No function here is "parity unpinned".
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 * Threads over output rows only (Sec. 4: multi-threading by parallelising the
 * outermost loop); every element is still computed by the naive k loop.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* s = sum_k (A[i,k]-za)(B[k,j]-zb) in int64; returned as is (no truncation). */
static int64_t dot_zp(const uint8_t *a_row, const int8_t *b_col, int64_t K,
                      int64_t za, int64_t zb)
{
    int64_t s = 0;
    for (int64_t k = 0; k < K; ++k)
        s += ((int64_t)a_row[k] - za) * ((int64_t)b_col[k] - zb);
    return s;
}

/* low 32 bits of a 64-bit sum, read as two's complement */
static int32_t wrap32(int64_t s)
{
    uint32_t u = (uint32_t)((uint64_t)s & 0xFFFFFFFFu);
    int32_t r;
    /* implementation-defined cast avoided: copy the bit pattern */
    __builtin_memcpy(&r, &u, sizeof r);
    return r;
}

/*
 * C[i*ldc + j] = wrap32( sum_k (A[i*lda+k]-za) * (B[j*ldb+k]-zb) ),  i<M, j<N.
 * A row-major (lda >= K), B column-major (ldb >= K), C row-major (ldc >= N).
 * Bytes of C outside the M x N window are not touched.
 */
void oracle_gemm_u8s8s32(int64_t M, int64_t N, int64_t K,
                         const uint8_t *A, int64_t lda, int32_t za,
                         const int8_t *B, int64_t ldb, int32_t zb,
                         int32_t *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j)
            C[i * ldc + j] = wrap32(dot_zp(A + i * lda, B + j * ldb, K, za, zb));
}

/* Signed variant (Sec. 3.1: other integer types follow the same scheme): A holds int8. */
void oracle_gemm_s8s8s32(int64_t M, int64_t N, int64_t K,
                         const int8_t *A, int64_t lda, int32_t za,
                         const int8_t *B, int64_t ldb, int32_t zb,
                         int32_t *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += ((int64_t)A[i * lda + k] - za) * ((int64_t)B[j * ldb + k] - zb);
            C[i * ldc + j] = wrap32(s);
        }
}

/* Unsigned-weight variant (Sec. 3.1: other integer types): both operands hold uint8. */
void oracle_gemm_u8u8s32(int64_t M, int64_t N, int64_t K,
                         const uint8_t *A, int64_t lda, int32_t za,
                         const uint8_t *B, int64_t ldb, int32_t zb,
                         int32_t *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += ((int64_t)A[i * lda + k] - za) * ((int64_t)B[j * ldb + k] - zb);
            C[i * ldc + j] = wrap32(s);
        }
}

/* 16-bit variant (Sec. 3.1 names s16 x s16 -> s32 among the types the method covers): the same
 * definition on int16 operands, zero-points in the int16 range, low 32 bits of the exact sum. */
void oracle_gemm_s16s16s32(int64_t M, int64_t N, int64_t K,
                           const int16_t *A, int64_t lda, int32_t za,
                           const int16_t *B, int64_t ldb, int32_t zb,
                           int32_t *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            /* |a - za| and |b - zb| stay below 2^16, so a product stays below 2^32 and the sum of
             * fewer than 2^31 of them below 2^63: int64 holds it exactly */
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += ((int64_t)A[i * lda + k] - za) * ((int64_t)B[j * ldb + k] - zb);
            C[i * ldc + j] = wrap32(s);
        }
}

/* Same sum without truncation, for the overflow-bound pins. */
void oracle_gemm_u8s8s64(int64_t M, int64_t N, int64_t K,
                         const uint8_t *A, int64_t lda, int32_t za,
                         const int8_t *B, int64_t ldb, int32_t zb,
                         int64_t *C, int64_t ldc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j)
            C[i * ldc + j] = dot_zp(A + i * lda, B + j * ldb, K, za, zb);
}

/* One requantised value; the sequence in the header, nothing else. */
static uint8_t requant_one(int32_t c, float scale, int32_t zc)
{
    volatile float f = (float)c;      /* volatile: no double intermediate, no contraction */
    volatile float g = f * scale;
    float r = nearbyintf(g);          /* default rounding mode: ties to even */
    int64_t q = (int64_t)r + (int64_t)zc;
    if (q < 0) q = 0;
    if (q > 255) q = 255;
    return (uint8_t)q;
}

void oracle_requant_s32u8(int64_t M, int64_t N,
                          const int32_t *C32, int64_t ldc32,
                          float scale, int32_t zc,
                          uint8_t *C8, int64_t ldc8)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j)
            C8[i * ldc8 + j] = requant_one(C32[i * ldc32 + j], scale, zc);
}

/* GEMM followed by requantisation of every element. */
void oracle_gemm_u8s8u8_requant(int64_t M, int64_t N, int64_t K,
                                const uint8_t *A, int64_t lda, int32_t za,
                                const int8_t *B, int64_t ldb, int32_t zb,
                                float scale, int32_t zc,
                                uint8_t *C8, int64_t ldc8)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int32_t c = wrap32(dot_zp(A + i * lda, B + j * ldb, K, za, zb));
            C8[i * ldc8 + j] = requant_one(c, scale, zc);
        }
}

/*
 * Per-column ("per-channel") form of the fused epilogue -- the realistic shape of the
 * "operation fusion" the paper names in Sec. 4 without defining it; this build's reading:
 *     c = wrap32( sum_k (A[i][k]-za) * (B[k][j]-zb_j) )      zb_j = zb_vec[j], or zb when zb_vec is NULL
 *     t = wrap32( c + bias[j] )                               bias NULL = 0
 *     g = (float)t * scale[j]                                 one binary32 multiply
 *     q = (int64)nearbyintf(g) + zc ;  if relu and q < zc: q = zc ;  clamp to [0,255]
 * (ReLU in the quantised domain: the real value (q - zc) * s_out is >= 0 iff q >= zc.)
 */
void oracle_gemm_u8s8u8_requant_channel(int64_t M, int64_t N, int64_t K,
                                        const uint8_t *A, int64_t lda, int32_t za,
                                        const int8_t *B, int64_t ldb, int32_t zb, const int32_t *zb_vec,
                                        const float *scale, const int32_t *bias, int32_t relu, int32_t zc,
                                        uint8_t *C8, int64_t ldc8)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            int64_t zbj = zb_vec ? (int64_t)zb_vec[j] : (int64_t)zb;
            int32_t c = wrap32(dot_zp(A + i * lda, B + j * ldb, K, za, zbj));
            int32_t t = wrap32((int64_t)c + (bias ? (int64_t)bias[j] : 0));
            volatile float f = (float)t;
            volatile float g = f * scale[j];
            float r = nearbyintf(g);
            int64_t q = (int64_t)r + (int64_t)zc;
            if (relu && q < zc) q = zc;
            if (q < 0) q = 0;
            if (q > 255) q = 255;
            C8[i * ldc8 + j] = (uint8_t)q;
        }
}

/*
 * Selected elements only: out[t] = C[rows[t]][cols[t]].  Lets the tests check
 * sampled outputs of shapes whose full product would take minutes here.
 */
void oracle_gemm_u8s8s32_sampled(int64_t K,
                                 const uint8_t *A, int64_t lda, int32_t za,
                                 const int8_t *B, int64_t ldb, int32_t zb,
                                 int64_t count, const int64_t *rows, const int64_t *cols,
                                 int32_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t)
        out[t] = wrap32(dot_zp(A + rows[t] * lda, B + cols[t] * ldb, K, za, zb));
}
