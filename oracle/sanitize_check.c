/*
 * Host-side sanitizer run of the CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Built together with ngemm_oracle.c under -fsanitize=address,undefined (tests/test_oracle_sanitized.py)
 * and run as a plain program: every oracle function is called on heap buffers that end exactly
 * where the documented extents end (rows of K bytes at pitch lda, the last row without the pitch's
 * slack), so that a read or write past an extent, a signed overflow, a misaligned access or an
 * out-of-range float-to-integer conversion stops the run.  The values themselves are pinned by
 * the Python tests; this program only checks a few of them again to make sure the calls did work.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_gemm_u8s8s32(int64_t, int64_t, int64_t, const uint8_t *, int64_t, int32_t, const int8_t *, int64_t, int32_t, int32_t *, int64_t);
void oracle_gemm_s8s8s32(int64_t, int64_t, int64_t, const int8_t *, int64_t, int32_t, const int8_t *, int64_t, int32_t, int32_t *, int64_t);
void oracle_gemm_u8u8s32(int64_t, int64_t, int64_t, const uint8_t *, int64_t, int32_t, const uint8_t *, int64_t, int32_t, int32_t *, int64_t);
void oracle_gemm_s16s16s32(int64_t, int64_t, int64_t, const int16_t *, int64_t, int32_t, const int16_t *, int64_t, int32_t, int32_t *, int64_t);
void oracle_gemm_u8s8s64(int64_t, int64_t, int64_t, const uint8_t *, int64_t, int32_t, const int8_t *, int64_t, int32_t, int64_t *, int64_t);
void oracle_requant_s32u8(int64_t, int64_t, const int32_t *, int64_t, float, int32_t, uint8_t *, int64_t);
void oracle_gemm_u8s8u8_requant(int64_t, int64_t, int64_t, const uint8_t *, int64_t, int32_t, const int8_t *, int64_t, int32_t, float, int32_t, uint8_t *, int64_t);
void oracle_gemm_u8s8u8_requant_channel(int64_t, int64_t, int64_t, const uint8_t *, int64_t, int32_t, const int8_t *, int64_t, int32_t,
                                        const int32_t *, const float *, const int32_t *, int32_t, int32_t, uint8_t *, int64_t);
void oracle_gemm_u8s8s32_sampled(int64_t, const uint8_t *, int64_t, int32_t, const int8_t *, int64_t, int32_t, int64_t,
                                 const int64_t *, const int64_t *, int32_t *);

static uint32_t rnd_state = 12345u;
static uint32_t rnd(void) { rnd_state = rnd_state * 1664525u + 1013904223u; return rnd_state >> 8; }

/* rows x cols elements of `size` bytes at pitch ld: exactly (rows-1)*ld + cols elements */
static void *extent(int64_t rows, int64_t cols, int64_t ld, size_t size)
{
    size_t n = rows > 0 ? (size_t)((rows - 1) * ld + cols) : 0;
    void *p = malloc(n * size + (n == 0));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    unsigned char *b = p;
    for (size_t i = 0; i < n * size; ++i) b[i] = (unsigned char)rnd();
    return p;
}

static int fail(const char *what) { fprintf(stderr, "sanitize_check: %s\n", what); return 1; }

int main(void)
{
    static const int64_t shapes[][3] = {{1, 1, 1}, {3, 5, 7}, {4, 4, 0}, {0, 3, 5}, {5, 0, 3}, {17, 9, 33}, {2, 2, 300}};
    for (size_t t = 0; t < sizeof shapes / sizeof shapes[0]; ++t) {
        const int64_t M = shapes[t][0], N = shapes[t][1], K = shapes[t][2];
        const int64_t lda = K + 3, ldb = K + 1, ldc = N + 2;
        uint8_t *A = extent(M, K, lda, 1);
        int8_t *B = extent(N, K, ldb, 1);
        int32_t *C = extent(M, N, ldc, 4);
        int64_t *C64 = extent(M, N, ldc, 8);
        uint8_t *C8 = extent(M, N, ldc, 1);
        int16_t *A16 = extent(M, K, lda, 2), *B16 = extent(N, K, ldb, 2);
        oracle_gemm_u8s8s32(M, N, K, A, lda, 255, B, ldb, -128, C, ldc);
        oracle_gemm_u8s8s32(M, N, K, A, lda, 0, B, ldb, 127, C, ldc);
        oracle_gemm_s8s8s32(M, N, K, (const int8_t *)A, lda, -128, B, ldb, 127, C, ldc);
        oracle_gemm_u8u8s32(M, N, K, A, lda, 255, (const uint8_t *)B, ldb, 255, C, ldc);
        oracle_gemm_s16s16s32(M, N, K, A16, lda, -32768, B16, ldb, 32767, C, ldc);
        oracle_gemm_u8s8s64(M, N, K, A, lda, 3, B, ldb, -3, C64, ldc);
        oracle_gemm_u8s8u8_requant(M, N, K, A, lda, 128, B, ldb, 0, 0x1p30f, -2147483647 - 1, C8, ldc);
        oracle_gemm_u8s8u8_requant(M, N, K, A, lda, 128, B, ldb, 0, 0x1p-30f, 2147483647, C8, ldc);
        {
            int32_t *zbv = malloc(sizeof(int32_t) * (size_t)(N + (N == 0))), *bias = malloc(sizeof(int32_t) * (size_t)(N + (N == 0)));
            float *sc = malloc(sizeof(float) * (size_t)(N + (N == 0)));
            for (int64_t j = 0; j < N; ++j) {
                zbv[j] = (int32_t)(rnd() % 256) - 128;
                bias[j] = j % 2 ? 2147483647 : -2147483647 - 1;
                sc[j] = j % 3 ? 0x1p30f : 0x1p-30f;
            }
            oracle_gemm_u8s8u8_requant_channel(M, N, K, A, lda, 77, B, ldb, 5, zbv, sc, bias, 1, 2147483647, C8, ldc);
            oracle_gemm_u8s8u8_requant_channel(M, N, K, A, lda, 77, B, ldb, 5, NULL, sc, NULL, 0, -2147483647 - 1, C8, ldc);
            free(zbv); free(bias); free(sc);
        }
        oracle_gemm_u8s8s32(M, N, K, A, lda, 7, B, ldb, -7, C, ldc);
        oracle_requant_s32u8(M, N, C, ldc, 0.37f, 11, C8, ldc);
        if (M > 0 && N > 0) {
            int64_t rows[3] = {0, M - 1, M / 2}, cols[3] = {N - 1, 0, N / 2};
            int32_t out[3];
            oracle_gemm_u8s8s32_sampled(K, A, lda, 7, B, ldb, -7, 3, rows, cols, out);
            for (int s = 0; s < 3; ++s)
                if (out[s] != C[rows[s] * ldc + cols[s]]) return fail("sampled element differs from the full product");
            int64_t want = 0;
            for (int64_t k = 0; k < K; ++k) want += ((int64_t)A[k] - 7) * ((int64_t)B[k] + 7);
            if (C[0] != (int32_t)want) return fail("C[0][0] differs from a direct sum");
        }
        free(A); free(B); free(C); free(C64); free(C8); free(A16); free(B16);
    }
    /* the wrap at a long K and the extremes of the requantising step */
    {
        const int64_t K = 66312;
        uint8_t *A = malloc((size_t)K);
        int8_t *B = malloc((size_t)K);
        memset(A, 255, (size_t)K);
        memset(B, 127, (size_t)K);
        int32_t c;
        oracle_gemm_u8s8s32(1, 1, K, A, K, 0, B, K, 0, &c, 1);
        if (c != (int32_t)(uint32_t)((uint64_t)K * 255u * 127u)) return fail("wrap at K = 66312");
        free(A); free(B);
        const int32_t cs[4] = {-2147483647 - 1, 2147483647, 1, -1};
        uint8_t q[4];
        oracle_requant_s32u8(1, 4, cs, 4, 0x1p30f, 0, q, 4);
        if (q[0] != 0 || q[1] != 255 || q[2] != 255 || q[3] != 0) return fail("requantised extremes");
    }
    puts("sanitize_check ok");
    return 0;
}
