/*
 * ngemm.h -- C ABI of the MI355X (gfx950) low-precision integer GEMM library.
 *
 *     C_s32[M x N] = sum_k (A_u8[M x K] - za) * (B_s8[K x N] - zb)
 *
 * The operation is the low-precision GEMM of the paper's problem statement
 * (Sec. 2.1: an unsigned 8-bit matrix times a signed 8-bit matrix, 32-bit
 * result) with the offline-packed operand of Sec. 3.1.1 / Sec. 4 "Layout"
 * (the weight matrix is marshalled once and reused).  Per-tensor zero-points
 * and the requantise-to-u8 epilogue are this library's reading of the
 * "operation fusion" remark of Sec. 4; the paper gives no formula for them.
 *
 * Operand conventions (all matrices live in DEVICE memory owned by the caller):
 *   A  uint8, row-major,    A[i*lda + k],  lda >= K   (activation, not packed)
 *   B  int8,  column-major, B[j*ldb + k],  ldb >= K   (column j is K contiguous
 *      bytes: the paper's [N x K] storage; packed once by ngemm_pack_b)
 *   C  int32 (or uint8 for the requantised variant), row-major, C[i*ldc + j],
 *      ldc >= N.  Exactly the M x N window is written; the gaps left by a
 *      larger ldc are never touched.
 * All arithmetic is exact integer arithmetic modulo 2^32: whenever the true
 * sum fits in int32 the result is that sum (Sec. 2.1: any reduction order
 * gives the same integers unless K is large enough to overflow); beyond that
 * it is the low 32 bits of the true sum.  With zero-points 0 the sum always
 * fits for K <= 65793.
 *
 * The library never allocates, frees or synchronises device memory in the
 * run calls: everything is enqueued on the caller's HIP stream.  Host handles
 * (ngemm_ctx, ngemm_packed_b) are small host objects.
 *
 * Errors are return codes; on an error nothing has been launched.
 */
#ifndef NGEMM_H
#define NGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ngemm_ctx ngemm_ctx;           /* opaque host object                                  */
typedef struct ngemm_packed_b ngemm_packed_b; /* opaque host descriptor of a caller-owned device buffer */

typedef enum {
    NGEMM_OK = 0,
    NGEMM_ERR_INVALID_ARG = -1,      /* null pointer, zero-point or scale out of range              */
    NGEMM_ERR_BAD_SHAPE = -2,        /* negative dimension, leading dimension too small             */
    NGEMM_ERR_BUFFER_TOO_SMALL = -3, /* packed buffer or workspace smaller than the size functions say */
    NGEMM_ERR_DEVICE = -4,           /* a HIP call failed (no device, launch error)                 */
    NGEMM_ERR_UNSUPPORTED_ARCH = -5, /* the device is not gfx950                                    */
    NGEMM_ERR_STATIC_LIMIT = -6      /* ngemm_run_u8s8s32_static: M beyond its static scratch       */
} ngemm_status;

/* Kernel selection for ngemm_set_kernel (tests and A/B measurements). */
enum {
    NGEMM_KERNEL_AUTO = -1,
    NGEMM_KERNEL_SKINNY = 0,     /* split-K streaming kernel, M <= 32 only                */
    NGEMM_KERNEL_TILE_64 = 1,    /* 64 x 64 workgroup tile                                */
    NGEMM_KERNEL_TILE_128 = 2,   /* 128 x 128 workgroup tile                              */
    NGEMM_KERNEL_TILE_256 = 3,   /* 256 x 256 workgroup tile (throughput configuration)   */
    NGEMM_KERNEL_SPLIT_K = 4,    /* 64 x 64 tiles, K split over workgroups; int32 outputs */
    NGEMM_KERNEL_TILE_192 = 5,   /* 192 x 256 workgroup tile: the throughput configuration's form for outputs
                                    that 256 x 256 tiles leave some compute units idle on; runs the 256 x 256
                                    tiles where it cannot (rows of A not 16-byte aligned, K < 128)            */
    NGEMM_KERNEL_COUNT = 6
};

/* Human-readable name of a status code (static string, never NULL). */
const char *ngemm_status_string(ngemm_status s);

/*
 * Create a context bound to HIP device `device_ordinal`: the handle under which a weight operand
 * is packed once and multiplied many times (Sec. 3.1.1 and Sec. 4 "Layout": the marshalling is
 * set-up work, outside the GEMM calls).  Reads the device's compute-unit and XCD counts, which
 * the launches are sized by.  Fails with NGEMM_ERR_DEVICE when there is no such device and
 * NGEMM_ERR_UNSUPPORTED_ARCH when it is not a gfx950 part.  Makes no large allocation.  *out is
 * a host object owned by the caller until ngemm_destroy.
 */
ngemm_status ngemm_create(ngemm_ctx **out, int device_ordinal);

/* Destroy a context (the end of the pack-once / multiply-many lifetime of Sec. 4 "Layout").  Host
 * memory only: packed operands and every other device buffer stay with the caller.  NULL is
 * accepted; a pointer that is not a live context gives NGEMM_ERR_INVALID_ARG. */
ngemm_status ngemm_destroy(ngemm_ctx *ctx);

/* Force one kernel for the run calls (NGEMM_KERNEL_*), or NGEMM_KERNEL_AUTO for
 * the shape heuristic.  Forcing NGEMM_KERNEL_SKINNY with M > 32 makes the run
 * call return NGEMM_ERR_INVALID_ARG.  NGEMM_KERNEL_SPLIT_K serves outputs with so few
 * 64 x 64 tiles that most compute units would idle: K is cut into parts of at least 1024
 * bytes, one workgroup per tile and part; C is cleared by a launch of its own and the parts
 * add their partial sums with atomic adds (integer addition in any order gives the same
 * bits, the property Sec. 2.1 rests on); when the workspace has the room ngemm_workspace_bytes
 * counts for it, the parts store their partial tiles there instead and a second kernel sums
 * them and finishes the epilogue, which also serves u8 outputs (per-tensor b_zero_point).
 * It needs 16-byte aligned rows of A and a K of at least 2048; every other call it is forced
 * on runs the 64 x 64 tiles (the streaming kernel when M <= 32). */
ngemm_status ngemm_set_kernel(ngemm_ctx *ctx, int kernel);

/*
 * Shape-driven tuning (the method searches its tiling per problem size, Sec. 3.1.1 and Sec. 4):
 * run every kernel that can serve this call's shape on the caller's own operands (C is
 * overwritten with the same, correct result each time), time them with events on the stream,
 * and remember the fastest for later run calls of any entry point with the same (M, N, K) on
 * this context while the kernel choice is NGEMM_KERNEL_AUTO.  Arguments as for
 * ngemm_run_u8s8s32.  The call waits for the stream; it belongs to set-up, next to the pack.
 * *best_kernel (may be NULL) receives the NGEMM_KERNEL_* value.  A context is not meant to be
 * tuned and used from several threads at once.
 */
ngemm_status ngemm_tune_u8s8s32(ngemm_ctx *ctx, int64_t M,
                                const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                                const ngemm_packed_b *B, int32_t b_zero_point,
                                int32_t *C_dev, int64_t ldc,
                                void *workspace_dev, size_t workspace_bytes,
                                void *hip_stream, int *best_kernel);

/* The kernel remembered for a shape by ngemm_tune_u8s8s32, or NGEMM_KERNEL_AUTO if none. */
ngemm_status ngemm_tuned_kernel(const ngemm_ctx *ctx, int64_t M, int64_t N, int64_t K, int *kernel);

/* Cap the number of persistent workgroups the large-tile kernel launches (0 = one per compute
 * unit, the default).  For sharing the device with other work, and for tests that want many
 * tiles per workgroup on a small problem. */
ngemm_status ngemm_set_max_workgroups(ngemm_ctx *ctx, int max_workgroups);

/*
 * Size in bytes of the packed form of a K x N int8 operand (pure function, no
 * device needed).  Kp = K rounded up to 64, Np = N rounded up to 32; the size
 * is Kp*Np + 4*Np: the zero-padded matrix itself (Sec. 3.1.1: pad with 0 when
 * the sizes are not multiples of the inner block) plus one int32 column sum per
 * padded column.  No further blow-up: the footprint is the matrix size, as in
 * the paper's pack-memory comparison (Sec. 5).  Returns 0 for negative K or N.
 *
 * Layout of the packed buffer (two-level, as in Sec. 3.1.1: an inner block that
 * one matrix instruction consumes as a single contiguous vector, iterated by an
 * outer order that a workgroup streams through contiguously):
 *   inner block ("fragment") = 32 columns x 32 k-values = 1024 bytes; the byte
 *     for (column j, depth k) of fragment (p = j/32, s = k/32) sits at
 *       16 * (32 * ((k%32)/16) + j%32) + k%16
 *     i.e. 16 consecutive k per wavefront lane, lane = 32*((k%32)/16) + j%32.
 *   outer order: fragment (p, s) starts at byte 1024 * (p * (Kp/32) + s), so one
 *     32-column panel is one contiguous run over all of K.
 *   column sums: int32 colsum[j] = sum_k B[k][j] at byte offset Kp*Np + 4*j
 *     (0 for the padded columns).
 */
size_t ngemm_packed_b_bytes(int64_t K, int64_t N);

/*
 * Pack B (device, column-major, ldb >= K) into `packed_dev` (device, caller-
 * owned, at least ngemm_packed_b_bytes(K,N) bytes, 16-byte aligned) and compute
 * the column sums; asynchronous on `hip_stream` (a hipStream_t, NULL = default
 * stream).  `*out` receives a host descriptor that refers to `packed_dev`; the
 * buffer must stay alive and unmodified while the descriptor is used.  The
 * packed bytes are position-independent and may be copied or saved bytewise.
 * K == 0 or N == 0 is valid.
 */
ngemm_status ngemm_pack_b(ngemm_ctx *ctx, int64_t K, int64_t N,
                          const int8_t *B_dev, int64_t ldb,
                          void *packed_dev, size_t packed_bytes,
                          void *hip_stream, ngemm_packed_b **out);

/* Free the host descriptor only; the device buffer stays with the caller.  NULL is accepted. */
ngemm_status ngemm_packed_b_free(ngemm_packed_b *b);

/* Read back the shape a descriptor was packed with. */
ngemm_status ngemm_packed_b_shape(const ngemm_packed_b *b, int64_t *K, int64_t *N);

/*
 * Workspace of the run calls (device bytes, pure function): room for the int32 row sums
 * of A, needed only when b_zero_point != 0 (a NULL workspace is accepted otherwise), and,
 * for outputs of few tiles with a long K, room for the partial results of the K split (at
 * most 4 MiB).  A workspace that holds the row sums only is always enough: the K split then
 * adds its parts to C with atomic adds (int32 outputs) or is not used (u8 outputs).
 * A workspace handed to a run call must be 16-byte aligned (NGEMM_ERR_INVALID_ARG otherwise):
 * the kernels move it in 16-byte pieces.
 */
size_t ngemm_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * The GEMM of the problem statement (Sec. 2.1: unsigned 8-bit times signed 8-bit, 32-bit sums;
 * Sec. 3.1 phases 1 and 2: every output element is accumulated in place over K, no reduction
 * across vector lanes), on a B packed beforehand (Sec. 3.1.1):
 *   C[i][j] = sum_k (A[i][k] - a_zero_point) * (B[k][j] - b_zero_point), int32.
 *   A_dev: device, M rows of K bytes, pitch lda >= K; C_dev: device, M rows of N int32, pitch
 *   ldc >= N; workspace_dev: device, ngemm_workspace_bytes(M, N, K) bytes or NULL (see there).
 *   a_zero_point in [0,255], b_zero_point in [-128,127], else INVALID_ARG.
 *   M == 0 or N == 0: nothing is written, NGEMM_OK.  K == 0: C is all zeros.
 * Asynchronous on `hip_stream`.  A and the packed buffer are only read; every buffer stays the
 * caller's.  On an error nothing has been launched.
 */
ngemm_status ngemm_run_u8s8s32(ngemm_ctx *ctx, int64_t M,
                               const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                               const ngemm_packed_b *B, int32_t b_zero_point,
                               int32_t *C_dev, int64_t ldc,
                               void *workspace_dev, size_t workspace_bytes,
                               void *hip_stream);

/*
 * ngemm_run_u8s8s32 for callers that cannot allocate device memory, not even a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same result,
 * same arguments without the workspace: the row sums of A that b_zero_point != 0 needs (4 bytes
 * per row; the only scratch memory of the int32 path) live in a static array inside the
 * library's device image, NGEMM_STATIC_MAX_M * 4 = 256 KiB, which every GPU the library runs on
 * holds until the process ends.  M > NGEMM_STATIC_MAX_M gives NGEMM_ERR_STATIC_LIMIT (whatever
 * b_zero_point is) and nothing is launched.  The call allocates and frees nothing, on the host
 * or the device.  All calls on one GPU share that GPU's array: two calls with b_zero_point != 0
 * that may overlap in time (different streams, or different contexts of one device) race on it;
 * calls on one stream are ordered and safe.  Nothing in the array needs clearing between calls
 * (every call overwrites the entries it reads).
 */
#define NGEMM_STATIC_MAX_M 65536
ngemm_status ngemm_run_u8s8s32_static(ngemm_ctx *ctx, int64_t M,
                                      const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                                      const ngemm_packed_b *B, int32_t b_zero_point,
                                      int32_t *C_dev, int64_t ldc,
                                      void *hip_stream);

/*
 * Unsigned-weight variant, u8 x u8 -> s32 (Sec. 3.1: other integer types).  ngemm_pack_b_u8 is
 * ngemm_pack_b for a uint8 operand: it stores B - 128 (the same exact shift as for A) in the same
 * layout and size, with the column sums of the stored bytes.  A descriptor made by it is accepted
 * only by ngemm_run_u8u8s32, which takes b_zero_point in [0,255] and is otherwise
 * ngemm_run_u8s8s32; the other run calls return NGEMM_ERR_INVALID_ARG for it, and this one does
 * for a descriptor made by ngemm_pack_b.
 */
ngemm_status ngemm_pack_b_u8(ngemm_ctx *ctx, int64_t K, int64_t N,
                             const uint8_t *B_dev, int64_t ldb,
                             void *packed_dev, size_t packed_bytes,
                             void *hip_stream, ngemm_packed_b **out);
ngemm_status ngemm_run_u8u8s32(ngemm_ctx *ctx, int64_t M,
                               const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                               const ngemm_packed_b *B, int32_t b_zero_point,
                               int32_t *C_dev, int64_t ldc,
                               void *workspace_dev, size_t workspace_bytes,
                               void *hip_stream);

/*
 * Signed variant, s8 x s8 -> s32 (Sec. 3.1: the method applies to other integer types too): A
 * holds int8, a_zero_point lies in [-128,127]; everything else as in ngemm_run_u8s8s32.  The
 * same kernels run without the unsigned-to-signed shift.
 */
ngemm_status ngemm_run_s8s8s32(ngemm_ctx *ctx, int64_t M,
                               const int8_t *A_dev, int64_t lda, int32_t a_zero_point,
                               const ngemm_packed_b *B, int32_t b_zero_point,
                               int32_t *C_dev, int64_t ldc,
                               void *workspace_dev, size_t workspace_bytes,
                               void *hip_stream);

/*
 * Same sum (Sec. 2.1, Sec. 3.1) with a requantise-to-u8 step fused behind it, the "operation
 * fusion" that Sec. 4 names without a formula; this library fixes it as follows, applied to the
 * int32 value c of every element in exactly this order:
 *     f = (float)c            binary32, round to nearest even
 *     g = f * scale           one binary32 multiply (not fused with anything)
 *     r = round-half-even(g)
 *     C[i][j] = (uint8) min(255, max(0, r + c_zero_point))
 * `scale` must be finite and in [2^-30, 2^30] (INVALID_ARG otherwise), which
 * keeps every intermediate a normal binary32 number.  C_dev: device, M rows of N bytes, pitch
 * ldc >= N; the other arguments, ownership and error behaviour as for ngemm_run_u8s8s32.
 */
ngemm_status ngemm_run_u8s8u8_requant(ngemm_ctx *ctx, int64_t M,
                                      const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                                      const ngemm_packed_b *B, int32_t b_zero_point,
                                      float scale, int32_t c_zero_point,
                                      uint8_t *C_dev, int64_t ldc,
                                      void *workspace_dev, size_t workspace_bytes,
                                      void *hip_stream);

/*
 * Per-column ("per-channel") form of the fused epilogue, the usual shape of a quantised layer:
 * every output column j has its own scale, optional int32 bias and optional zero-point of B,
 * and a ReLU can be fused (this library's reading of the "operation fusion" remark of Sec. 4):
 *     c = sum_k (A[i][k] - a_zero_point) * (B[k][j] - zb_j)      zb_j = b_zero_points_dev[j],
 *                                                                or b_zero_point when that is NULL
 *     t = c + bias_dev[j]                  (int32, wrapping; bias_dev NULL = no bias)
 *     g = (float)t * scales_dev[j]         (one binary32 multiply)
 *     q = round-half-even(g) + c_zero_point;  if relu: q = max(q, c_zero_point)
 *     C[i][j] = (uint8) min(255, max(0, q))
 * scales_dev (N floats), bias_dev and b_zero_points_dev (N int32 each) are device arrays.  The
 * scales must be finite and in [2^-30, 2^30] and the zero-points in [-128,127]; being device
 * data they are not checked.  The workspace is needed when b_zero_points_dev is given or
 * b_zero_point != 0.
 */
ngemm_status ngemm_run_u8s8u8_requant_channel(ngemm_ctx *ctx, int64_t M,
                                              const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                                              const ngemm_packed_b *B, int32_t b_zero_point,
                                              const int32_t *b_zero_points_dev,
                                              const float *scales_dev, const int32_t *bias_dev,
                                              int32_t relu, int32_t c_zero_point,
                                              uint8_t *C_dev, int64_t ldc,
                                              void *workspace_dev, size_t workspace_bytes,
                                              void *hip_stream);

/*
 * 16-bit variant, s16 x s16 -> s32 (Sec. 3.1 lists it among the types the method covers):
 * C[i][j] = low 32 bits of sum_k (A[i][k] - a_zero_point) * (B[k][j] - b_zero_point) on int16
 * operands, zero-points in [-32768, 32767].  The target has no 16-bit integer matrix
 * instruction: the operands are split into byte planes and multiplied by four 8-bit matrix
 * ops per block, exactly (mod 2^32).
 *   ngemm_packed_b_bytes_s16 / ngemm_pack_b_s16: as ngemm_packed_b_bytes / ngemm_pack_b for an
 *     int16 operand (ldb in elements, B_dev 2-byte aligned); the packed form takes
 *     2 * (K rounded up to 32) * (N rounded up to 32) + 4 * (N rounded up to 32) bytes.
 *   ngemm_run_s16s16s32: as ngemm_run_u8s8s32 (lda in elements).  Rows of A must be 16-byte
 *     aligned (A_dev and 2 * lda multiples of 16), else NGEMM_ERR_INVALID_ARG; the workspace
 *     (ngemm_workspace_bytes) is always needed.  A descriptor from ngemm_pack_b_s16 is accepted
 *     by this call only, and this call accepts no other.
 */
size_t ngemm_packed_b_bytes_s16(int64_t K, int64_t N);
ngemm_status ngemm_pack_b_s16(ngemm_ctx *ctx, int64_t K, int64_t N,
                              const int16_t *B_dev, int64_t ldb,
                              void *packed_dev, size_t packed_bytes,
                              void *hip_stream, ngemm_packed_b **out);
ngemm_status ngemm_run_s16s16s32(ngemm_ctx *ctx, int64_t M,
                                 const int16_t *A_dev, int64_t lda, int32_t a_zero_point,
                                 const ngemm_packed_b *B, int32_t b_zero_point,
                                 int32_t *C_dev, int64_t ldc,
                                 void *workspace_dev, size_t workspace_bytes,
                                 void *hip_stream);

/*
 * Unpacked-B path, for the uncommon case where both operands are inputs of the call
 * (Sec. 3.1.1: packing then has to happen online, at a cost): B is given in its plain
 * column-major form (N rows of K contiguous int8, pitch ldb).  When the rows of A and of B are
 * 16-byte aligned (pointers and pitches multiples of 16) and M > 32, nothing is packed at all:
 * the tile kernels copy B's tiles from the caller's storage as they copy A's, and only the
 * column sums are computed beforehand.  Otherwise B is packed into the workspace on the stream
 * and multiplied at once.  The workspace must hold ngemm_unpacked_workspace_bytes(M, N, K)
 * bytes (16-byte aligned) for either way.  Result identical to ngemm_pack_b followed by
 * ngemm_run_u8s8s32.
 */
size_t ngemm_unpacked_workspace_bytes(int64_t M, int64_t N, int64_t K);
ngemm_status ngemm_run_u8s8s32_unpacked(ngemm_ctx *ctx, int64_t M, int64_t N, int64_t K,
                                        const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                                        const int8_t *B_dev, int64_t ldb, int32_t b_zero_point,
                                        int32_t *C_dev, int64_t ldc,
                                        void *workspace_dev, size_t workspace_bytes,
                                        void *hip_stream);

/* One member of a batch of independent GEMMs (host struct, device pointers inside). */
typedef struct ngemm_problem {
    int64_t M;
    const uint8_t *A_dev;
    int64_t lda;
    int32_t a_zero_point;
    int32_t b_zero_point;
    const ngemm_packed_b *B;
    int32_t *C_dev;
    int64_t ldc;
} ngemm_problem;

/* Workspace for a batch: 0 (the grouped kernels form the row sums a weight zero-point needs
 * themselves); kept so that callers size the argument of the run call by it. */
size_t ngemm_batched_workspace_bytes(int count, const ngemm_problem *problems);

/*
 * Run `count` independent int32-output GEMMs (arbitrary shapes, per-GEMM
 * zero-points) on one stream.  All members are validated before anything is
 * launched.  Results are those of `count` calls of ngemm_run_u8s8s32.  The members run in
 * grouped launches (one grid for the panels of the members with M <= 32 and the tiles of the
 * others, at most 67 members per grid); workspace_dev may be NULL.
 */
ngemm_status ngemm_run_batched_u8s8s32(ngemm_ctx *ctx, int count, const ngemm_problem *problems,
                                       void *workspace_dev, size_t workspace_bytes,
                                       void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* NGEMM_H */
