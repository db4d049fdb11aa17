// Device kernels of the gfx950 u8 x s8 -> s32 GEMM.  Included only by ngemm.hip.
//
// Mapping of the paper's method onto CDNA4 (Sec. 3.1 of the paper):
//  * phase 1 (multiply narrow operands, widen, one partial sum per output
//    element held in its own SIMD lane) and phase 2 (accumulate partials
//    straight into the result vector, no horizontal tree reduction) are one
//    matrix instruction -- v_mfma_i32_32x32x32_i8 (1024 distinct C elements per
//    wavefront) or, in the large int32-output kernel, v_mfma_i32_16x16x64_i8
//    (256 of them) -- each element accumulated in place over the K loop.
//  * the packed operand's inner block (Sec. 3.1.1) is the 1 KiB fragment one
//    MFMA consumes: lane l of the wavefront holds 16 consecutive k-values of
//    column l%32, depth half l/32.
//  * the unsigned operand is mapped onto the signed matrix instruction by the
//    exact shift A' = A - 128 (byte-wise xor 0x80); the epilogue adds
//    (128 - za) * colsum_B[j] - zb * rowsum_A'[i] - zb * (128 - za) * K, all in
//    wrapping 32-bit arithmetic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ngemm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v4i_a4 __attribute__((ext_vector_type(4), aligned(4)));   // the same with the alignment of an int
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kFragBytes = 1024;   // 32 columns x 32 k-values

struct GemmParams {
    const uint8_t *A;       // row-major u8
    int64_t lda;
    const uint8_t *Bp;      // packed fragments
    const int32_t *colsum;  // Np entries
    const int32_t *rowsum;  // M entries of sum_k (A[i][k] - 128), or nullptr when zb == 0
    void *C;                // int32 or uint8, row-major
    int64_t ldc;
    int M, N, K, Kp;        // Kp = K rounded up to 64
    int npanels;            // Np / 32
    int tiles_m, tiles_n;
    uint32_t za_term;       // shift - za, shift = 128 for unsigned A, 0 for signed A
    uint32_t zb;            // zb (two's complement)
    uint32_t kconst;        // -zb * (shift - za) * K  (mod 2^32)
    float scale;
    int32_t zc;
    // per-column form of the requantising epilogue (all nullptr / 0 for the per-tensor form)
    const float *scale_vec;   // N scales, replaces `scale`
    const int32_t *bias_vec;  // N int32 biases added to the sum before scaling
    const int32_t *zb_vec;    // N zero-points of B's columns, replaces `zb`
    uint32_t rconst;          // (shift - za) * K: sum_k (A[i][k] - za) = rowsum[i] + rconst
    int relu;                 // clamp from below at zc
    // operand type of A: 0x80808080 for unsigned bytes (shifted to signed by xor), 0 for signed
    // bytes (used as they are; za_term and rconst are then -za and -za*K)
    uint32_t a_xor;
    // K split over workgroups (gemm_tile_deep_kernel, SPLITK forms): unit u of the grid is tile
    // u % ntiles, bytes [kchunk * (u / ntiles), + kchunk) of K; kchunk is a multiple of 256.
    // part_ws (SPLITK = 2): the parts' partial results, `ksplit` dense int32 matrices of M rows,
    // row pitch N rounded up to 4.
    int ksplit, kchunk;
    int32_t *part_ws;
    // number of XCDs of the device (hipDeviceAttributeNumberOfXccs): consecutive workgroup ids are
    // dispatched to them round-robin, which the tile order and the staggered epilogues build on
    int nxcd;
};

// ---- small helpers -------------------------------------------------------------------------

// 16 bytes from an address with no alignment promise.
__device__ __forceinline__ v4i load16_any(const uint8_t *p)
{
    v4i v;
    __builtin_memcpy(&v, p, 16);
    return v;
}

// First `valid` (0..15) bytes of a 16-byte chunk, the rest zero; never reads past p + valid.
__device__ __forceinline__ v4i load16_partial(const uint8_t *p, int valid)
{
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int b = 0; b < 16; ++b)
        if (b < valid) w[b >> 2] |= (uint32_t)p[b] << (8 * (b & 3));
    v4i v;
    v.x = (int)w[0]; v.y = (int)w[1]; v.z = (int)w[2]; v.w = (int)w[3];
    return v;
}

// u8 -> s8 shift of 16 packed bytes: a xor 0x80 == a - 128 read as signed (mask 0x80808080);
// a signed A operand passes with mask 0.
__device__ __forceinline__ v4i shift_u8_to_s8(v4i v, uint32_t mask)
{
    v.x ^= (int)mask; v.y ^= (int)mask;
    v.z ^= (int)mask; v.w ^= (int)mask;
    return v;
}

// int32 value of one output element from its shifted-form accumulator.
__device__ __forceinline__ int32_t finish_s32(const GemmParams &p, int32_t acc, uint32_t cs_term, int row)
{
    uint32_t v = (uint32_t)acc + cs_term + p.kconst;
    if (p.rowsum) v -= p.zb * (uint32_t)p.rowsum[row];
    return (int32_t)v;
}

// Requantise-to-u8 sequence of the header: cvt, one multiply, round-half-even, add zc, optional
// floor at zc (ReLU in the quantised domain), clamp.
__device__ __forceinline__ uint8_t requant_u8(int32_t c, float scale, int32_t zc, int relu)
{
    float f = (float)c;
    float g = __fmul_rn(f, scale);
    float r = rintf(g);
    // q = r + zc exactly, without a float -> int64 conversion (|r| <= 2^61 here: |c| <= 2^31, scale <= 2^30).
    // Inside the int32 range (which includes -2^31) r converts exactly and the sum is a 64-bit add.
    // r > 2^31: r >= 2^31 + 256, so q >= 256 + zc + 2^31 >= 256 whatever zc is.  r == 2^31: q = 2^31 + zc,
    // which lies in [0, 2^32).  r < -2^31: r <= -2^31 - 256, so q < 0 and q < zc.
    const float lim = 2147483648.0f;
    const float rc = fminf(fmaxf(r, -lim), 2147483520.0f);           // 2^31 - 128: the largest float below 2^31
    long long q = (long long)(int)rc + (long long)zc;
    if (r >= lim) q = (r == lim) ? (long long)((uint32_t)zc + 0x80000000u) : 256;
    if (r < -lim) q = -4294967296LL;                                 // below 0 and below every zc
    if (relu && q < (long long)zc) q = zc;
    q = q < 0 ? 0 : (q > 255 ? 255 : q);
    return (uint8_t)q;
}

// The same values when |zc| < 2^23 (the caller checks; every practical zero-point), in binary32 throughout,
// four packed into a word: r = rint(c * scale), q = r + zc, the ReLU floor, and v_cvt_pk_u8_f32, which converts
// with saturation to [0, 255] and writes one byte of the word (checked on the target: -inf .. 0.5 -> 0,
// 255.5 .. +inf -> 255, ties to even) -- five vector instructions per value, no clamps, no shifts to pack.
// r beyond +-2^24 cannot land in [0, 255] after adding zc, nor on the other side of zc; up to there binary32
// addition of two integers is exact, beyond it the sum is off by little and far from 0, 255 and zc.
// floor_f: zc for the ReLU form, -FLT_MAX otherwise.
__device__ __forceinline__ uint32_t requant4_u8_small_zc(const int32_t (&c)[4], const float4 &scale, float zcf, float floor_f)
{
    uint32_t w = 0u;
    w = __builtin_amdgcn_cvt_pk_u8_f32(fmaxf(rintf(__fmul_rn((float)c[0], scale.x)) + zcf, floor_f), 0, w);
    w = __builtin_amdgcn_cvt_pk_u8_f32(fmaxf(rintf(__fmul_rn((float)c[1], scale.y)) + zcf, floor_f), 1, w);
    w = __builtin_amdgcn_cvt_pk_u8_f32(fmaxf(rintf(__fmul_rn((float)c[2], scale.z)) + zcf, floor_f), 2, w);
    w = __builtin_amdgcn_cvt_pk_u8_f32(fmaxf(rintf(__fmul_rn((float)c[3], scale.w)) + zcf, floor_f), 3, w);
    return w;
}

// General (per-column capable) value of one requantised element from its shifted-form
// accumulator: c = acc + (128-za)*colsum_j - zb_j * sum_k(A[i][k]-za), t = c + bias_j.
__device__ __forceinline__ uint8_t finish_u8(const GemmParams &p, int32_t acc, uint32_t cs_term, int row, int col)
{
    const uint32_t zbj = p.zb_vec ? (uint32_t)p.zb_vec[col] : p.zb;
    const uint32_t rsum = (p.rowsum ? (uint32_t)p.rowsum[row] : 0u) + p.rconst;
    uint32_t t = (uint32_t)acc + cs_term - zbj * rsum;
    if (p.bias_vec) t += (uint32_t)p.bias_vec[col];
    return requant_u8((int32_t)t, p.scale_vec ? p.scale_vec[col] : p.scale, p.zc, p.relu);
}

template <bool REQUANT>
__device__ __forceinline__ void store_out(const GemmParams &p, int row, int col, int32_t acc, uint32_t cs_term)
{
    if (REQUANT)
        ((uint8_t *)p.C)[(int64_t)row * p.ldc + col] = finish_u8(p, acc, cs_term, row, col);
    else
        ((int32_t *)p.C)[(int64_t)row * p.ldc + col] = finish_s32(p, acc, cs_term, row);
}

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---- pack: column-major B -> fragment order, zero padded, with column sums --------------------
// One workgroup per (32-column panel, 512 bytes of K = 16 fragments).  Global reads follow the
// columns (32 consecutive lanes read 512 contiguous bytes of one column), the block is turned
// in LDS (row pitch 512 + 16 bytes: conflict-free both ways), and the 16 KiB of fragments leave as
// one contiguous run.  Column sums: every 16-byte chunk is summed with a dot-product-with-ones,
// the 32 lanes sharing a column are added across lanes (the one horizontal reduction of the
// path; Sec. 2.1 phase 3) and one integer atomic per column and workgroup goes to colsum, which
// zero_i32_kernel has cleared beforehand (integer adds: the result does not depend on the order).
constexpr int kPackKBytes = 512;

__global__ __launch_bounds__(256) void zero_i32_kernel(int32_t *__restrict__ dst, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) dst[i] = 0;
}

// Clears the M x N int32 outputs of C (row pitch ldc; the gaps between rows are left alone):
// workgroup u covers 1024 columns of row u / segs.
__global__ __launch_bounds__(256) void zero_c_kernel(int32_t *__restrict__ C, int64_t ldc, int N, int segs)
{
    const int row = blockIdx.x / segs, seg = blockIdx.x - row * segs;
    const int col = seg * 1024 + threadIdx.x * 4;
    int32_t *dst = C + (int64_t)row * ldc + col;
#pragma unroll
    for (int t = 0; t < 4; ++t)
        if (col + t < N) dst[t] = 0;
}

__global__ __launch_bounds__(256) void pack_b_kernel(const int8_t *__restrict__ B, int64_t ldb, int K, int N,
                                                     int Kp, int kblocks, uint32_t b_xor,
                                                     uint8_t *__restrict__ packed, int32_t *__restrict__ colsum)
{
    __shared__ __attribute__((aligned(16))) uint8_t turn[32 * (kPackKBytes + 16)];
    const int tid = threadIdx.x;
    const int pnl = blockIdx.x / kblocks, kblk = blockIdx.x % kblocks;
    const int nslices = Kp / 32;
    const int k_base = kblk * kPackKBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i;                     // chunk: column c/32 of the panel, k-chunk c%32
        const int jl = c >> 5, kc = c & 31;
        const int j = pnl * 32 + jl, k0 = k_base + kc * 16;
        v4i v = {0, 0, 0, 0};
        if (j < N && k0 < K) {
            const uint8_t *src = (const uint8_t *)B + (int64_t)j * ldb + k0;
            v = (k0 + 16 <= K) ? load16_any(src) : load16_partial(src, K - k0);
            if (b_xor) {
                // unsigned B: shift the bytes that exist to signed; the padding stays zero
                const int nb = K - k0;
                int *w = (int *)&v;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int vb = nb - 4 * q;
                    const uint32_t m = vb >= 4 ? 0xffffffffu : (vb <= 0 ? 0u : (1u << (8 * vb)) - 1u);
                    w[q] ^= (int)(b_xor & m);
                }
            }
        }
        *(v4i *)(turn + jl * (kPackKBytes + 16) + kc * 16) = v;
        // column sum of this chunk, then over the 32 lanes that hold the same column
        int s = __builtin_amdgcn_sdot4(v.x, 0x01010101, 0, false);
        s = __builtin_amdgcn_sdot4(v.y, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4(v.z, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4(v.w, 0x01010101, s, false);
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if ((tid & 31) == 0 && j < N && s != 0) atomicAdd(colsum + j, s);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int o = tid + 256 * i;                     // output chunk: fragment o/64 of the block, lane o%64
        const int s = o >> 6, l = o & 63;
        const int slice = kblk * (kPackKBytes / 32) + s;
        if (slice < nslices) {
            const v4i v = *(const v4i *)(turn + (l & 31) * (kPackKBytes + 16) + (2 * s + (l >> 5)) * 16);
            *(v4i *)(packed + ((int64_t)pnl * nslices + slice) * kFragBytes + l * 16) = v;
        }
    }
}

// rowsum[i] = sum_k (A[i][k] - 128); needed only when zb != 0.  One wavefront per row, 16 bytes
// per lane and step: the bytes are shifted to signed (xor 0x80) and summed by a dot product with
// ones, then across the lanes.
__device__ __forceinline__ int row_sum_shifted(const uint8_t *row, int K, int lane, uint32_t mask)
{
    int s = 0;
    for (int k = lane * 16; k < K; k += 64 * 16) {
        v4i v = (k + 16 <= K) ? load16_any(row + k) : load16_partial(row + k, K - k);
        v = shift_u8_to_s8(v, mask);
        if (k + 16 > K && mask) {
            // bytes past K were zero before the shift: take their -128 back out
            s += 128 * (k + 16 - K);
        }
        s = __builtin_amdgcn_sdot4(v.x, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4(v.y, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4(v.z, 0x01010101, s, false);
        s = __builtin_amdgcn_sdot4(v.w, 0x01010101, s, false);
    }
    return wave_sum(s);
}

__global__ __launch_bounds__(256) void rowsum_a_kernel(const uint8_t *__restrict__ A, int64_t lda, int M, int K,
                                                       uint32_t mask, int32_t *__restrict__ rowsum)
{
    int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (i >= M) return;
    const int s = row_sum_shifted(A + (int64_t)i * lda, K, lane, mask);
    if (lane == 0) rowsum[i] = s;
}

// ---- tiled MFMA kernel ----------------------------------------------------------------------
// Workgroup tile BM x BN, WGM x WGN wavefronts, each owning (TM*32) x (TN*32) of C in
// accumulators; BK bytes of K are staged per main-loop step, double buffered in LDS.
//
// LDS layout of a stage.  B: the packed fragments as they are (lane l's 16 bytes at 16*l of
// its 1 KiB fragment), so the global->LDS copy is linear and every fragment read is one
// conflict-free 16-byte-per-lane LDS load.  A (row-major in memory, fragment order needed by
// the matrix instruction): 16-byte chunk (row r, k-chunk c) goes to 16-byte slot
//     (r/32) * (CPR*32) + c*32 + ((r%32) xor (c*SW)),   CPR = BK/16, SW = 16/CPR,
// which keeps both sides conflict-free: a fragment read (fixed c, 16 consecutive rows) and a
// stage write (CPR consecutive lanes cover BK contiguous bytes of one row, so the global load
// is coalesced, and 16 consecutive lanes still hit 16 different 16-byte bank groups).
template <int BM, int BN, int WGM, int WGN, int BK>
struct TileCfg {
    static constexpr int kThreads = WGM * WGN * 64;
    static constexpr int TM = BM / (WGM * 32);
    static constexpr int TN = BN / (WGN * 32);
    static constexpr int KS = BK / 32;                        // matrix-instruction sub-steps per stage
    static constexpr int CPR = BK / 16;                       // 16-byte chunks per A row per stage
    static constexpr int SW = 16 / CPR;
    static constexpr int kAChunks = BM * BK / 16;
    static constexpr int kBChunks = BN * BK / 16;
    static constexpr int kAIters = kAChunks / kThreads;
    static constexpr int kBIters = kBChunks / kThreads;
    static constexpr int kABytes = BM * BK;
    static constexpr int kStageBytes = (BM + BN) * BK;
    static constexpr int kEpiBytes = WGM * WGN * 32 * (TN * 128 + 16) + BN * 12;  // epilogue: transposition patches + three per-column arrays
    static constexpr int kLdsBytes = 2 * kStageBytes > kEpiBytes ? 2 * kStageBytes : kEpiBytes;
    static_assert(BK == 64 || BK == 128, "stage depth");
    static_assert(kAChunks % kThreads == 0 && kBChunks % kThreads == 0, "loader shape");
    static_assert(TM >= 1 && TN >= 1, "wave tile");
};

// XCD-aware tile order: consecutive workgroup ids land on different XCDs (`nxcd` of them, each
// with its own L2), so give each XCD one contiguous run of the logical tile order, and make that
// order walk groups of GM tile-rows column by column so that the tiles in flight on one XCD
// share A row-panels and B column-panels.
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int nxcd, int &tm, int &tn)
{
    const int nb = tiles_m * tiles_n;
    const int q = nb / nxcd, r = nb - q * nxcd;
    const int local = bid / nxcd, xcd = bid - local * nxcd;
    const int logical = xcd * q + (xcd < r ? xcd : r) + local;
    constexpr int GM = 4;
    const int per_group = GM * tiles_n;
    const int group = logical / per_group;
    const int first_m = group * GM;
    const int gsize = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
    const int in_group = logical - group * per_group;
    tm = first_m + in_group % gsize;
    tn = in_group / gsize;
}

// Workgroup barrier that orders LDS traffic only: outstanding global loads (the prefetch of a
// later stage) stay in flight across it.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Epilogue shared by the tiled kernels: zero-point terms, optional requantisation, stores.
// acc[i][j] is the accumulator of A block i, B block j of this wavefront with the packed
// operand as the first matrix-instruction source: lane l holds row l%32 of the A block and, in
// registers 4q..4q+3, the four consecutive columns 8q + 4*(l/32) + (0..3) of the B block.
//
// int32 results leave through an LDS patch per wavefront (`xpose`, this wavefront's own,
// 32 rows x TN*128 bytes): a row of TN blocks is written in accumulator order and read back
// row-wise, so that one store instruction writes full 128-byte lines (TN*128 contiguous bytes per
// row) instead of 32-byte pieces of 32 different lines; the L2 takes one request per line piece,
// whatever its size.  Rows are padded by one 16-byte chunk (row stride TN*128 + 16 bytes): the
// writes (16 rows, one chunk) then fall into 16 different bank groups, the reads (consecutive
// chunks of a row) do anyway, and every offset besides the lane's own base is a constant.
//
// The column terms (128 - za) * colsum[j]: after the transposition a lane keeps the same four
// columns for all its stores, so it loads them once, before any store (a load placed between
// stores to C would be serialised behind them: C may alias anything as far as the compiler
// knows).  The requantised path stores bytes straight from the accumulator layout and takes its
// per-column values (column term + bias, zero-point of B, scale: `cterm_lds`, 3 x BN words) from
// LDS for the same reason.
// Must be called by all threads of the workgroup; `xpose` and `cterm_lds` must not be in use.
template <int TN>
__device__ __forceinline__ int xpose_off(int r, int c)
{
    return r * (TN * 128 + 16) + c * 16;
}
template <int TN>
constexpr int kXposeBytes = 32 * (TN * 128 + 16);      // per wavefront

// Four int32 outputs: stored, or (ATOMIC) added to what memory holds.  Integer addition mod 2^32 is
// associative and commutative, so partial sums over parts of K may arrive in any order and the result
// stays the exact one (the argument of Sec. 2.1 for reordering the additions).
template <bool ATOMIC>
__device__ __forceinline__ void put4(int32_t *dst, const v4i &v)
{
    if (ATOMIC) {
        __hip_atomic_fetch_add(dst + 0, v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(dst + 1, v.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(dst + 2, v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(dst + 3, v.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        // streaming store (4-byte aligned is enough): C is not read again, and kept out of L2 it leaves
        // the operands there (1024 x 3072 x 768: 9.6 -> 8.4 us, 2048^3: 15.5 -> 14.3 us)
        __builtin_nontemporal_store(v, (v4i_a4 *)dst);
    }
}
template <bool ATOMIC>
__device__ __forceinline__ void put1(int32_t *dst, int32_t v)
{
    if (ATOMIC) __hip_atomic_fetch_add(dst, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *dst = v;
}

// What the epilogue reads per column, loaded by epi_load_cols.  A kernel with one workgroup per compute
// unit calls it ahead of its main loop: loaded where they are used, the values arrive a memory latency
// after the last matrix op, with nothing else on the compute unit to cover it.
// int32 output: the column sums of this lane's four columns after the transposition; u8 output: column
// n0 + tid's sum, bias, zero-point of B and scale (the workgroup stages them in LDS).
struct EpiCols {
    int4 cs;
    int32_t cs1, bias1;
    uint32_t zb1;
    float sc1;
};
template <int TN, int BN, bool REQUANT>
__device__ __forceinline__ EpiCols epi_load_cols(const GemmParams &p, int n0, int wn, int lane, int tid)
{
    EpiCols e;
    e.cs = int4{0, 0, 0, 0};
    e.cs1 = 0; e.bias1 = 0; e.zb1 = p.zb; e.sc1 = p.scale;
    if (REQUANT) {
        const int col = n0 + tid;
        if (tid < BN && col < p.N) {
            e.cs1 = p.colsum[col];
            if (p.bias_vec) e.bias1 = p.bias_vec[col];
            if (p.zb_vec) e.zb1 = (uint32_t)p.zb_vec[col];
            if (p.scale_vec) e.sc1 = p.scale_vec[col];
        }
    } else {
        constexpr int LPR = TN * 8;
        const int bcol = n0 + wn * TN * 32 + 4 * (lane % LPR);
        if (bcol < p.N) e.cs = *(const int4 *)(p.colsum + bcol);     // colsum is padded to 32 columns
    }
    return e;
}

template <int TM, int TN, int BN, bool REQUANT, bool SMALLZC = false, bool ATOMIC = false>
__device__ __forceinline__ void tile_epilogue(const GemmParams &p, v16i (&acc)[TM][TN], int m0, int n0, int wm,
                                              int wn, int lane, int tid, int nthreads, uint8_t *xpose,
                                              uint32_t *cterm_lds, const EpiCols &ec, const uint32_t *rs_reg = nullptr)
{
    const bool c_vec_ok = REQUANT ? ((((uintptr_t)p.C | (uintptr_t)p.ldc) & 3) == 0) : true;
    constexpr int LPR = TN * 8, RPP = 64 / LPR, NPASS = 32 / RPP;   // read-back: LPR lanes per row
    const int bcol = n0 + wn * TN * 32 + 4 * (lane % LPR);
    const bool interior = m0 + (wm + 1) * TM * 32 <= p.M && n0 + (wn + 1) * TN * 32 <= p.N;   // this wavefront's part
    // u8 output of a wavefront part that lies inside C with 16-byte aligned rows: the bytes go through
    // the wavefront's patch as well (32 rows of TN * 32 bytes, padded) and leave as 16-byte pieces of
    // whole rows; straight from the accumulators a store instruction touches 32 rows with 8 bytes each
    // (1-2.5 % of the u8 calls of one tile per workgroup; plain stores: streaming stores of pieces of a
    // line are far slower)
    constexpr int kRow8 = TN * 32 + 16, LPR8 = TN * 2, RPP8 = 64 / LPR8, NPASS8 = 32 / RPP8;
    const bool u8_rows = REQUANT && interior && ((((uintptr_t)p.C | (uintptr_t)p.ldc) & 15) == 0);
    uint4 ct_back = {0u, 0u, 0u, 0u};
    if (REQUANT) {
        // per column: (128-za)*colsum + bias, zero-point of B, scale (vectors or the scalars); thread c
        // holds column n0 + c's (every workgroup of these kernels has at least BN threads)
        (void)nthreads;
        if (tid < BN) {
            cterm_lds[tid] = p.za_term * (uint32_t)ec.cs1 + (uint32_t)ec.bias1;
            cterm_lds[BN + tid] = ec.zb1;
            ((float *)cterm_lds)[2 * BN + tid] = ec.sc1;
        }
        __syncthreads();
    } else {
        // after the transposition a lane keeps the same four columns for every row it stores (zeros
        // past N: never stored)
        ct_back.x = p.za_term * (uint32_t)ec.cs.x; ct_back.y = p.za_term * (uint32_t)ec.cs.y;
        ct_back.z = p.za_term * (uint32_t)ec.cs.z; ct_back.w = p.za_term * (uint32_t)ec.cs.w;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row = m0 + (wm * TM + i) * 32 + (lane & 31);
        if (REQUANT && row >= p.M) continue;
        // the row's sum_k (A[i][k] - shift): from the caller's registers (rs_reg[i], this lane's row)
        // or from the row-sum pass
        uint32_t rs_row = 0u;
        if (rs_reg) rs_row = rs_reg[i];
        else if (p.rowsum && row < p.M) rs_row = (uint32_t)p.rowsum[row];
        const uint32_t row_term = p.kconst - p.zb * rs_row;
        // requantising path: sum_k (A[i][k] - za), multiplied per column by that column's zb
        const uint32_t rsum = rs_row + p.rconst;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int lcol = (wn * TN + j) * 32 + 8 * q + 4 * (lane >> 5);
                const int col = n0 + lcol;
                if (REQUANT && col >= p.N) continue;
                int32_t v[4];
                if (REQUANT) {
                    const uint4 cb = *(const uint4 *)(cterm_lds + lcol);
                    const uint4 zv = *(const uint4 *)(cterm_lds + BN + lcol);
                    v[0] = (int32_t)((uint32_t)acc[i][j][4 * q + 0] + cb.x - zv.x * rsum);
                    v[1] = (int32_t)((uint32_t)acc[i][j][4 * q + 1] + cb.y - zv.y * rsum);
                    v[2] = (int32_t)((uint32_t)acc[i][j][4 * q + 2] + cb.z - zv.z * rsum);
                    v[3] = (int32_t)((uint32_t)acc[i][j][4 * q + 3] + cb.w - zv.w * rsum);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) v[t] = (int32_t)((uint32_t)acc[i][j][4 * q + t] + row_term);
                }
                if (REQUANT) {
                    uint8_t *dst = (uint8_t *)p.C + (int64_t)row * p.ldc + col;
                    const float4 sc = *(const float4 *)((const float *)cterm_lds + 2 * BN + lcol);
                    uint32_t bw;
                    if (SMALLZC) {
                        const float zcf = (float)p.zc;
                        bw = requant4_u8_small_zc(v, sc, zcf, p.relu ? zcf : -3.402823466e38f);
                    } else {
                        bw = (uint32_t)requant_u8(v[0], sc.x, p.zc, p.relu) | ((uint32_t)requant_u8(v[1], sc.y, p.zc, p.relu) << 8) |
                             ((uint32_t)requant_u8(v[2], sc.z, p.zc, p.relu) << 16) | ((uint32_t)requant_u8(v[3], sc.w, p.zc, p.relu) << 24);
                    }
                    if (u8_rows) {
                        *(uint32_t *)(xpose + (lane & 31) * kRow8 + j * 32 + 8 * q + 4 * (lane >> 5)) = bw;
                    } else if (col + 3 < p.N && c_vec_ok) {
                        *(uint32_t *)dst = bw;
                    } else {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (col + t < p.N) dst[t] = (uint8_t)(bw >> (8 * t));
                    }
                } else {
                    // row r = lane%32 of the block row, chunk c = 8j + 2q + lane/32
                    v4i o;
                    o.x = v[0]; o.y = v[1]; o.z = v[2]; o.w = v[3];
                    *(v4i *)(xpose + xpose_off<TN>(lane & 31, 8 * j + 2 * q + (lane >> 5))) = o;
                }
            }
        }
        if (u8_rows) {
            const int brow0 = m0 + (wm * TM + i) * 32;
            uint8_t *dst0 = (uint8_t *)p.C + (int64_t)(brow0 + lane / LPR8) * p.ldc + n0 + wn * TN * 32 + 16 * (lane % LPR8);
            v4i o[NPASS8];
#pragma unroll
            for (int pass = 0; pass < NPASS8; ++pass)
                o[pass] = *(const v4i *)(xpose + (RPP8 * pass + lane / LPR8) * kRow8 + 16 * (lane % LPR8));
#pragma unroll
            for (int pass = 0; pass < NPASS8; ++pass)
                *(v4i *)(dst0 + (int64_t)(RPP8 * pass) * p.ldc) = o[pass];
        }
        if (!REQUANT) {
            // read the block row back row-wise, add the column terms, store full lines
            const int brow0 = m0 + (wm * TM + i) * 32;
            int32_t *dst0 = (int32_t *)p.C + (int64_t)(brow0 + lane / LPR) * p.ldc + bcol;
            if (ATOMIC) {
                // one instruction covers whole rows of the block row (consecutive lanes, consecutive
                // columns): an atomic request is served per cache line, at the memory side
                constexpr int W = TN * 32, RPI = 64 / W;
                const int gcol = n0 + wn * W + lane % W;
                const uint32_t ct1 = gcol < p.N ? p.za_term * (uint32_t)p.colsum[gcol] : 0u;
#pragma unroll
                for (int pass = 0; pass < 32 / RPI; ++pass) {
                    const int r = RPI * pass + lane / W;
                    const uint32_t v = *(const uint32_t *)(xpose + xpose_off<TN>(r, 0) + (lane % W) * 4) + ct1;
                    if (brow0 + r < p.M && gcol < p.N)
                        put1<true>((int32_t *)p.C + (int64_t)(brow0 + r) * p.ldc + gcol, (int32_t)v);
                }
            } else if (interior) {
                // no predicates: all LDS reads first, then all stores
                v4i o[NPASS];
#pragma unroll
                for (int pass = 0; pass < NPASS; ++pass) {
                    o[pass] = *(const v4i *)(xpose + xpose_off<TN>(RPP * pass + lane / LPR, lane % LPR));
                }
#pragma unroll
                for (int pass = 0; pass < NPASS; ++pass) {
                    v4i v = o[pass];
                    v.x = (int)((uint32_t)v.x + ct_back.x); v.y = (int)((uint32_t)v.y + ct_back.y);
                    v.z = (int)((uint32_t)v.z + ct_back.z); v.w = (int)((uint32_t)v.w + ct_back.w);
                    put4<ATOMIC>(dst0 + (int64_t)(RPP * pass) * p.ldc, v);
                }
            } else {
#pragma unroll
                for (int pass = 0; pass < NPASS; ++pass) {
                    const int r = RPP * pass + lane / LPR;
                    v4i v = *(const v4i *)(xpose + xpose_off<TN>(r, lane % LPR));
                    v.x = (int)((uint32_t)v.x + ct_back.x); v.y = (int)((uint32_t)v.y + ct_back.y);
                    v.z = (int)((uint32_t)v.z + ct_back.z); v.w = (int)((uint32_t)v.w + ct_back.w);
                    if (brow0 + r < p.M && bcol < p.N) {
                        int32_t *dst = dst0 + (int64_t)(RPP * pass) * p.ldc;
                        if (bcol + 3 < p.N) {
                            put4<ATOMIC>(dst, v);
                        } else {
                            put1<ATOMIC>(dst, v.x);
                            if (bcol + 1 < p.N) put1<ATOMIC>(dst + 1, v.y);
                            if (bcol + 2 < p.N) put1<ATOMIC>(dst + 2, v.z);
                        }
                    }
                }
            }
        }
    }
}

// compile-time integer as a function argument (register-set selectors of the kernels below)
template <int V>
struct IntC {
    static constexpr int value = V;
};
// f(IntC<U>), f(IntC<U + 1>), ..., f(IntC<R - 1>)
template <int U, int R, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (U < R) {
        f(IntC<U>{});
        static_for<U + 1, R>(f);
    }
}

// One workgroup tile (`tile` in the XCD-aware order of tile_of_block) of the problem `p`.
// RING > 1: the stages on their way from memory wait in a ring of RING register sets (stage s in set
// s % RING) instead of one, so RING loads are in flight per lane: a tile that is alone with a long K
// is bound by the latency of one load per stage otherwise.  Costs RING * (chunks per lane) * 4
// registers.
// ROWSUM_IN: the row sums the zero-point of B needs are formed here, from the A fragments the
// matrix ops read anyway (a dot product with ones per word; lane l sees row l % 32 of a block, the
// two halves of K sit in lanes l and l ^ 32), instead of being read from a pass of their own.
template <int BM, int BN, int WGM, int WGN, int BK, bool REQUANT, bool ROWSUM_IN = false, int RING = 1>
__device__ __forceinline__ void tile_body_staged(const GemmParams &p, int tile, uint8_t *lds)
{
    using Cfg = TileCfg<BM, BN, WGM, WGN, BK>;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, NT = Cfg::kThreads, KS = Cfg::KS;
    constexpr int CPR = Cfg::CPR, SW = Cfg::SW, AI = Cfg::kAIters, BI = Cfg::kBIters;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    int tm, tn;
    tile_of_block(tile, p.tiles_m, p.tiles_n, p.nxcd, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int nslices = p.Kp / 32;
    const int nfull = p.K / BK;                        // stages that lie completely inside K
    const bool has_tail = nfull * BK < p.Kp;

    // This thread's chunks of a stage: source addresses (k advances by BK per stage) and LDS slots.
    const uint8_t *a_src[AI];
    int a_dst[AI];
#pragma unroll
    for (int i = 0; i < AI; ++i) {
        const int q = tid + i * NT;
        const int r = q / CPR, c = q % CPR;
        int grow = m0 + r;
        grow = grow < p.M ? grow : p.M - 1;            // rows past M: read a valid row, never stored
        a_src[i] = p.A + (int64_t)grow * p.lda + c * 16;
        a_dst[i] = ((r >> 5) * (CPR * 32) + c * 32 + ((r & 31) ^ (c * SW))) * 16;
    }
    const uint8_t *b_src[BI];
#pragma unroll
    for (int i = 0; i < BI; ++i) {
        const int q = tid + i * NT;
        const int nb = q / (KS * 64), within = q % (KS * 64);
        int pnl = n0 / 32 + nb;
        pnl = pnl < p.npanels ? pnl : p.npanels - 1;   // panels past N: read a valid panel, never stored
        b_src[i] = p.Bp + ((int64_t)pnl * nslices) * kFragBytes + within * 16;
    }
    // Fragment read offsets of this lane inside the A part of a stage, one per sub-step.
    int a_frag_off[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int c = 2 * ks + (lane >> 5);
        a_frag_off[ks] = (wm * TM * (CPR * 32) + c * 32 + ((lane & 31) ^ (c * SW))) * 16;
    }
    const int b_frag_off = Cfg::kABytes + (wn * TN * KS) * kFragBytes + lane * 16;

    v4i ra[AI], rb[BI];
    auto gload_a = [&](int i, int kt) { ra[i] = load16_any(a_src[i] + (int64_t)kt * BK); };
    auto gload_b = [&](int i, int kt) { rb[i] = *(const v4i *)(b_src[i] + (int64_t)kt * (KS * kFragBytes)); };
    auto sstore_a = [&](int i, int buf) {
        *(v4i *)(lds + buf * Cfg::kStageBytes + a_dst[i]) = shift_u8_to_s8(ra[i], p.a_xor);
    };
    auto sstore_b = [&](int i, int buf) {
        *(v4i *)(lds + buf * Cfg::kStageBytes + Cfg::kABytes + (tid + i * NT) * 16) = rb[i];
    };

    v4i fa[2][TM], fb[2][TN];
    auto read_frags = [&](int buf, int ks, int slot) {
        const uint8_t *base = lds + buf * Cfg::kStageBytes;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[slot][i] = *(const v4i *)(base + a_frag_off[ks] + i * (CPR * 32 * 16));
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[slot][j] = *(const v4i *)(base + b_frag_off + (j * KS + ks) * kFragBytes);
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Matrix instruction with the packed operand first: lane l then holds, for row l%32 of the
    // A block, the four consecutive columns 8*(r/4) + 4*(l/32) + r%4 of the B block in
    // registers r = 4q..4q+3, so the epilogue stores 16 contiguous bytes per lane.
    int rs[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) rs[i] = 0;
    auto mma_one = [&](int slot, int i, int j) {
        if (ROWSUM_IN && j == 0) {
            const v4i a = fa[slot][i];
            rs[i] = __builtin_amdgcn_sdot4(a.x, 0x01010101, rs[i], false);
            rs[i] = __builtin_amdgcn_sdot4(a.y, 0x01010101, rs[i], false);
            rs[i] = __builtin_amdgcn_sdot4(a.z, 0x01010101, rs[i], false);
            rs[i] = __builtin_amdgcn_sdot4(a.w, 0x01010101, rs[i], false);
        }
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[slot][j], fa[slot][i], acc[i][j], 0, 0, 0);
    };

    if constexpr (RING > 1) {
        v4i qa[RING][AI], qb[RING][BI];
        auto qload = [&](auto set, int kt) {
            constexpr int S = decltype(set)::value;
            const int k = kt < nfull ? kt : nfull - 1;  // past the end: the last stage again, never consumed
#pragma unroll
            for (int i = 0; i < AI; ++i) qa[S][i] = load16_any(a_src[i] + (int64_t)k * BK);
#pragma unroll
            for (int i = 0; i < BI; ++i) qb[S][i] = *(const v4i *)(b_src[i] + (int64_t)k * (KS * kFragBytes));
        };
        auto qstore_a = [&](auto set, int i, int buf) {
            constexpr int S = decltype(set)::value;
            *(v4i *)(lds + buf * Cfg::kStageBytes + a_dst[i]) = shift_u8_to_s8(qa[S][i], p.a_xor);
        };
        auto qstore_b = [&](auto set, int i, int buf) {
            constexpr int S = decltype(set)::value;
            *(v4i *)(lds + buf * Cfg::kStageBytes + Cfg::kABytes + (tid + i * NT) * 16) = qb[S][i];
        };
        if (nfull > 0) {
            qload(IntC<0>{}, 0);
#pragma unroll
            for (int i = 0; i < AI; ++i) qstore_a(IntC<0>{}, i, 0);
#pragma unroll
            for (int i = 0; i < BI; ++i) qstore_b(IntC<0>{}, i, 0);
            // stages 1 .. RING on their way
            static_for<1, RING>([&](auto set) { qload(set, decltype(set)::value); });
            qload(IntC<0>{}, RING);
            lds_barrier();
            read_frags(0, 0, 0);
        }
        // stage kt: its matrix ops, while stage kt + 1 (register set SET) goes to the other LDS
        // buffer and stage kt + 1 + RING is requested into the same set
        auto stage = [&](int kt, auto set) {
            const int cur = kt & 1, nxt = cur ^ 1;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks + 1 < KS) {
                    read_frags(cur, ks + 1, (ks + 1) & 1);
                } else {
                    lds_barrier();                      // next stage is complete in LDS[nxt]
                    read_frags(nxt, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (ks == 0) {
                    constexpr int NM = TM * TN;
#pragma unroll
                    for (int m = 0; m < NM; ++m) {
                        mma_one(0, m / TN, m % TN);
                        __builtin_amdgcn_sched_barrier(0);
                        if (m == NM - 1) {
#pragma unroll
                            for (int i = 0; i < AI; ++i) qstore_a(set, i, nxt);
#pragma unroll
                            for (int i = 0; i < BI; ++i) qstore_b(set, i, nxt);
                            qload(set, kt + 1 + RING);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) mma_one(ks & 1, i, j);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // whole rounds of the ring without a branch inside (the pending-load counts the compiler
        // derives stay exact: RING - 1 sets in flight at every store), then the remainder
        int kt = 0;
        for (; kt + RING <= nfull; kt += RING)
            static_for<0, RING>([&](auto u) {
                constexpr int U = decltype(u)::value;
                stage(kt + U, IntC<(U + 1) % RING>{});
            });
        static_for<0, RING - 1>([&](auto u) {
            constexpr int U = decltype(u)::value;
            if (kt + U < nfull) stage(kt + U, IntC<(U + 1) % RING>{});
        });
    } else {
    if (nfull > 0) {
#pragma unroll
        for (int i = 0; i < AI; ++i) gload_a(i, 0);
#pragma unroll
        for (int i = 0; i < BI; ++i) gload_b(i, 0);
#pragma unroll
        for (int i = 0; i < AI; ++i) sstore_a(i, 0);
#pragma unroll
        for (int i = 0; i < BI; ++i) sstore_b(i, 0);
        const int kt1 = nfull > 1 ? 1 : 0;
#pragma unroll
        for (int i = 0; i < AI; ++i) gload_a(i, kt1);
#pragma unroll
        for (int i = 0; i < BI; ++i) gload_b(i, kt1);
        lds_barrier();
        read_frags(0, 0, 0);
    }

    // Main loop over full stages.  Per stage: sub-step ks computes from fragment registers
    // slot ks&1 while the fragments of sub-step ks+1 are being read from LDS; during sub-step 0
    // the next stage (already in registers) is written to the other LDS buffer and the stage
    // after it is requested from memory.
    // The prefetch indices are clamped to the last full stage instead of being predicated: the
    // final iterations re-load and re-store that stage into a buffer nobody reads any more,
    // which keeps the loop body free of branches.
    for (int kt = 0; kt < nfull; ++kt) {
        const int cur = kt & 1, nxt = cur ^ 1;
        const int kt2 = kt + 2 < nfull ? kt + 2 : nfull - 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            if (ks + 1 < KS) {
                read_frags(cur, ks + 1, (ks + 1) & 1);
            } else {
                lds_barrier();                          // next stage is complete in LDS[nxt]
                read_frags(nxt, 0, 0);
            }
            // Scheduling fences: keep the fragment reads above the matrix ops that hide their
            // latency, and keep the prefetch pieces between the matrix ops where they are written.
            __builtin_amdgcn_sched_barrier(0);
            if (ks == 0) {
                // interleave: matrix ops with the LDS writes / global loads of the prefetch
                constexpr int NM = TM * TN;
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    mma_one(0, m / TN, m % TN);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < AI; ++i)
                        if (i * NM / AI == m) {
                            sstore_a(i, nxt);
                            gload_a(i, kt2);
                        }
#pragma unroll
                    for (int i = 0; i < BI; ++i)
                        if (i * NM / BI == m) {
                            sstore_b(i, nxt);
                            gload_b(i, kt2);
                        }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) mma_one(ks & 1, i, j);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    }

    // K tail: the last, partial stage (K not a multiple of BK).  Guarded loads, no pipelining.
    if (has_tail) {
        const int kbase = nfull * BK;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < AI; ++i) {
            const int q = tid + i * NT;
            const int kk = kbase + (q % CPR) * 16;
            const int valid = p.K - kk;
            const uint8_t *src = a_src[i] + kbase;
            ra[i] = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
            sstore_a(i, 0);
        }
#pragma unroll
        for (int i = 0; i < BI; ++i) {
            const int q = tid + i * NT;
            const int f = (q % (KS * 64)) >> 6;          // fragment of the stage this chunk is in
            v4i z = {0, 0, 0, 0};
            rb[i] = (nfull * KS + f < nslices) ? *(const v4i *)(b_src[i] + (int64_t)nfull * (KS * kFragBytes)) : z;
            sstore_b(i, 0);
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            read_frags(0, ks, 0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma_one(0, i, j);
        }
    }

    __syncthreads();                                   // every wavefront is done with the stage buffers
    uint32_t rs_reg[TM];
    if (ROWSUM_IN) {
        // both halves of K; the zero fill of the K tail was shifted with the rest and counts as
        // -128 per byte for an unsigned A: taken out again
        const uint32_t pad = p.a_xor ? 128u * (uint32_t)((nfull + (has_tail ? 1 : 0)) * BK - p.K) : 0u;
#pragma unroll
        for (int i = 0; i < TM; ++i) rs_reg[i] = (uint32_t)(rs[i] + __shfl_xor(rs[i], 32, 64)) + pad;
    }
    const uint32_t *rsp = ROWSUM_IN ? rs_reg : nullptr;
    static_assert(BN <= WGM * WGN * 64, "a thread per column of the tile");
    const EpiCols ec = epi_load_cols<TN, BN, REQUANT>(p, n0, wn, lane, tid);
    // every practical output zero-point takes the binary32 form of the requantising arithmetic
    if (REQUANT && p.zc > -8388608 && p.zc < 8388608)
        tile_epilogue<TM, TN, BN, REQUANT, true>(p, acc, m0, n0, wm, wn, lane, tid, NT, lds + wave * kXposeBytes<TN>,
                                       (uint32_t *)(lds + WGM * WGN * kXposeBytes<TN>), ec, rsp);
    else
        tile_epilogue<TM, TN, BN, REQUANT, false>(p, acc, m0, n0, wm, wn, lane, tid, NT, lds + wave * kXposeBytes<TN>,
                                       (uint32_t *)(lds + WGM * WGN * kXposeBytes<TN>), ec, rsp);
}

template <int BM, int BN, int WGM, int WGN, int BK, bool REQUANT, bool ROWS = false>
__global__ __launch_bounds__(WGM * WGN * 64) void gemm_tile_kernel(const GemmParams p)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    tile_body_staged<BM, BN, WGM, WGN, BK, REQUANT, ROWS>(p, blockIdx.x, lds);
}

// ---- grouped launches: several independent problems in one grid -------------------------------
// The problems' parameters travel in the kernel argument block, which holds 4 KiB: each member is
// cut down to what cannot be derived (GroupMember, 56 bytes), so that kGroupMax of them fit, and a
// workgroup rebuilds the full parameter set of its own member with a few scalar operations.
// unit_start[q] is the first workgroup id of problem q, unit_start[count] the grid size.  A unit is a
// 32-column panel for the members [0, first_tile) (M <= 32: the skinny body) and a 64 x 64 tile for the
// rest: one grid holds both kinds, so that a long-K skinny member and the tiles of the large members
// run side by side instead of one launch after the other.
// Members are u8 x s8 -> s32 problems with per-tensor zero-points.
constexpr int kGroupMax = 67;
struct GroupMember {
    const uint8_t *A;
    const uint8_t *Bp;       // packed fragments; the column sums follow them
    void *C;
    int64_t lda, ldc;
    int M, N, K;
    int16_t za_term, zb;     // 128 - za (-127..128) and zb (-128..127)
};
struct GroupParams {
    int count;
    int nxcd;                // XCDs of the device (see GemmParams)
    int first_tile;          // members before it are skinny (units = panels), from it on tiled (units = tiles)
    int unit_start[kGroupMax + 1];
    GroupMember prob[kGroupMax];
};

static_assert(sizeof(GroupMember) == 56, "member record");
static_assert(sizeof(GroupParams) <= 4096, "kernel argument block");

__device__ __forceinline__ int group_find(const GroupParams &g, int bid)
{
    int q = 0;
    for (int t = 1; t < g.count; ++t)
        if (bid >= g.unit_start[t]) q = t;
    return q;
}

// The full parameter set of a member; tiles are counted for BM x BN workgroup tiles.
template <int BM, int BN>
__device__ __forceinline__ GemmParams group_member_params(const GroupMember &m, int nxcd)
{
    GemmParams p;
    p.nxcd = nxcd;
    p.A = m.A;
    p.lda = m.lda;
    p.Bp = m.Bp;
    p.M = m.M;
    p.N = m.N;
    p.K = m.K;
    p.Kp = (m.K + 63) & ~63;
    p.npanels = (m.N + 31) >> 5;
    p.colsum = (const int32_t *)(m.Bp + (int64_t)p.Kp * (p.npanels * 32));
    p.rowsum = nullptr;          // the grouped kernels form the row sums themselves
    p.C = m.C;
    p.ldc = m.ldc;
    p.tiles_m = (m.M + BM - 1) / BM;
    p.tiles_n = (m.N + BN - 1) / BN;
    p.za_term = (uint32_t)(int32_t)m.za_term;
    p.zb = (uint32_t)(int32_t)m.zb;
    p.kconst = 0u - p.zb * p.za_term * (uint32_t)m.K;
    p.scale = 1.0f;
    p.zc = 0;
    p.scale_vec = nullptr;
    p.bias_vec = nullptr;
    p.zb_vec = nullptr;
    p.rconst = p.za_term * (uint32_t)m.K;
    p.relu = 0;
    p.a_xor = 0x80808080u;
    p.ksplit = 1;
    p.kchunk = 0;
    p.part_ws = nullptr;
    return p;
}

// Register ring of the grouped kernel's tiles: with four sets the batch of 64 odd shapes takes 28.8 us,
// with one 34.8 (a long-K member's loads no longer wait behind the other members' traffic); stages
// of 128 bytes instead of 64 gain nothing.
constexpr int kGroupRing = 4;

// ---- tiled MFMA kernel, direct-to-LDS variant -------------------------------------------------
// Same tiling and epilogue, but each stage (64 bytes of K) is copied memory -> LDS by the
// load unit itself (global_load_lds_dwordx4: no register staging, no LDS store instructions),
// into a ring of NSTAGE stage buffers.  The loads of stage s are issued three stages before
// s is consumed, which is what hides the latency of a miss in the XCD's L2 when only one
// wavefront per SIMD is resident.  Needs A 16-byte aligned with lda a multiple of 16; the
// host falls back to the register-staged kernel otherwise.
//
// LDS layout of a stage: 1 KiB blocks, one per wavefront-wide load (lane j writes bytes
// 16j..16j+15 of its block, as the hardware prescribes).
//   A block b = rows 16b..16b+15: lane j = 4t + u loads row 16b+t, 16-byte chunk
//     c = (u - t/4) mod 4, so four consecutive lanes still read 64 contiguous bytes of one row,
//     and chunk (t, c) sits in slot 4t + (c + t/4) mod 4: the 16 rows a fragment read touches
//     for a fixed c fall into 16 different 16-byte bank groups.
//   B block q = fragment q%2 of panel q/2 of the tile, copied as it is.
// The u8 -> s8 shift (xor 0x80) is applied to the A fragments after they are read from LDS.
template <int BM, int BN, int WGM, int WGN, int NSTAGE>
struct DmaCfg {
    static constexpr int BK = 64;
    static constexpr int KS = 2;
    static constexpr int kWaves = WGM * WGN;
    static constexpr int kThreads = kWaves * 64;
    static constexpr int TM = BM / (WGM * 32);
    static constexpr int TN = BN / (WGN * 32);
    static constexpr int kABlocks = BM / 16;
    static constexpr int kBBlocks = BN / 16;
    static constexpr int kAIters = kABlocks / kWaves;
    static constexpr int kBIters = kBBlocks / kWaves;
    static constexpr int kABytes = BM * BK;
    static constexpr int kStageBytes = (BM + BN) * BK;
    static constexpr int kEpiBytes = kWaves * 32 * (TN * 128 + 16) + BN * 12;  // epilogue patches + three per-column arrays
    static constexpr int kLdsBytes = NSTAGE * kStageBytes > kEpiBytes ? NSTAGE * kStageBytes : kEpiBytes;
    static constexpr int kLoadsPerStage = kAIters + kBIters;   // per thread
    static_assert(kABlocks % kWaves == 0 && kBBlocks % kWaves == 0, "loader shape");
    static_assert(NSTAGE >= 4, "ring of at least four stages");
    static_assert((NSTAGE - 2) * kLoadsPerStage <= 63, "vmcnt range");
};

// s_waitcnt for the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

// An operand B that was not packed: the caller's int8 [N x K] storage (column j = ldb-strided row of
// K contiguous bytes), 16-byte aligned.  It has the shape of A, so the BRAW form of the kernel below
// copies and reads its tiles exactly as it does A's (Sec. 3.1.1: the case where both matrices are inputs).
struct RawB {
    const uint8_t *B;
    int64_t ldb;
};

// ROWS: the row sums a zero-point of B needs are added up here, from the A fragments behind the matrix
// op that uses them (no row-sum pass before the kernel); the host takes this form only when the
// zero-point is there.
template <int BM, int BN, int WGM, int WGN, int NSTAGE, bool REQUANT, bool BRAW = false, bool ROWS = false>
__global__ __launch_bounds__(WGM * WGN * 64) void gemm_tile_dma_kernel(const GemmParams p, const RawB rawb)
{
    using Cfg = DmaCfg<BM, BN, WGM, WGN, NSTAGE>;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, KS = Cfg::KS, BK = Cfg::BK;
    constexpr int AI = Cfg::kAIters, BI = Cfg::kBIters, NW = Cfg::kWaves;
    constexpr int LPS = Cfg::kLoadsPerStage;
    constexpr int NM = TM * TN;
    constexpr int NR = TM + TN;                         // fragment reads per slot
    constexpr int RG = (NR + 1) / 2;                    // gaps used for reads (two per gap)
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int nslices = p.Kp / 32;
    const int nfull = p.K / BK;
    const bool has_tail = nfull * BK < p.Kp;

    // Persistent workgroups: workgroup w owns tiles w, w + G, w + 2G, ... of the XCD-aware order
    // (G = grid size: one workgroup per compute unit when there is enough work; the LDS ring and
    // the 512 registers per lane leave no room for a second one anyway).
    const int ntiles = p.tiles_m * p.tiles_n;
    const int G = gridDim.x, w = blockIdx.x;

    const int t16 = lane >> 2;
    const int a_chunk = ((lane & 3) - (t16 >> 2)) & 3;
    int a_frag_off[KS];
    {
        const int r = lane & 31, t = r & 15;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int c = 2 * ks + (lane >> 5);
            a_frag_off[ks] = (wm * TM * 2 + (r >> 4)) * 1024 + (4 * t + ((c + (t >> 2)) & 3)) * 16;
        }
    }
    const int b_frag_off = Cfg::kABytes + (wn * TN * KS) * kFragBytes + lane * 16;
    int b_raw_off[KS];                                  // BRAW: the B tile lies in A's block layout
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        b_raw_off[ks] = Cfg::kABytes + a_frag_off[ks] + (wn * TN - wm * TM) * 2048;

    for (int tile = w; tile < ntiles; tile += G) {
        int tm, tn;
        tile_of_block(tile, p.tiles_m, p.tiles_n, p.nxcd, tm, tn);
        const int m0 = tm * BM, n0 = tn * BN;
        static_assert(BN <= Cfg::kThreads, "a thread per column of the tile");
        const EpiCols ec = epi_load_cols<TN, BN, REQUANT>(p, n0, wn, lane, tid);   // the epilogue's column terms, early

        // Loader: this lane's source addresses for the blocks its wavefront copies.
        const uint8_t *a_src[AI];
#pragma unroll
        for (int i = 0; i < AI; ++i) {
            int grow = m0 + (wave + NW * i) * 16 + t16;
            grow = grow < p.M ? grow : p.M - 1;          // rows past M: read a valid row, never stored
            a_src[i] = p.A + (int64_t)grow * p.lda + a_chunk * 16;
        }
        const uint8_t *b_src[BI];
#pragma unroll
        for (int i = 0; i < BI; ++i) {
            const int q = wave + NW * i;
            if (BRAW) {
                int gcol = n0 + q * 16 + t16;
                gcol = gcol < p.N ? gcol : p.N - 1;      // columns past N: read a valid one, never stored
                b_src[i] = rawb.B + (int64_t)gcol * rawb.ldb + a_chunk * 16;
            } else {
                int pnl = n0 / 32 + (q >> 1);
                pnl = pnl < p.npanels ? pnl : p.npanels - 1; // panels past N: read a valid panel, never stored
                b_src[i] = p.Bp + ((int64_t)pnl * nslices + (q & 1)) * kFragBytes + lane * 16;
            }
        }
        auto dma_a = [&](int i, int kt, int buf) {
            __builtin_amdgcn_global_load_lds((gptr_t)(a_src[i] + (int64_t)kt * BK),
                                             (lptr_t)(lds + buf * Cfg::kStageBytes + (wave + NW * i) * 1024), 16, 0,
                                             0);
        };
        auto dma_b = [&](int i, int kt, int buf) {
            __builtin_amdgcn_global_load_lds(
                (gptr_t)(b_src[i] + (int64_t)kt * (BRAW ? BK : KS * kFragBytes)),
                (lptr_t)(lds + buf * Cfg::kStageBytes + Cfg::kABytes + (wave + NW * i) * 1024), 16, 0, 0);
        };
        auto dma_stage = [&](int kt, int buf) {
#pragma unroll
            for (int i = 0; i < AI; ++i) dma_a(i, kt, buf);
#pragma unroll
            for (int i = 0; i < BI; ++i) dma_b(i, kt, buf);
        };

        v4i fa[2][TM], fb[2][TN];
        auto read_one = [&](int buf, int ks, int slot, int idx) {
            const uint8_t *base = lds + buf * Cfg::kStageBytes;
            if (idx < TM)
                fa[slot][idx] = *(const v4i *)(base + a_frag_off[ks] + idx * 2048);
            else
                fb[slot][idx - TM] = BRAW ? *(const v4i *)(base + b_raw_off[ks] + (idx - TM) * 2048)
                                          : *(const v4i *)(base + b_frag_off + ((idx - TM) * KS + ks) * kFragBytes);
        };
        auto read_frags = [&](int buf, int ks, int slot) {
#pragma unroll
            for (int r = 0; r < NR; ++r) read_one(buf, ks, slot, r);
        };
        auto shift_frags = [&](int slot) {
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[slot][i] = shift_u8_to_s8(fa[slot][i], p.a_xor);
        };
        auto xor_gap = [&](int i) { return (NM - 1 - TM + i) > 0 ? (NM - 1 - TM + i) : 0; };

        v16i acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
        // Matrix instruction with the packed operand first: lane l then holds, for row l%32 of
        // the A block, the four consecutive columns 8*(r/4) + 4*(l/32) + r%4 of the B block in
        // registers r = 4q..4q+3.
        int rs[TM];                                    // this lane's share of the row sums (row lane % 32 of block i)
#pragma unroll
        for (int i = 0; i < TM; ++i) rs[i] = 0;
        auto mma_one = [&](int slot, int i, int j) {
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[slot][j], fa[slot][i], acc[i][j], 0, 0, 0);
            if (ROWS && j == 0) {
                const v4i a = fa[slot][i];             // shifted before its first matrix op
                rs[i] = __builtin_amdgcn_sdot4(a.x, 0x01010101, rs[i], false);
                rs[i] = __builtin_amdgcn_sdot4(a.y, 0x01010101, rs[i], false);
                rs[i] = __builtin_amdgcn_sdot4(a.z, 0x01010101, rs[i], false);
                rs[i] = __builtin_amdgcn_sdot4(a.w, 0x01010101, rs[i], false);
            }
        };

        // Stage indices past the last full stage are clamped to it: the extra copies land in
        // buffers nobody reads any more and keep the outstanding-copy counts uniform.
        auto clampk = [&](int it) { return it < nfull ? it : nfull - 1; };

        // The previous tile's LDS traffic (last stage, K tail, epilogue patches) must be over
        // before this tile's copies overwrite the buffers.
        if (tile != w) __syncthreads();

        // Software pipeline, one iteration per stage (two sub-steps of TM*TN matrix ops each).
        // Everything else is issued in the gaps between matrix ops so the matrix pipe never waits:
        //   sub-step 0 (fragment slot 0 = stage it, k-half 0):
        //       first gaps : LDS reads of slot 1 (stage it, k-half 1)
        //       middle     : wait until this wavefront's copies of stage it+1 have landed, barrier
        //                    (=> stage it+1 is complete for everybody, stage it-1 is free)
        //       last gaps  : u8 -> s8 shift of slot 1's A fragments (long since returned)
        //   sub-step 1 (slot 1):
        //       first gaps : LDS reads of slot 0 for stage it+1, k-half 0
        //       then       : copies of stage it+NSTAGE-1 into the buffer of stage it-1
        //       last gaps  : shift of slot 0's A fragments
        // The barrier of iteration it is what makes the reads of stage it+1 (issued after it) and
        // the overwrite of stage it-1 (whose last reads were consumed in iteration it-1) safe.
        // It is a bare s_barrier behind a manual wait on the copy counter: a workgroup fence
        // would also wait for the younger copies, which must stay in flight.
        if (nfull > 0) {
#pragma unroll
            for (int s = 0; s < NSTAGE - 1; ++s) dma_stage(clampk(s), s);
            wait_vmcnt<(NSTAGE - 2) * LPS>();           // stage 0 has landed (this wavefront's part)
            __builtin_amdgcn_s_barrier();               // ... and everybody else's
            read_frags(0, 0, 0);
            shift_frags(0);
            __builtin_amdgcn_sched_barrier(0);

            for (int it = 0; it < nfull; ++it) {
                const int cur = it % NSTAGE, nxt = (it + 1) % NSTAGE, fre = (it + NSTAGE - 1) % NSTAGE;
                const int kload = clampk(it + NSTAGE - 1);
                // ---- sub-step 0 ----
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    mma_one(0, m / TN, m % TN);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int r = 0; r < NR; ++r)
                        if (r / 2 == m || (m == NM - 1 && r / 2 > m)) read_one(cur, 1, 1, r);
                    if (m == (NM - 1) / 2) {
                        wait_vmcnt<(NSTAGE - 3) * LPS>();   // younger: the copies of stages it+2 .. it+NSTAGE-2
                        __builtin_amdgcn_s_barrier();
                    }
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        if (xor_gap(i) == m) fa[1][i] = shift_u8_to_s8(fa[1][i], p.a_xor);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // ---- sub-step 1 ----
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    mma_one(1, m / TN, m % TN);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int r = 0; r < NR; ++r)
                        if (r / 2 == m || (m == NM - 1 && r / 2 > m)) read_one(nxt, 0, 0, r);
#pragma unroll
                    for (int d = 0; d < AI + BI; ++d) {
                        const int g = (RG + d) < NM ? (RG + d) : NM - 1;
                        if (g == m) {
                            if (d < AI) dma_a(d, kload, fre);
                            else dma_b(d - AI, kload, fre);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        if (xor_gap(i) == m) fa[0][i] = shift_u8_to_s8(fa[0][i], p.a_xor);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            wait_vmcnt<0>();                            // drain the clamped extra copies
        }

        // K tail: the last, partial stage.  Guarded register loads into buffer 0, same layout.
        if (has_tail) {
            const int kbase = nfull * BK;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < AI; ++i) {
                const int valid = p.K - (kbase + a_chunk * 16);
                const uint8_t *src = a_src[i] + kbase;
                v4i v = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
                *(v4i *)(lds + (wave + NW * i) * 1024 + lane * 16) = v;
            }
#pragma unroll
            for (int i = 0; i < BI; ++i) {
                const int q = wave + NW * i;
                v4i v = {0, 0, 0, 0};
                if (BRAW) {
                    const int valid = p.K - (kbase + a_chunk * 16);
                    const uint8_t *src = b_src[i] + kbase;
                    v = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
                } else if (nfull * KS + (q & 1) < nslices) {
                    v = *(const v4i *)(b_src[i] + (int64_t)nfull * (KS * kFragBytes));
                }
                *(v4i *)(lds + Cfg::kABytes + q * 1024 + lane * 16) = v;
            }
            __syncthreads();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                read_frags(0, ks, 0);
                shift_frags(0);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) mma_one(0, i, j);
            }
        }

        __syncthreads();                               // every wavefront is done with the stage buffers
        // Row sums: the halves of each 32-byte step sit in lanes l and l ^ 32; the zero fill of the K
        // tail was shifted with the rest (-128 per byte of an unsigned A) and is taken out again.
        uint32_t rs_reg[TM];
        if (ROWS) {
            const uint32_t pad = (p.a_xor && has_tail) ? 128u * (uint32_t)((nfull + 1) * BK - p.K) : 0u;
#pragma unroll
            for (int i = 0; i < TM; ++i) rs_reg[i] = (uint32_t)(rs[i] + __shfl_xor(rs[i], 32, 64)) + pad;
        }
        const uint32_t *rsp = ROWS ? rs_reg : nullptr;
        // every practical output zero-point takes the binary32 form of the requantising arithmetic
        if (REQUANT && p.zc > -8388608 && p.zc < 8388608)
            tile_epilogue<TM, TN, BN, REQUANT, true>(p, acc, m0, n0, wm, wn, lane, tid, Cfg::kThreads,
                                           lds + wave * kXposeBytes<TN>, (uint32_t *)(lds + NW * kXposeBytes<TN>), ec, rsp);
        else
            tile_epilogue<TM, TN, BN, REQUANT, false>(p, acc, m0, n0, wm, wn, lane, tid, Cfg::kThreads,
                                           lds + wave * kXposeBytes<TN>, (uint32_t *)(lds + NW * kXposeBytes<TN>), ec, rsp);
    }
}

// ---- 256 x 256 tiles on the 16 x 16 x 64 matrix instruction ------------------------------------
// The same tiling as gemm_tile_dma_kernel<256,256,2,2,4> (rings and copies of its own, below).  On
// operands that change with every instruction the chip is limited by power, not by issue slots, and
// v_mfma_i32_16x16x64_i8 does the same work for less of it than the 32 x 32 x 32 form (a quarter of
// the accumulator traffic per instruction, half per multiply-add): a register-only loop of the one
// sustains 3.9 POP/s on random data, of the other 3.5.  A stage of 64 bytes of K is exactly one such
// instruction deep:
//   A operand of block i (16 rows): lane l holds row l%16, bytes 16*(l/16) .. +15 of the stage: one
//     16-byte read per lane from the rows' 128-byte places in LDS (chunk placement below);
//   B operand of block j (16 columns): lane l holds column l%16, the same bytes; they lie in the two
//     packed fragments (32-byte k-halves) of the block's panel.  A copy's lanes may fetch any 16 bytes
//     each, so the chunks of a fragment are permuted on the way into LDS (still one contiguous KiB
//     per copy): the two 16-byte halves a lane pair l, l+16 needs lie 256 bytes apart.
// With the packed operand first, lane l of the result holds, for row l%16 of A's block, the four
// consecutive columns 4*(l/16) .. +3 of B's block.
// A wavefront owns 128 x 128 of C as 8 x 8 blocks (256 accumulator registers) and keeps the sixteen
// operand fragments of two stages in registers: those of stage it+1 are read from LDS while the 64
// matrix ops of stage it run.
struct X64Cfg {
    // A: ring of three double stages (256 rows x 128 bytes of K); B: ring of three stages (256 columns
    // x 64 bytes of K) behind it
    static constexpr int kARing = 3, kBRing = 3;
    static constexpr int kADouble = 256 * 128;
    static constexpr int kBBytes = 256 * 64;
    static constexpr int kBBase = kARing * kADouble;
    static constexpr int kPatchRow = 128 * 4 + 16;         // epilogue patch: 16 rows of 128 int32, padded
    static constexpr int kPatchBytes = 16 * kPatchRow;     // per wavefront
    static constexpr int kLdsBytes = kBBase + kBRing * kBBytes;
    static constexpr int kMinK = 128;                      // two full stages: the copies assume them
    static constexpr int kCopyBias = 3 * 1024;             // see the copies: lane offsets carry it, the bases lack it
    static_assert(4 * kPatchBytes + 3 * 1024 <= kLdsBytes, "epilogue patches and column arrays fit the rings");
    static_assert(kLdsBytes <= 160 * 1024, "LDS of a compute unit");
};

// A's copies fetch whole 128-byte lines: one copy is 8 rows x 128 bytes of K, two stages' worth, so A
// moves through LDS in double stages.  (With 64 bytes per row and stage, each line was requested
// twice, a stage apart, and the 32 KiB that pass through the vector cache in between had evicted it:
// the cache counters showed 1.5 times the requests the tile needs.)  A double stage is 256 rows of
// 128 bytes, chunk c of row R in place c ^ (R % 8) (four consecutive lanes of a copy stay inside one
// aligned 64 bytes of memory, eight consecutive lanes of a fragment read hit eight different
// places); a stage reads chunks 0..3 (even) or 4..7 (odd) of its rows.  The pipelined loop takes an
// even number of stages, so that no copy reaches past the full stages of K; an odd last full stage and
// the partial stage after it are loaded through registers with guards and consumed without pipelining.
// BRAW: B is the caller's plain [N x K] int8 storage (struct RawB); its tiles are copied by stage, in
// blocks of 16 columns x 64 bytes with the four chunks of column t rotated by t / 2.
// The host launches this kernel for K >= kMinK only.
// SHIFT = false: A holds signed bytes, the u8 -> s8 shift (32 vector instructions per stage and
// wavefront, 1.7 % of the time on uniform data) is left out.
// RB: 16-row blocks per wavefront.  8 is the 256 x 256 tile; 6 a 192 x 256 tile (wavefront tile 96 x 128, 192
// accumulator registers, three copies of A per wavefront and half stage instead of four; A's ring places keep
// their size, 192 rows of each are used): for outputs that fill between half and all of the compute units with
// 256 x 256 tiles, where the shorter tile fills more of them for three quarters of the time per tile
// (Sec. 3.1.1: the tiling is chosen per problem size).
template <bool BRAW, bool REQUANT = false, bool SHIFT = true, int RB = 8>
__global__ __launch_bounds__(256) void gemm_tile_x64_kernel(const GemmParams p, const RawB rawb)
{
    using Cfg = X64Cfg;
    static_assert(RB == 8 || RB == 6, "wavefront tile of 128 or 96 rows");
    constexpr int CPH = RB / 2;                          // copies of A per wavefront and half of a double stage
    constexpr int LPS = CPH + 4;                         // copies per stage and wavefront: half a double stage of A, a stage of B
    constexpr int WROWS = 16 * RB, TROWS = 2 * WROWS;    // rows of a wavefront's tile, of the workgroup's
    constexpr int NMMA = 8 * RB;                         // matrix ops per stage and wavefront
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int nslices = p.Kp / 32;
    const int nfull = p.K / 64 & ~1;                     // stages of the pipelined loop: an even number
    const int nstages = p.Kp / 64;                       // the one or two after them (full, partial) go unpipelined
    const int ntiles = p.tiles_m * p.tiles_n;
    const int gsz = gridDim.x, w = blockIdx.x;

    const int ft = lane & 15, fc = lane >> 4;            // fragments: row / column of the block, 16-byte chunk
    // A fragment of a 16-row block: lane l takes row l % 16, chunk l / 16 (+ 4 in the odd position).
    // Eight consecutive lanes then cover eight different 16-byte columns of LDS: no bank conflicts.
    const int a_off0 = (wm * WROWS + ft) * 128 + (fc ^ (ft & 7)) * 16;
    const int a_off1 = a_off0 ^ 64;
    int b_off = Cfg::kBBase + (BRAW ? (wn * 8) * 1024 + (4 * ft + ((fc + (ft >> 1)) & 3)) * 16
                                    : (wn * 8 + (fc >> 1)) * 1024 + ((fc & 1) * 16 + ft) * 16);
    // B's ring lies beyond the 64 KiB an LDS instruction's immediate offset reaches: keep its base in
    // this one register (left to itself the compiler forms a register per ring place and fragment)
    asm volatile("" : "+v"(b_off));

    // With several tiles per workgroup, the workgroups of an XCD (every eighth id) start in four
    // phases some 6000 cycles apart: in lockstep they would all write their 256 KiB of C at the same
    // moments (measured: epilogue 8.7 -> 6.7 us per tile on uniform data, 9.6 -> 5.7 us at the full
    // clock, for one start delay of at most 10 us).
    if (ntiles >= 3 * gsz)
        for (int sk = 0; sk < 3 * (int)((blockIdx.x / (unsigned)p.nxcd) & 3); ++sk) __builtin_amdgcn_s_sleep(32);

    for (int tile = w; tile < ntiles; tile += gsz) {
        int tm, tn;
        tile_of_block(tile, p.tiles_m, p.tiles_n, p.nxcd, tm, tn);
        const int m0 = tm * TROWS, n0 = tn * 256;

        // (the loaders' lane arithmetic is redone per tile: kept across the main loop it would be
        // spilled, and a reload waits for every store of the tile before still in flight)
        int lane_t = lane;
        asm volatile("" : "+v"(lane_t));
        const int r8 = lane_t >> 3;                          // A loader: row of the 8-row block
        const int a_chunk8 = (lane_t & 7) ^ r8;              //   and which of the row's eight chunks
        const int t16 = lane_t >> 2;                         // BRAW loader of B: column of the 16-column block
        const int b_chunk = ((lane_t & 3) - (t16 >> 1)) & 3;

        // Loader addresses in buffer form: the tile's first row of A / first panel (BRAW: column) of B
        // as base of a raw buffer descriptor (no bounds: every offset used below lies inside), a 32-bit
        // lane offset, and the advance along K as a scalar offset, so that a copy costs no vector
        // arithmetic (the host checks that 256 rows of A, and eight panels or 256 columns of B, span
        // less than 4 GiB).  A: copy d of half h takes rows 8 * (4 * CPH * h + CPH * wave + d) .. +7.
        const uint8_t *b_tile = BRAW ? rawb.B + (int64_t)n0 * rawb.ldb
                                     : p.Bp + (int64_t)(n0 / 32) * nslices * kFragBytes;
        // A wavefront's four copies of one operand go to four consecutive KiB of LDS: the LDS base (M0)
        // is written once for the four, and copy d carries the immediate offset 1024 * d, which the
        // instruction adds to the LDS address and to the memory address alike.  The lane offsets take
        // the latter back (+ kCopyBias - 1024 * d, never negative), the descriptors' bases start
        // kCopyBias early (an address only: nothing below the operand is touched).
        const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((uintptr_t)(p.A + (int64_t)m0 * p.lda) - Cfg::kCopyBias), (short)0, -1, 0x00020000);
        const __amdgpu_buffer_rsrc_t rsrc_b = __builtin_amdgcn_make_buffer_rsrc(
            (void *)((uintptr_t)b_tile - Cfg::kCopyBias), (short)0, -1, 0x00020000);
        uint32_t a_voff[8], b_voff[4];                   // (2 * CPH of a_voff are used; an array of dependent size here makes the host pass drop the kernel)
        const uint32_t lda32 = (uint32_t)p.lda;                // 256 rows span less than 4 GiB
        // A B fragment (32 columns x 32 bytes of K, 1 KiB) is copied with its 16-byte chunks permuted:
        // LDS slot 16 * (2 * h + khalf) + t takes column 16 * h + t, k-half khalf (packed slot
        // 32 * khalf + 16 * h + t), so that the two k-halves of a 16-column block lie side by side
        const uint32_t b_lane = (uint32_t)((32 * ((lane_t >> 4) & 1) + 16 * (lane_t >> 5) + (lane_t & 15)) * 16);
#pragma unroll
        for (int i = 0; i < 2 * CPH; ++i) {
            int grow = m0 + ((i / CPH) * (4 * CPH) + CPH * wave + (i % CPH)) * 8 + r8;
            grow = grow < p.M ? grow : p.M - 1;          // rows past M: read a valid row, never stored
            a_voff[i] = (uint32_t)(grow - m0) * lda32 + (uint32_t)a_chunk8 * 16u + (uint32_t)(Cfg::kCopyBias - 1024 * (i % CPH));
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = 4 * wave + i;                  // panel q / 2, k-half q % 2 (BRAW: 16-column block q)
            const uint32_t bias = (uint32_t)(Cfg::kCopyBias - 1024 * i);
            if (BRAW) {
                int gcol = n0 + q * 16 + t16;
                gcol = gcol < p.N ? gcol : p.N - 1;      // columns past N: read a valid one, never stored
                b_voff[i] = (uint32_t)(gcol - n0) * (uint32_t)rawb.ldb + (uint32_t)b_chunk * 16u + bias;
            } else {
                int pnl = n0 / 32 + (q >> 1);
                pnl = pnl < p.npanels ? pnl : p.npanels - 1; // panels past N: read a valid panel, never stored
                b_voff[i] = ((uint32_t)(pnl - n0 / 32) * (uint32_t)nslices + (uint32_t)(q & 1)) * (uint32_t)kFragBytes + b_lane + bias;
            }
        }
        // K offset of double stage D's copies (past the end: the last one again, a copy nobody reads)
        auto a_soff = [&](int D) { return 128 * D < 64 * nfull - 128 ? 128 * D : 64 * nfull - 128; };
        // (slot: byte offset of the ring place, here and below)
        auto dma_a = [&](auto half, int soff, int d, int slot) {     // copy d (0..CPH-1) of one half of a double stage
            constexpr int H = decltype(half)::value;
            const lptr_t to = (lptr_t)(lds + slot + (4 * CPH * H + CPH * wave) * 1024);
            switch (d) {                                 // the immediate offset has to be a literal
            case 0: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, to, 16, a_voff[CPH * H + 0], soff, 0, 0); break;
            case 1: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, to, 16, a_voff[CPH * H + 1], soff, 1024, 0); break;
            case 2: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, to, 16, a_voff[CPH * H + 2], soff, 2048, 0); break;
            default:
                if constexpr (CPH > 3)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, to, 16, a_voff[CPH * H + 3], soff, 3072, 0);
                break;
            }
        };
        auto b_soff = [&](int s) {                       // K offset of stage s's copies
            const int g = s < nfull ? s : nfull - 1;     // past the end: a copy nobody reads
            return BRAW ? g * 64 : g * (2 * kFragBytes);
        };
        auto dma_b = [&](int soff, int d, int slot) {    // copy d (0..3) of a stage
            const lptr_t to = (lptr_t)(lds + Cfg::kBBase + slot + (4 * wave) * 1024);
            switch (d) {
            case 0: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, to, 16, b_voff[0], soff, 0, 0); break;
            case 1: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, to, 16, b_voff[1], soff, 1024, 0); break;
            case 2: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, to, 16, b_voff[2], soff, 2048, 0); break;
            default: __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_b, to, 16, b_voff[3], soff, 3072, 0); break;
            }
        };

        // B fragments of a stage serve all 64 of its matrix ops: two register sets, the one of stage
        // it+1 filled while stage it runs.  An A fragment serves eight: a rolling window of four.
        // The window's places: fragment i of a stage of parity S sits in place (i + S * RB) % 4, so that the
        // fragments RB, RB + 1, ... a stage reads ahead are the next stage's 0, 1, ... (RB = 8: i % 4 throughout).
        v4i fb[2][8], fa[4];
        auto read_b = [&](auto set, const uint8_t *from, int j) {     // from: lds + place + b_off
            constexpr int S = decltype(set)::value;
            fb[S][j] = *(const v4i *)(from + (BRAW ? j * 1024 : (j >> 1) * 2048 + (j & 1) * 512));
        };
        auto read_a = [&](auto set, const uint8_t *from, int i, int frag) {   // from: lds + place + a_off0 or a_off1; block i into the place of fragment `frag`
            constexpr int S = decltype(set)::value;
            fa[(frag + S * RB) & 3] = *(const v4i *)(from + i * 2048);
        };

        v4i acc[RB][8];                                  // started by the first stage (K >= kMinK: there is one)
        // matrix op m of a stage: row block m / 8, column block m % 8
        auto mma = [&](auto set, int m) {
            constexpr int S = decltype(set)::value;
            const int i = m >> 3, j = m & 7;
            acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fb[S][j], fa[(i + S * RB) & 3], acc[i][j], 0, 0, 0);
        };
        auto mma_first = [&](auto set, int m) {          // the first stage starts the sums
            constexpr int S = decltype(set)::value;
            const int i = m >> 3, j = m & 7;
            acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fb[S][j], fa[(i + S * RB) & 3], v4i{0, 0, 0, 0}, 0, 0, 0);
        };
        auto shift_a = [&](auto set, int frag) {         // u8 -> s8
            constexpr int S = decltype(set)::value;
            if (SHIFT) fa[(frag + S * RB) & 3] = shift_u8_to_s8(fa[(frag + S * RB) & 3], p.a_xor);
        };
        auto shift_a_word = [&](auto set, int frag, int wd) {          // one dword of it
            constexpr int S = decltype(set)::value;
            if (SHIFT) fa[(frag + S * RB) & 3][wd] ^= (int)p.a_xor;
        };

        if (tile != w) __syncthreads();                  // the previous tile's LDS traffic is over

        {
            // in flight ahead of the loop: A's double stages 0 and 1 (stages 0..3), B's stages 0..2
            {
                const int s0 = a_soff(0), s1 = a_soff(1);
#pragma unroll
                for (int d = 0; d < CPH; ++d) dma_a(IntC<0>{}, s0, d, 0);
#pragma unroll
                for (int d = 0; d < CPH; ++d) dma_a(IntC<1>{}, s0, d, 0);
#pragma unroll
                for (int d = 0; d < 4; ++d) dma_b(b_soff(0), d, 0);
#pragma unroll
                for (int d = 0; d < 4; ++d) dma_b(b_soff(1), d, Cfg::kBBytes);
#pragma unroll
                for (int d = 0; d < CPH; ++d) dma_a(IntC<0>{}, s1, d, Cfg::kADouble);
#pragma unroll
                for (int d = 0; d < CPH; ++d) dma_a(IntC<1>{}, s1, d, Cfg::kADouble);
#pragma unroll
                for (int d = 0; d < 4; ++d) dma_b(b_soff(2), d, 2 * Cfg::kBBytes);
            }
            wait_vmcnt<8 + 2 * CPH>();                   // A's stages 0, 1 and B's stage 0 have landed (this wavefront's part)
            __builtin_amdgcn_s_barrier();
#pragma unroll
            for (int j = 0; j < 8; ++j) read_b(IntC<0>{}, lds + b_off, j);
            read_a(IntC<0>{}, lds + a_off0, 0, 0);
            read_a(IntC<0>{}, lds + a_off0, 1, 1);
            read_a(IntC<0>{}, lds + a_off0, 2, 2);
            shift_a(IntC<0>{}, 0);
            __builtin_amdgcn_sched_barrier(0);

            // One stage: 64 matrix ops, row block by row block (eight ops each, gaps j = 0..7).  One
            // wavefront per SIMD issues in order, about one instruction every four cycles, and a matrix
            // op takes sixteen: a gap has room for three other instructions, a fourth delays the next
            // matrix op.  So everything sits in a gap of its own choosing:
            //   j = 4..7 of row i: the u8 -> s8 shift of A fragment i+1, one dword per gap;
            //   j = 5 of row i: the read of A fragment i+3 (rows 5..7: fragments 0..2 of stage it+1),
            //     two rows ahead of its shift;
            //   j = 6, 7 of rows 2..5: the B fragments of stage it+1 into the other register set;
            //   j = 1 of rows 2..7 and j = 3 of rows 3, 5: one copy each (M0, the wait state it needs,
            //     the copy) -- four of A (one half of the double stage two ahead of this stage's: the
            //     even stage issues rows 0..127, the odd one the rest), then four of B's stage it+3.
            //     Eight copies in a row from each of the four wavefronts fill the compute unit's memory
            //     pipe and hold the wavefronts up at issue: spread out they cost 4 % less time;
            //   j = 0..3 of rows 0, 1: the scalar bookkeeping (ring places as byte offsets, carried from
            //     stage to stage; K offsets of the copies) and the three LDS addresses it feeds.
            // Before row 2: wait until at most this wavefront's eight copies of the stage before are
            // outstanding, barrier (=> everything stage it+1 reads is complete for everybody, and
            // everybody's reads of stage it-1 were consumed a stage ago, so its places are free: A's
            // double stage before this one's, B's stage it, read into registers during stage it-1).
            int ra = 0, rb = 0;                          // A: place of stage it's double stage; B: of stage it
            auto body = [&](auto set, auto other, auto first, int it) {
                constexpr int S = decltype(set)::value;              // == it & 1
                constexpr bool FIRST = decltype(first)::value != 0;
                constexpr int kA = Cfg::kADouble, kB = Cfg::kBBytes;
                int as_n = 0, as_f = 0, bs_n = 0, soff_a = 0, soff_b = 0;
                const uint8_t *pa_c = nullptr, *pa_n = nullptr, *pb_n = nullptr;
#pragma unroll
                for (int m = 0; m < NMMA; ++m) {
                    const int i = m >> 3, j = m & 7;
                    if (m == 0) as_n = !S ? ra : (ra == 2 * kA ? 0 : ra + kA);    // double stage of stage it+1
                    if (m == 1) pa_c = lds + ra + (S ? a_off1 : a_off0);
                    if (m == 2) as_f = ra == 0 ? 2 * kA : ra - kA;               // two double stages ahead
                    if (m == 3) pa_n = lds + as_n + (S ? a_off0 : a_off1);
                    if (m == 8) bs_n = rb == 2 * kB ? 0 : rb + kB;
                    if (m == 9) soff_a = a_soff((it >> 1) + 2);
                    if (m == 10) soff_b = b_soff(it + 3);
                    if (m == 11) pb_n = lds + bs_n + b_off;
                    if (m == 16) {
                        wait_vmcnt<LPS>();
                        __builtin_amdgcn_s_barrier();
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (j >= 4) shift_a_word(set, i + 1, j - 4);
                    if (j == 5) {
                        if (i < RB - 3) read_a(set, pa_c, i + 3, i + 3);
                        else read_a(set, pa_n, i - (RB - 3), i + 3);
                    }
                    if (j >= 6 && i >= 2 && i < 6) read_b(other, pb_n, 2 * (i - 2) + (j - 6));
                    if (RB == 8) {
                        if (i >= 2 && (j == 1 || (j == 3 && (i == 3 || i == 5)))) {
                            // copies 0..7 in the gaps m = 17, 25, 27, 33, 41, 43, 49, 57
                            const int d = i == 2 ? 0 : i == 3 ? (j == 1 ? 1 : 2) : i == 4 ? 3 : i == 5 ? (j == 1 ? 4 : 5) : i;
                            if (d < 4) dma_a(set, soff_a, d, as_f);
                            else dma_b(soff_b, d - 4, rb);
                        }
                    } else {
                        if (i >= 2 && (j == 1 || (j == 3 && i < 5))) {
                            // copies 0..6 in the gaps m = 17, 19, 25, 27, 33, 35, 41
                            const int d = 2 * (i - 2) + (j == 3);
                            if (d < CPH) dma_a(set, soff_a, d, as_f);
                            else dma_b(soff_b, d - CPH, rb);
                        }
                    }
                    if (m == NMMA - 6) {                 // step the rings
                        rb = bs_n;
                        ra = as_n;
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (FIRST) mma_first(set, m);
                    else mma(set, m);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            // the first stage starts the sums (no zeroed accumulators ahead of the loop)
            body(IntC<0>{}, IntC<1>{}, IntC<1>{}, 0);
            body(IntC<1>{}, IntC<0>{}, IntC<0>{}, 1);
            for (int it = 2; it < nfull; it += 2) {
                body(IntC<0>{}, IntC<1>{}, IntC<0>{}, it);
                body(IntC<1>{}, IntC<0>{}, IntC<0>{}, it + 1);
            }
            wait_vmcnt<0>();                             // drain the copies nobody reads
        }

        // What the rest of the tile derives from the lane index is computed from here on (the compiler
        // would otherwise prepare the addresses of the K tail and of the epilogue ahead of the main
        // loop, carry them across it in registers the loop needs, and spill them; a reload then waits
        // for every copy or store in flight).
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));

        // What is left of K: an odd last full stage and / or a partial one.  Guarded register loads
        // into the first places of the rings (A: even position), same layouts, no pipelining.
        for (int ts = nfull; ts < nstages; ++ts) {
            const int kbase = ts * 64;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < CPH; ++i) {
                const int R = 16 * (CPH * wave + i) + (lane_e >> 2), c = lane_e & 3;   // 16-row blocks of A
                const int grow = m0 + R < p.M ? m0 + R : p.M - 1;
                const int valid = p.K - (kbase + c * 16);
                const uint8_t *src = p.A + (int64_t)grow * p.lda + kbase + c * 16;
                v4i v = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
                *(v4i *)(lds + R * 128 + (c ^ (R & 7)) * 16) = v;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int q = 4 * wave + i;                // B's blocks as the copies divide them (b_voff[i])
                v4i z = {0, 0, 0, 0};
                if (BRAW) {
                    const int bvalid = p.K - (kbase + (((lane_e & 3) - (lane_e >> 3)) & 3) * 16);
                    const uint8_t *bs = b_tile + (b_voff[i] - (uint32_t)(Cfg::kCopyBias - 1024 * i)) + kbase;
                    z = bvalid >= 16 ? load16_any(bs) : load16_partial(bs, bvalid < 0 ? 0 : bvalid);
                } else if (ts * 2 + (q & 1) < nslices) {
                    z = *(const v4i *)(b_tile + (b_voff[i] - (uint32_t)(Cfg::kCopyBias - 1024 * i)) + (int64_t)ts * (2 * kFragBytes));
                }
                *(v4i *)(lds + Cfg::kBBase + q * 1024 + lane_e * 16) = z;
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) read_b(IntC<0>{}, lds + b_off, j);
#pragma unroll
            for (int m = 0; m < NMMA; ++m) {
                if ((m & 7) == 0) {
                    read_a(IntC<0>{}, lds + a_off0, m >> 3, m >> 3);
                    shift_a(IntC<0>{}, m >> 3);
                }
                mma(IntC<0>{}, m);
            }
        }

        __syncthreads();                                 // every wavefront is done with the stage buffers

        const int ft = lane_e & 15, fc = lane_e >> 4;
        uint8_t *patch = lds + wave * Cfg::kPatchBytes;
        if (REQUANT) {
            // Requantising epilogue (per tensor or per column).  The three per-column arrays of the tile
            // -- (128-za)*colsum + bias, zero-point of B, scale -- are staged in LDS behind the patches.
            // A lane requantises its four consecutive columns of each block to four bytes, the 16 x 128
            // byte block goes through the wavefront's patch and is stored as full 128-byte row pieces.
            uint32_t *cterm = (uint32_t *)(lds + 4 * Cfg::kPatchBytes);
            for (int c = tid; c < 256; c += 256) {
                const int col = n0 + c;
                const bool ok = col < p.N;
                uint32_t cb = ok ? p.za_term * (uint32_t)p.colsum[col] : 0u;
                if (ok && p.bias_vec) cb += (uint32_t)p.bias_vec[col];
                cterm[c] = cb;
                cterm[256 + c] = (ok && p.zb_vec) ? (uint32_t)p.zb_vec[col] : p.zb;
                ((float *)cterm)[512 + c] = (ok && p.scale_vec) ? p.scale_vec[col] : p.scale;
            }
            __syncthreads();
            constexpr int kRow8 = 128 + 16;              // byte patch: 16 rows of 128 bytes, padded
            const int cg8 = lane_e & 7, r8 = lane_e >> 3;    // read-back: 8 lanes of 16 bytes per row, 8 rows per pass
            const int bcol8 = n0 + wn * 128 + 16 * cg8;
            const bool interior = m0 + (wm + 1) * WROWS <= p.M && n0 + (wn + 1) * 128 <= p.N &&
                                  ((((uintptr_t)p.C | (uintptr_t)p.ldc) & 15) == 0);
            const bool small_zc = p.zc > -8388608 && p.zc < 8388608;   // uniform: picks the binary32 form
            const float zcf = (float)p.zc;
            auto requant_rows = [&](auto small) __attribute__((always_inline)) {
            constexpr bool SMALL = decltype(small)::value != 0;
            auto rq = [&](uint32_t v, float sc) -> uint32_t { return requant_u8((int32_t)v, sc, p.zc, p.relu); };
            const float floor_f = p.relu ? zcf : -3.402823466e38f;
            // sum_k (A[i][k] - za) of this lane's row in each of the eight blocks, multiplied per column
            // by that column's zero-point of B (all loaded first: a load between the blocks would wait
            // for the stores of the block before it)
            uint32_t rsums[RB];
#pragma unroll
            for (int i = 0; i < RB; ++i) rsums[i] = p.rconst;
            if (p.rowsum) {                              // rows past M read row M - 1 and are never stored
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int row = m0 + wm * WROWS + 16 * i + ft;
                    rsums[i] += (uint32_t)p.rowsum[row < p.M ? row : p.M - 1];
                }
            }
            // this lane's columns are the same in every block: their three terms are read once
            uint4 cbs[8], zvs[8];
            float4 scs[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int lcol = wn * 128 + 16 * j + 4 * fc;
                cbs[j] = *(const uint4 *)(cterm + lcol);
                zvs[j] = *(const uint4 *)(cterm + 256 + lcol);
                scs[j] = *(const float4 *)((const float *)cterm + 512 + lcol);
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int brow0 = m0 + wm * WROWS + 16 * i;
                const uint32_t rsum = rsums[i];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint4 cb = cbs[j], zv = zvs[j];
                    const float4 sc = scs[j];
                    const v4i v = acc[i][j];
                    const int32_t c4[4] = {(int32_t)((uint32_t)v.x + cb.x - zv.x * rsum), (int32_t)((uint32_t)v.y + cb.y - zv.y * rsum),
                                           (int32_t)((uint32_t)v.z + cb.z - zv.z * rsum), (int32_t)((uint32_t)v.w + cb.w - zv.w * rsum)};
                    uint32_t bw;
                    if (SMALL) bw = requant4_u8_small_zc(c4, sc, zcf, floor_f);
                    else bw = rq((uint32_t)c4[0], sc.x) | (rq((uint32_t)c4[1], sc.y) << 8) | (rq((uint32_t)c4[2], sc.z) << 16) | (rq((uint32_t)c4[3], sc.w) << 24);
                    *(uint32_t *)(patch + ft * kRow8 + 16 * j + 4 * fc) = bw;
                }
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const v4i o = *(const v4i *)(patch + (8 * q + r8) * kRow8 + cg8 * 16);
                    const int orow = brow0 + 8 * q + r8;
                    uint8_t *dst = (uint8_t *)p.C + (int64_t)orow * p.ldc + bcol8;
                    if (interior) {
                        __builtin_nontemporal_store(o, (v4i *)dst);   // streaming, as the int32 form's
                    } else if (orow < p.M) {
                        const uint8_t *ob = (const uint8_t *)&o;
#pragma unroll
                        for (int t = 0; t < 16; ++t)
                            if (bcol8 + t < p.N) dst[t] = ob[t];
                    }
                }
            }
            };
            if (small_zc) requant_rows(IntC<1>{});
            else requant_rows(IntC<0>{});
        } else {
        // Epilogue.  Per 16-row block: row terms added, the 16 x 128 block written to an LDS patch as
        // it lies in the accumulators, read back two rows per instruction, column terms added, stored
        // as full 512-byte row pieces.
        const int cg = lane_e & 31, r2 = lane_e >> 5;
        const int bcol = n0 + wn * 128 + 4 * cg;
        uint4 ct = {0u, 0u, 0u, 0u};
        if (bcol < p.N) {
            const int4 cs = *(const int4 *)(p.colsum + bcol);        // colsum is padded to 32 columns
            ct.x = p.za_term * (uint32_t)cs.x; ct.y = p.za_term * (uint32_t)cs.y;
            ct.z = p.za_term * (uint32_t)cs.z; ct.w = p.za_term * (uint32_t)cs.w;
        }
        const bool interior = m0 + (wm + 1) * WROWS <= p.M && n0 + (wn + 1) * 128 <= p.N;
        // the row terms of all eight blocks first, as eight independent loads (rows past M read row
        // M - 1 and are never stored): loaded block by block, each load would wait for its own
        // latency and for the stores of the block before it
        uint32_t row_terms[RB];
#pragma unroll
        for (int i = 0; i < RB; ++i) row_terms[i] = p.kconst;
        if (p.rowsum) {
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int row = m0 + wm * WROWS + 16 * i + ft;
                row_terms[i] -= p.zb * (uint32_t)p.rowsum[row < p.M ? row : p.M - 1];
            }
        }
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            const int brow0 = m0 + wm * WROWS + 16 * i;
            const uint32_t row_term = row_terms[i];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                v4i v = acc[i][j];
                v.x = (int)((uint32_t)v.x + row_term); v.y = (int)((uint32_t)v.y + row_term);
                v.z = (int)((uint32_t)v.z + row_term); v.w = (int)((uint32_t)v.w + row_term);
                *(v4i *)(patch + ft * Cfg::kPatchRow + (16 * j + 4 * fc) * 4) = v;
            }
            v4i o[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) o[q] = *(const v4i *)(patch + (2 * q + r2) * Cfg::kPatchRow + cg * 16);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                o[q].x = (int)((uint32_t)o[q].x + ct.x); o[q].y = (int)((uint32_t)o[q].y + ct.y);
                o[q].z = (int)((uint32_t)o[q].z + ct.z); o[q].w = (int)((uint32_t)o[q].w + ct.w);
            }
            int32_t *dst = (int32_t *)p.C + (int64_t)(brow0 + r2) * p.ldc + bcol;   // this lane's first row of the block
            if (interior) {                              // one branch per block, no per-lane tests
#pragma unroll
                for (int q = 0; q < 8; ++q, dst += 2 * p.ldc) {
                    // streaming store (4-byte aligned is enough): C is not read again, and kept out of
                    // L2 it leaves the A and B panels there (6 % fewer main-loop cycles at the full clock)
                    __builtin_nontemporal_store(o[q], (v4i_a4 *)dst);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q, dst += 2 * p.ldc) {
                    const v4i v = o[q];
                    if (brow0 + 2 * q + r2 < p.M && bcol < p.N) {
                        if (bcol + 3 < p.N) {
                            __builtin_memcpy(dst, &v, 16);
                        } else {
                            dst[0] = v.x;
                            if (bcol + 1 < p.N) dst[1] = v.y;
                            if (bcol + 2 < p.N) dst[2] = v.z;
                        }
                    }
                }
            }
        }
        }
    }
}

// ---- small tiles with a long pipeline ---------------------------------------------------------
// For outputs with at most one 64 x 64 (T = 1) or 128 x 128 (T = 2) tile per compute unit.  There
// a workgroup is alone on its compute unit, one wavefront per SIMD, and the kernel above spends
// its time waiting for LDS: with T = 1 a wavefront has two matrix ops per 64 bytes of K and one
// barrier, with fragment reads issued one matrix op ahead.  Here a stage is SUB sub-blocks of
// 64 bytes of K in the layout above (32 KiB per stage), so one barrier pays for 2 * SUB * T * T
// matrix ops per wavefront, and all fragments of stage it+1 are read into a second register set
// while the matrix ops of stage it run: the LDS latency has half a stage to pass.  Ring of NSTAGE
// stage buffers, copies memory -> LDS as above; the sub-blocks of the last, partial stage and
// the K tail are consumed without pipelining.
template <int T, int SUB, int NSTAGE>
struct DeepCfg {
    static constexpr int BMN = 64 * T;                     // tile edge
    static constexpr int kABytes = BMN * 64;               // A part of a sub-block
    static constexpr int kSubBytes = 2 * kABytes;          // A BMN x 64 + B BMN x 64
    static constexpr int kStageBytes = SUB * kSubBytes;
    static constexpr int kLoadsPerStage = 2 * T * SUB;     // per lane: T blocks of A, T of B per sub-block
    static constexpr int kEpiBytes = 4 * kXposeBytes<T> + BMN * 12;
    static constexpr int kLdsBytes = NSTAGE * kStageBytes > kEpiBytes ? NSTAGE * kStageBytes : kEpiBytes;
    static_assert(T == 1 || T == 2, "wavefront tile of 32 x 32 or 64 x 64");
    static_assert(NSTAGE >= 3 && NSTAGE * kStageBytes <= 160 * 1024, "ring depth");
    static_assert((NSTAGE - 2) * kLoadsPerStage <= 63, "vmcnt range");
};

// ROWS: form the row sums a zero-point of B needs here (four more vector instructions per A fragment:
// 8 % to 28 % on the T = 1 form, whose wavefronts are bound by instruction issue, so the host picks
// this form only when the zero-point is there; it then saves the launch of the row-sum pass).
// SPLITK: 0 one workgroup per tile; 1 K split, the parts add their partial tiles to a cleared C with
// atomic adds; 2 K split, the parts store their partial tiles (row terms taken off already) to
// p.part_ws and splitk_reduce_kernel forms the output (any output type).
template <int T, int SUB, int NSTAGE, bool REQUANT, int SPLITK = 0, bool ROWS = false>
__global__ __launch_bounds__(256) void gemm_tile_deep_kernel(const GemmParams p)
{
    using Cfg = DeepCfg<T, SUB, NSTAGE>;
    constexpr int BMN = Cfg::BMN, LPS = Cfg::kLoadsPerStage;
    constexpr int NF = 2 * SUB;                          // 32-byte steps of K per stage
    constexpr int NM = T * T;                            // matrix ops per such step
    constexpr int G = (NF / 2) * NM;                     // matrix ops (= gaps) in the second half of a stage
    constexpr int NREADS = NF * 2 * T;                   // fragment reads per stage
    constexpr int RPG = (NREADS + G / 2 - 1) / (G / 2);  // reads per gap: all in the first half of the gaps
    constexpr int DPG = (LPS + G - 1) / G;               // copies per gap
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    static_assert(!(SPLITK != 0 && REQUANT), "partial sums are int32");
    const int nslices = p.Kp / 32;
    const int ntiles = p.tiles_m * p.tiles_n;
    const int nunits = (SPLITK != 0) ? ntiles * p.ksplit : ntiles;
    const int gsz = gridDim.x, w = blockIdx.x;

    const int t16 = lane >> 2;
    const int a_chunk = ((lane & 3) - (t16 >> 2)) & 3;
    int a_frag_off[2];
    {
        const int r = lane & 31, t = r & 15;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int c = 2 * ks + (lane >> 5);
            a_frag_off[ks] = (wm * T * 2 + (r >> 4)) * 1024 + (4 * t + ((c + (t >> 2)) & 3)) * 16;
        }
    }
    const int b_frag_off = Cfg::kABytes + (wn * T * 2) * kFragBytes + lane * 16;

    for (int unit = w; unit < nunits; unit += gsz) {
        // this unit's tile and part of K: bytes [k0, k0 + kc), k0 a multiple of 256
        const int split = (SPLITK != 0) ? unit / ntiles : 0;
        const int tile = (SPLITK != 0) ? unit - split * ntiles : unit;
        const int k0 = (SPLITK != 0) ? split * p.kchunk : 0;
        const int kc = (SPLITK != 0) ? (p.K - k0 < p.kchunk ? p.K - k0 : p.kchunk) : p.K;
        const int nsub = kc / 64;                         // full 64-byte sub-blocks of K
        const int nst = nsub / SUB, rem = nsub % SUB;     // full stages, sub-blocks of the partial one
        const int nstages = nst + (rem > 0 ? 1 : 0);
        const bool has_tail = nsub * 64 < kc;
        int tm, tn;
        tile_of_block(tile, p.tiles_m, p.tiles_n, p.nxcd, tm, tn);
        const int m0 = tm * BMN, n0 = tn * BMN;
        static_assert(BMN <= 256, "a thread per column of the tile");
        const EpiCols ec = epi_load_cols<T, BMN, REQUANT>(p, n0, wn, lane, tid);   // the epilogue's column terms, early

        // Loader: wavefront v copies, for every sub-block, the 16-row blocks v, v+4, ... of the A
        // tile and the fragments v, v+4, ... (panel q/2, k-half q%2) of the B tile.
        const uint8_t *a_src[T], *b_src[T];
#pragma unroll
        for (int i = 0; i < T; ++i) {
            int grow = m0 + (wave + 4 * i) * 16 + t16;
            grow = grow < p.M ? grow : p.M - 1;          // rows past M: read a valid row, never stored
            a_src[i] = p.A + (int64_t)grow * p.lda + a_chunk * 16 + k0;
            const int q = wave + 4 * i;
            int pnl = n0 / 32 + (q >> 1);
            pnl = pnl < p.npanels ? pnl : p.npanels - 1; // panels past N: read a valid panel, never stored
            b_src[i] = p.Bp + ((int64_t)pnl * nslices + k0 / 32 + (q & 1)) * kFragBytes + lane * 16;
        }
        // copy number d of stage s into ring buffer buf: sub-block d / 2T, then T blocks of A, T of B
        auto dma_one = [&](int s, int d, int buf) {
            const int q = d / (2 * T), e = d % (2 * T);
            int g = s * SUB + q;
            g = g < nsub ? g : nsub - 1;                 // past the end: a copy nobody reads
            uint8_t *dst = lds + buf * Cfg::kStageBytes + q * Cfg::kSubBytes;
            if (e < T)
                __builtin_amdgcn_global_load_lds((gptr_t)(a_src[e] + (int64_t)g * 64),
                                                 (lptr_t)(dst + (wave + 4 * e) * 1024), 16, 0, 0);
            else
                __builtin_amdgcn_global_load_lds((gptr_t)(b_src[e - T] + (int64_t)g * (2 * kFragBytes)),
                                                 (lptr_t)(dst + Cfg::kABytes + (wave + 4 * (e - T)) * 1024), 16, 0, 0);
        };
        auto clamps = [&](int s) { return s < nstages ? s : nstages - 1; };

        v4i fa[2][NF][T], fb[2][NF][T];                  // [register set][32-byte step of the stage][block]
        // fragment read number r of a stage: step r / 2T, then T fragments of A, T of B
        auto read_one = [&](auto set, int buf, int r) {
            constexpr int S = decltype(set)::value;
            const int idx = r / (2 * T), e = r % (2 * T);
            const uint8_t *base = lds + buf * Cfg::kStageBytes + (idx >> 1) * Cfg::kSubBytes;
            if (e < T)
                fa[S][idx][e] = *(const v4i *)(base + a_frag_off[idx & 1] + e * 2048);
            else
                fb[S][idx][e - T] = *(const v4i *)(base + b_frag_off + ((e - T) * 2 + (idx & 1)) * kFragBytes);
        };

        v16i acc[T][T];
#pragma unroll
        for (int i = 0; i < T; ++i)
#pragma unroll
            for (int j = 0; j < T; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
        // matrix op m of step idx; packed operand first, as in the kernels above (the epilogue
        // expects that register layout).  The u8 -> s8 shift of an A fragment precedes its first use.
        int rs[T];                                      // this lane's share of the row sums (row lane % 32 of block i)
#pragma unroll
        for (int i = 0; i < T; ++i) rs[i] = 0;
        auto mma = [&](auto set, int idx, int m) {
            constexpr int S = decltype(set)::value;
            const int i = m / T, j = m % T;
            if (j == 0) fa[S][idx][i] = shift_u8_to_s8(fa[S][idx][i], p.a_xor);
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[S][idx][j], fa[S][idx][i], acc[i][j], 0, 0, 0);
            if (ROWS && j == 0) {
                // the row sums a zero-point of B needs, from the fragments as they pass; issued behind
                // the matrix op, whose passes they overlap
                __builtin_amdgcn_sched_barrier(0);
                const v4i a = fa[S][idx][i];
                rs[i] = __builtin_amdgcn_sdot4(a.x, 0x01010101, rs[i], false);
                rs[i] = __builtin_amdgcn_sdot4(a.y, 0x01010101, rs[i], false);
                rs[i] = __builtin_amdgcn_sdot4(a.z, 0x01010101, rs[i], false);
                rs[i] = __builtin_amdgcn_sdot4(a.w, 0x01010101, rs[i], false);
            }
        };

        if (unit != w) __syncthreads();                  // the previous tile's LDS traffic is over

        if (nsub > 0) {
#pragma unroll
            for (int s = 0; s < NSTAGE - 1; ++s)
#pragma unroll
                for (int d = 0; d < LPS; ++d) dma_one(clamps(s), d, s);
            wait_vmcnt<(NSTAGE - 2) * LPS>();            // stage 0 has landed (this wavefront's part)
            __builtin_amdgcn_s_barrier();                // ... and everybody else's
#pragma unroll
            for (int r = 0; r < NREADS; ++r) read_one(IntC<0>{}, 0, r);
            __builtin_amdgcn_sched_barrier(0);

            // One full stage: register set S holds its fragments, the other set receives those of
            // stage it+1.  First half: half of the matrix ops, then the wait for this wavefront's
            // copies of stage it+1 and the barrier (=> stage it+1 is complete for everybody, and
            // everybody's reads of stage it-1 were consumed long ago, so its buffer is free).
            // Second half: reads of stage it+1 (all in the early gaps: they have the longest way)
            // and copies of stage it+NSTAGE-1 in the gaps between the other matrix ops.
            auto body = [&](auto set, auto other, int it) {
                const int buf_n = (it + 1) % NSTAGE, buf_f = (it + NSTAGE - 1) % NSTAGE;
                const int sload = clamps(it + NSTAGE - 1);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    mma(set, g / NM, g % NM);
                    __builtin_amdgcn_sched_barrier(0);
                }
                wait_vmcnt<(NSTAGE - 3) * LPS>();
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int g = 0; g < G; ++g) {
#pragma unroll
                    for (int r = g * RPG; r < (g + 1) * RPG; ++r)
                        if (r < NREADS) read_one(other, buf_n, r);
#pragma unroll
                    for (int d = g * DPG; d < (g + 1) * DPG; ++d)
                        if (d < LPS) dma_one(sload, d, buf_f);
                    __builtin_amdgcn_sched_barrier(0);
                    mma(set, NF / 2 + g / NM, g % NM);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            // The partial stage (rem sub-blocks), whose fragments the last full stage has read.
            auto finish = [&](auto set) {
#pragma unroll
                for (int q = 0; q < SUB - 1; ++q)
                    if (q < rem) {
#pragma unroll
                        for (int m = 0; m < 2 * NM; ++m) mma(set, 2 * q + m / NM, m % NM);
                    }
            };
            int it = 0;
            for (; it + 1 < nst; it += 2) {
                body(IntC<0>{}, IntC<1>{}, it);
                body(IntC<1>{}, IntC<0>{}, it + 1);
            }
            if (it < nst) {
                body(IntC<0>{}, IntC<1>{}, it);
                finish(IntC<1>{});
            } else {
                finish(IntC<0>{});
            }
            wait_vmcnt<0>();                             // drain the copies nobody reads
        }

        // K tail: the last, partial 64 bytes.  Guarded register loads into sub-block 0 of buffer 0.
        if (has_tail) {
            const int kbase = nsub * 64;
            __syncthreads();
#pragma unroll
            for (int i = 0; i < T; ++i) {
                const int q = wave + 4 * i;
                const int valid = kc - (kbase + a_chunk * 16);
                const uint8_t *src = a_src[i] + kbase;
                v4i v = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
                *(v4i *)(lds + q * 1024 + lane * 16) = v;
                v4i z = {0, 0, 0, 0};
                if (k0 / 32 + nsub * 2 + (q & 1) < nslices) z = *(const v4i *)(b_src[i] + (int64_t)nsub * (2 * kFragBytes));
                *(v4i *)(lds + Cfg::kABytes + q * 1024 + lane * 16) = z;
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 2 * 2 * T; ++r) read_one(IntC<0>{}, 0, r);
#pragma unroll
            for (int m = 0; m < 2 * NM; ++m) mma(IntC<0>{}, m / NM, m % NM);
        }

        __syncthreads();                                 // every wavefront is done with the stage buffers
        // Row sums over this unit's part of K: the two halves of each 32-byte step sit in lanes l and
        // l ^ 32; the zero fill of the K tail was shifted with the rest and counts as -128 per byte
        // for an unsigned A, which is taken out again.
        uint32_t rs_reg[T];
        {
            const uint32_t pad = (p.a_xor && has_tail) ? 128u * (uint32_t)((nsub + 1) * 64 - kc) : 0u;
#pragma unroll
            for (int i = 0; i < T; ++i) rs_reg[i] = (uint32_t)(rs[i] + __shfl_xor(rs[i], 32, 64)) + pad;
        }
        if (SPLITK == 2) {
            // partial tile of this part, dense, with this part's share of the row term; the column
            // and constant terms are added when the parts are summed
            GemmParams pe = p;
            pe.za_term = 0u;
            pe.kconst = 0u;
            pe.ldc = (p.N + 3) & ~3;                     // row pitch of the partial matrices
            pe.C = p.part_ws + (int64_t)split * p.M * pe.ldc;
            tile_epilogue<T, T, BMN, false, false, false>(pe, acc, m0, n0, wm, wn, lane, tid, 256, lds + wave * kXposeBytes<T>,
                                                          (uint32_t *)(lds + 4 * kXposeBytes<T>), ec, ROWS ? rs_reg : nullptr);
        } else if (SPLITK == 1) {
            // the column and constant terms belong to the whole sum: the first part of K brings
            // them; the row term is linear in the row sum, so every part takes its own share
            GemmParams pe = p;
            if (split > 0) {
                pe.za_term = 0u;
                pe.kconst = 0u;
            }
            tile_epilogue<T, T, BMN, false, false, true>(pe, acc, m0, n0, wm, wn, lane, tid, 256, lds + wave * kXposeBytes<T>,
                                                         (uint32_t *)(lds + 4 * kXposeBytes<T>), ec, ROWS ? rs_reg : nullptr);
        } else
        // every practical output zero-point takes the binary32 form of the requantising arithmetic
        if (REQUANT && p.zc > -8388608 && p.zc < 8388608)
            tile_epilogue<T, T, BMN, REQUANT, true>(p, acc, m0, n0, wm, wn, lane, tid, 256, lds + wave * kXposeBytes<T>,
                                          (uint32_t *)(lds + 4 * kXposeBytes<T>), ec, ROWS ? rs_reg : nullptr);
        else
            tile_epilogue<T, T, BMN, REQUANT, false>(p, acc, m0, n0, wm, wn, lane, tid, 256, lds + wave * kXposeBytes<T>,
                                          (uint32_t *)(lds + 4 * kXposeBytes<T>), ec, ROWS ? rs_reg : nullptr);
    }
}

// Sum of the K split's partial results (SPLITK = 2) and the rest of the epilogue: column term,
// constant term, and for u8 outputs the requantising sequence.  The partial matrices are dense with
// a row pitch of N rounded up to 4 (16-byte loads).  A workgroup of up to 16 wavefronts (as many as
// there are parts) covers 64 groups of four columns: wavefront w sums the parts w, w + nw, ... (all
// its loads in flight at once), the shares meet in LDS and wavefront 0 finishes and stores.
constexpr int kReduceWaves = 16;
__host__ __device__ inline int64_t splitk_part_pitch(int64_t N) { return (N + 3) & ~(int64_t)3; }

template <bool REQUANT>
__global__ __launch_bounds__(64 * kReduceWaves) void splitk_reduce_kernel(const GemmParams p, int parts)
{
    __shared__ uint4 red[kReduceWaves][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int64_t ldp = splitk_part_pitch(p.N), quads = ldp / 4;
    const int64_t u = (int64_t)blockIdx.x * 64 + lane;
    const bool ok = u < (int64_t)p.M * quads;
    const int row = ok ? (int)(u / quads) : 0, col = ok ? (int)(u - (int64_t)row * quads) * 4 : 0;
    const int64_t mn = (int64_t)p.M * ldp;
    uint4 v = {0u, 0u, 0u, 0u};
    if (ok) {
        const int32_t *src = p.part_ws + (int64_t)row * ldp + col + (int64_t)wave * mn;
#pragma unroll 4
        for (int sp = wave; sp < parts; sp += nw) {
            const uint4 t = *(const uint4 *)src;        // columns past N: never written, never used
            v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
            src += (int64_t)nw * mn;
        }
    }
    red[wave][lane] = v;
    __syncthreads();
    if (wave != 0 || !ok) return;
    for (int w = 1; w < nw; ++w) {
        const uint4 t = red[w][lane];
        v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
    }
    // the parts took the row term off already: what is left has no row-dependent part
    GemmParams pe = p;
    pe.rowsum = nullptr;
    pe.zb = 0u;
    pe.zb_vec = nullptr;
    if (REQUANT) pe.rconst = 0u;
    const uint32_t vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int t = 0; t < 4; ++t)
        if (col + t < p.N) {
            const uint32_t cs_term = p.za_term * (uint32_t)p.colsum[col + t];
            // finish_s32 adds kconst itself; the requantising form has it inside the row term
            store_out<REQUANT>(pe, row, col + t, (int32_t)(REQUANT ? vv[t] + p.kconst : vv[t]), cs_term);
        }
}

// ---- 16-bit operands: s16 x s16 -> s32 on the 8-bit matrix pipe -------------------------------
// There is no 16-bit integer matrix instruction; a 16-bit value is split into its bytes,
//     a - 128 = 256 * ah + al',   ah = a >> 8 (signed),   al' = (a & 255) - 128 = (a & 255) xor 0x80,
// and likewise for b, so that
//     sum (a-128)(b-128) = 65536 * sum ah*bh + 256 * (sum ah*bl' + sum al'*bh) + sum al'*bl'   (mod 2^32)
// is four 8-bit matrix ops per block of the output, one per product of byte planes, summed with the
// shifts in the epilogue; every step is exact in the ring of integers mod 2^32.  The zero-points enter as for the unsigned 8-bit operand:
//     sum (a-za)(b-zb) = sum (a-128)(b-128) + (128-zb) * rowsum'[i] + (128-za) * colsum'[j] + K (128-za)(128-zb)
// with rowsum'[i] = sum_k (a[i][k] - 128), colsum'[j] = sum_k (b[k][j] - 128): the epilogue above with
// zb - 128 in the place of zb.
//
// Packed B: per 32-column panel and 32 elements of K two fragments, the ah-plane and the al'-plane, in
// the fragment layout of the 8-bit pack (byte n of lane l = element 16 * (l / 32) + n of column l % 32),
// panel contiguous over K; zero padded to (K rounded up to 32) x (N rounded up to 32).  A's bytes are
// separated after the LDS read by byte permutes.

// Row sums of an int16 matrix minus 128 per element: out[i] = sum_k (X[i][k] - 128), rows >= rows_valid
// give 0.  One wavefront per row.
__global__ __launch_bounds__(256) void rowsum_s16_kernel(const int16_t *__restrict__ X, int64_t ldx, int rows_valid,
                                                         int rows_out, int K, int32_t *__restrict__ out)
{
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (i >= rows_out) return;
    int s = 0;
    if (i < rows_valid) {
        const int16_t *row = X + (int64_t)i * ldx;
        for (int k = lane * 8; k < K; k += 64 * 8) {
            if (k + 8 <= K) {
                int16_t v[8];
                __builtin_memcpy(v, row + k, 16);
#pragma unroll
                for (int t = 0; t < 8; ++t) s += (int)v[t] - 128;
            } else {
                for (int t = 0; k + t < K; ++t) s += (int)row[k + t] - 128;
            }
        }
    }
    s = wave_sum(s);
    if (lane == 0) out[i] = s;
}

// Pack of the int16 operand.  One thread per (panel, 32-element slice, lane of the fragment): it reads
// its 16 elements and writes 16 bytes into each plane.
__global__ __launch_bounds__(256) void pack_b_s16_kernel(const int16_t *__restrict__ B, int64_t ldb, int K, int N,
                                                         int nslices, int64_t nchunks, uint8_t *__restrict__ packed)
{
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= nchunks) return;
    const int l = (int)(id & 63);
    const int64_t f = id >> 6;                           // (panel, slice)
    const int s = (int)(f % nslices);
    const int64_t pnl = f / nslices;
    const int64_t j = pnl * 32 + (l & 31);
    const int k0 = s * 32 + (l >> 5) * 16;
    uint32_t hi[4] = {0u, 0u, 0u, 0u}, lo[4] = {0u, 0u, 0u, 0u};
    if (j < N) {
        const int16_t *src = B + j * ldb + k0;
#pragma unroll
        for (int n = 0; n < 16; ++n)
            if (k0 + n < K) {
                const uint32_t v = (uint32_t)(uint16_t)src[n];
                hi[n >> 2] |= (v >> 8) << (8 * (n & 3));
                lo[n >> 2] |= ((v & 255u) ^ 0x80u) << (8 * (n & 3));
            }
    }
    v4i h, w;
    h.x = (int)hi[0]; h.y = (int)hi[1]; h.z = (int)hi[2]; h.w = (int)hi[3];
    w.x = (int)lo[0]; w.y = (int)lo[1]; w.z = (int)lo[2]; w.w = (int)lo[3];
    uint8_t *dst = packed + (f * 2) * kFragBytes + l * 16;
    *(v4i *)dst = h;
    *(v4i *)(dst + kFragBytes) = w;
}

struct S16Cfg {
    static constexpr int NSTAGE = 4;
    static constexpr int kABytes = 128 * 128;              // 128 rows x 64 elements
    static constexpr int kStageBytes = 2 * kABytes;        // + 4 panels x (2 slices x 2 planes) x 1 KiB
    static constexpr int kLoadsPerStage = 8;               // per lane: 4 copies of A (8 rows each), 4 fragments of B
    static constexpr int kPatchRow = 64 * 4 + 16;          // epilogue patch: 16 rows of 64 int32, padded
    static constexpr int kPatchBytes = 16 * kPatchRow;     // per wavefront
    static constexpr int kLdsBytes = NSTAGE * kStageBytes;
    static_assert(4 * kPatchBytes <= kLdsBytes, "epilogue patches fit the ring");
    static_assert((NSTAGE - 2) * kLoadsPerStage <= 63, "vmcnt range");
    static_assert(kLdsBytes <= 160 * 1024, "LDS of a compute unit");
};

// p.A / p.lda: the int16 matrix as bytes (lda in bytes, a multiple of 16, rows 16-byte aligned);
// p.K: elements; p.Kp: bytes of one packed column (2 * K rounded up to 32 elements); p.zb: zb - 128;
// p.rowsum / p.colsum: the sums above.  128 x 128 tiles, four wavefronts of 64 x 64 as 4 x 4 blocks of
// v_mfma_i32_16x16x64_i8 (on random operands that form does a fifth more work per joule than
// 32 x 32 x 32, and this kernel runs at the power limit like the 8-bit one).
// A stage is 64 elements of K: 128 bytes per row of A, copied as whole lines (one copy = 8 rows), and per
// panel the four fragments of two slices (ah, al', ah, al') as they lie in the pack.  Row R of A's tile
// lies in place R ^ ((R / 8) % 2) (the rows of every other group of eight swapped in pairs), chunk c of it
// at place c ^ (R % 8) of the 128 bytes: the sixteen lanes of a fragment read that share a chunk index
// then hit sixteen different 16-byte columns of the 256 bytes the banks span (measured: without the
// swap, rows R and R + 8 collide and every read of A takes twice the cycles).
// Operands of a 16-row / 16-column block: lane l takes row / column l % 16 and elements 16 (l / 16) .. + 15
// of the stage, i.e. two 16-byte chunks of A (separated into the byte planes by permutes) and from each
// plane of B the half (l / 16) % 2 of slice l / 32.
// With the packed operand first, lane l of a result block holds, for row l % 16 of A's block, the four
// consecutive columns 4 (l / 16) .. + 3 of B's block.
__global__ __launch_bounds__(256) void gemm_s16_tile_kernel(const GemmParams p)
{
    using Cfg = S16Cfg;
    constexpr int NSTAGE = Cfg::NSTAGE, LPS = Cfg::kLoadsPerStage;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int nfrag = p.Kp / 32;                         // fragments per panel (two per 32 elements)
    const int nfull = p.K / 64 & ~1;                     // stages of the pipelined loop: an even number
    const int nstages = (p.K + 63) / 64;                 // the one or two after them (full, partial) go unpipelined
    const int ntiles = p.tiles_m * p.tiles_n;
    const int gsz = gridDim.x, w = blockIdx.x;

    const int ft = lane & 15, fc = lane >> 4;
    const int a_off0 = (wm * 64 + (ft ^ (ft >> 3))) * 128 + ((2 * fc) ^ (ft & 7)) * 16;   // chunk 2 fc of the row; chunk 2 fc + 1: ^ 16
    const int b_off = Cfg::kABytes + (wn * 8 + (fc >> 1) * 2) * kFragBytes + ((fc & 1) * 32 + ft) * 16;
    // a copy of A (8 rows, group q = wave + 4 d: its parity is the wavefront's): lane -> row of the eight, chunk
    const int cp_row = (lane >> 3) ^ (wave & 1), cp_chunk = (lane & 7) ^ cp_row;

    for (int tile = w; tile < ntiles; tile += gsz) {
        int tm, tn;
        tile_of_block(tile, p.tiles_m, p.tiles_n, p.nxcd, tm, tn);
        const int m0 = tm * 128, n0 = tn * 128;

        // copy d of this wavefront: rows 8 q .. + 7 of A's tile, q = wave + 4 d; fragment `wave` (plane and
        // slice) of panel d of B's tile
        const uint8_t *a_src[4], *b_src[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            int grow = m0 + (wave + 4 * d) * 8 + cp_row;
            grow = grow < p.M ? grow : p.M - 1;          // rows past M: read a valid row, never stored
            a_src[d] = p.A + (int64_t)grow * p.lda + cp_chunk * 16;
            int pnl = n0 / 32 + d;
            pnl = pnl < p.npanels ? pnl : p.npanels - 1;
            b_src[d] = p.Bp + ((int64_t)pnl * nfrag + wave) * kFragBytes + lane * 16;
        }
        auto dma_one = [&](int s, int d, int buf) {      // copy d (0..7) of stage s
            const int g = s < nfull ? s : nfull - 1;     // past the end: a copy nobody reads
            uint8_t *dst = lds + buf * Cfg::kStageBytes;
            if (d < 4)
                __builtin_amdgcn_global_load_lds((gptr_t)(a_src[d] + (int64_t)g * 128),
                                                 (lptr_t)(dst + (wave + 4 * d) * 1024), 16, 0, 0);
            else
                __builtin_amdgcn_global_load_lds((gptr_t)(b_src[d - 4] + (int64_t)g * (4 * kFragBytes)),
                                                 (lptr_t)(dst + Cfg::kABytes + (4 * (d - 4) + wave) * 1024), 16, 0, 0);
        };

        // Raw chunks of A's blocks (one set: block i's are consumed by the separation into planes before
        // the next stage's are read) and the fragments of B (two sets, [set][block][plane]).
        v4i ar[4][2], br[2][4][2];
        auto read_one = [&](auto set, int buf, int r) {  // fragment read r (0..15) of a stage: A's blocks, then B's
            constexpr int S = decltype(set)::value;
            const uint8_t *base = lds + buf * Cfg::kStageBytes;
            const int blk = (r >> 1) & 3, x = r & 1;
            if (r < 8)
                ar[blk][x] = *(const v4i *)(base + (a_off0 ^ (x * 16)) + blk * 2048);
            else
                br[S][blk][x] = *(const v4i *)(base + b_off + (blk >> 1) * (4 * kFragBytes) + (blk & 1) * 256 + x * kFragBytes);
        };

        // Four accumulators per block, one per product of byte planes (0: ah bh, 1: ah bl', 2: al' bl',
        // 3: al' bh): 256 registers, each updated once per stage.  (Products 1 and 3 could share one; with
        // every accumulator register taken the compiler keeps each sum in place, and operands out of them.)
        v4i acc[4][4][4];
        v4i ah[4], al[4];
        // bytes of 4 consecutive elements of block i (word wd of the two chunks) -> their high bytes and
        // their shifted low bytes
        auto split_word = [&](int i, int wd) {
            const v4i c = ar[i][wd >> 1];
            const uint32_t lo = (uint32_t)((wd & 1) ? c.z : c.x), hi = (uint32_t)((wd & 1) ? c.w : c.y);
            ah[i][wd] = (int)__builtin_amdgcn_perm(hi, lo, 0x07050301u);
            al[i][wd] = (int)(__builtin_amdgcn_perm(hi, lo, 0x06040200u) ^ 0x80808080u);
        };
        // matrix op m (0..63) of a stage: row block m / 16, product (m / 4) % 4, column block m % 4.
        // Packed operand first.  FIRST: the stage that starts the sums (a literal zero: accumulators
        // zeroed ahead of the loop make the compiler shuffle them between registers inside it).
        auto mma = [&](auto set, auto first, int m) {
            constexpr int S = decltype(set)::value;
            constexpr bool FIRST = decltype(first)::value != 0;
            const int i = m >> 4, q = (m >> 2) & 3, j = m & 3;
            const v4i b = br[S][j][(q == 1 || q == 2) ? 1 : 0], a = q < 2 ? ah[i] : al[i];
            if (FIRST) acc[q][i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b, a, v4i{0, 0, 0, 0}, 0, 0, 0);
            else acc[q][i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(b, a, acc[q][i][j], 0, 0, 0);
        };

        if (tile != w) __syncthreads();                  // the previous tile's LDS traffic is over

        if (nfull > 0) {
#pragma unroll
            for (int s = 0; s < NSTAGE - 1; ++s)
#pragma unroll
                for (int d = 0; d < LPS; ++d) dma_one(s, d, s);
            wait_vmcnt<(NSTAGE - 2) * LPS>();            // stage 0 has landed (this wavefront's part)
            __builtin_amdgcn_s_barrier();
#pragma unroll
            for (int r = 0; r < 16; ++r) read_one(IntC<0>{}, 0, r);
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) split_word(0, wd);
            __builtin_amdgcn_sched_barrier(0);

            // One stage: 64 matrix ops of sixteen cycles each; one wavefront per SIMD issues in order, about
            // one instruction every four cycles, so a gap between two matrix ops has room for three other
            // instructions.  Block i + 1's bytes are separated in the gaps 4..7 of block i (three
            // instructions each).  Behind the barrier in the middle, which makes stage it+1 complete and
            // the buffer of stage it-1 free: the fragments of stage it+1 (A's into the one set as its
            // blocks fall free, B's into the other set), one read per gap; then the copies of stage
            // it+NSTAGE-1 into the free buffer, every other gap; the gaps 56..59 separate block 0 of
            // stage it+1.
            auto body = [&](auto set, auto other, auto first, int it) {
                const int buf_n = (it + 1) % NSTAGE, buf_f = (it + NSTAGE - 1) % NSTAGE;
#pragma unroll
                for (int m = 0; m < 64; ++m) {
                    if (m == 32) {
                        wait_vmcnt<(NSTAGE - 3) * LPS>();
                        __builtin_amdgcn_s_barrier();
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if ((m & 15) >= 4 && (m & 15) < 8 && m < 48) split_word((m >> 4) + 1, m & 3);
                    if (m >= 56 && m < 60) split_word(0, m & 3);
                    // reads 0..5 (A's blocks 0..2), 8, 9 (B's block 0), 6, 7 (A's block 3, whose old chunks
                    // the gaps 36..39 consume), 10..15
                    if (m >= 32 && m < 48) read_one(other, buf_n, m < 38 ? m - 32 : m < 40 ? m - 30 : m < 42 ? m - 34 : m - 32);
                    if (m >= 48 && (m & 1)) dma_one(it + NSTAGE - 1, (m - 49) >> 1, buf_f);
                    __builtin_amdgcn_sched_barrier(0);
                    mma(set, first, m);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            body(IntC<0>{}, IntC<1>{}, IntC<1>{}, 0);
            body(IntC<1>{}, IntC<0>{}, IntC<0>{}, 1);
            for (int it = 2; it < nfull; it += 2) {
                body(IntC<0>{}, IntC<1>{}, IntC<0>{}, it);
                body(IntC<1>{}, IntC<0>{}, IntC<0>{}, it + 1);
            }
            wait_vmcnt<0>();                             // drain the copies nobody reads
        }

        // What is left of K: an odd last full stage and / or a partial one.  Guarded register loads of A,
        // the zero-padded planes of B (a slice the pack does not hold counts as zero), into the first
        // buffer in the stage's layout; no pipelining.  Without a pipelined part (K < 128) the first of them
        // starts the sums; K = 0 leaves a stage of zeros to do that.
        bool started = nfull > 0;
        for (int ts = nfull; ts < (nstages > 0 ? nstages : 1); ++ts) {
            const int kbase = ts * 128;                  // bytes into a row of A
            __syncthreads();
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int valid = 2 * p.K - (kbase + cp_chunk * 16);
                const uint8_t *src = a_src[d] + kbase;
                const v4i v = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
                *(v4i *)(lds + (wave + 4 * d) * 1024 + lane * 16) = v;
                v4i z = {0, 0, 0, 0};
                if (ts * 4 + wave < nfrag) z = *(const v4i *)(b_src[d] + (int64_t)ts * (4 * kFragBytes));
                *(v4i *)(lds + Cfg::kABytes + (4 * d + wave) * 1024 + lane * 16) = z;
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < 16; ++r) read_one(IntC<0>{}, 0, r);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int wd = 0; wd < 4; ++wd) split_word(i, wd);
            if (started) {
#pragma unroll
                for (int m = 0; m < 64; ++m) mma(IntC<0>{}, IntC<0>{}, m);
            } else {
#pragma unroll
                for (int m = 0; m < 64; ++m) mma(IntC<0>{}, IntC<1>{}, m);
            }
            started = true;
        }

        __syncthreads();                                 // every wavefront is done with the stage buffers

        // Epilogue.  Per 16-row block: (a-128)(b-128) sums = 65536 * acc0 + 256 * (acc1 + acc3) + acc2
        // (wrapping) plus the row term, written to the wavefront's LDS patch as they lie in the accumulators, read back
        // four rows per instruction, column terms added, stored as 256-byte row pieces.
        // (what the epilogue derives from the lane index is computed here: prepared ahead of the main loop
        // it would be carried across it in registers the loop needs, and spilled)
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        const int ft = lane_e & 15, fc = lane_e >> 4;
        uint8_t *patch = lds + wave * Cfg::kPatchBytes;
        const int cg = lane_e & 15, r4 = lane_e >> 4;
        const int bcol = n0 + wn * 64 + 4 * cg;
        uint4 ct = {0u, 0u, 0u, 0u};
        if (bcol < p.N) {
            const int4 cs = *(const int4 *)(p.colsum + bcol);        // colsum is padded to 32 columns
            ct.x = p.za_term * (uint32_t)cs.x; ct.y = p.za_term * (uint32_t)cs.y;
            ct.z = p.za_term * (uint32_t)cs.z; ct.w = p.za_term * (uint32_t)cs.w;
        }
        const bool interior = m0 + (wm + 1) * 64 <= p.M && n0 + (wn + 1) * 64 <= p.N;
        uint32_t row_terms[4];                           // all four first: independent loads
#pragma unroll
        for (int i = 0; i < 4; ++i) row_terms[i] = p.kconst;
        if (p.rowsum) {                                  // rows past M read row M - 1 and are never stored
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = m0 + wm * 64 + 16 * i + ft;
                row_terms[i] -= p.zb * (uint32_t)p.rowsum[row < p.M ? row : p.M - 1];
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // (block by block: the compiler would otherwise move all 256 accumulators into vector registers
            // ahead of the first block, where they do not fit beside what is live, and spill some of them)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) asm volatile("" : "+a"(acc[q][i][j]));
            const int brow0 = m0 + wm * 64 + 16 * i;
            const uint32_t rt = row_terms[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v4i v;
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    v[t] = (int)(((uint32_t)acc[0][i][j][t] << 16) + (((uint32_t)acc[1][i][j][t] + (uint32_t)acc[3][i][j][t]) << 8) +
                                 (uint32_t)acc[2][i][j][t] + rt);
                *(v4i *)(patch + ft * Cfg::kPatchRow + (16 * j + 4 * fc) * 4) = v;
            }
            v4i o[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = *(const v4i *)(patch + (4 * q + r4) * Cfg::kPatchRow + cg * 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                o[q].x = (int)((uint32_t)o[q].x + ct.x); o[q].y = (int)((uint32_t)o[q].y + ct.y);
                o[q].z = (int)((uint32_t)o[q].z + ct.z); o[q].w = (int)((uint32_t)o[q].w + ct.w);
            }
            int32_t *dst = (int32_t *)p.C + (int64_t)(brow0 + r4) * p.ldc + bcol;   // this lane's first row of the block
            if (interior) {
#pragma unroll
                for (int q = 0; q < 4; ++q, dst += 4 * p.ldc) __builtin_nontemporal_store(o[q], (v4i_a4 *)dst);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q, dst += 4 * p.ldc) {
                    const v4i v = o[q];
                    if (brow0 + 4 * q + r4 < p.M && bcol < p.N) {
                        if (bcol + 3 < p.N) {
                            __builtin_memcpy(dst, &v, 16);
                        } else {
                            dst[0] = v.x;
                            if (bcol + 1 < p.N) dst[1] = v.y;
                            if (bcol + 2 < p.N) dst[2] = v.z;
                        }
                    }
                }
            }
        }
    }
}

// ---- skinny-M kernel (M <= 32) --------------------------------------------------------------
// Bandwidth-bound: one workgroup per P adjacent 32-column panels; its wavefronts split K
// (wavefront v takes fragments v, v + nwaves, ... so that the workgroup sweeps a panel
// contiguously), each streaming its fragments of the packed operand straight from memory into
// registers (no LDS for B) and the few rows of A straight from cache.  An A fragment is loaded
// once and used against the P panels: with one panel per workgroup the cached reads of A grow to
// M/32 of the HBM traffic of B and cost 40 % of the bandwidth at M = 32, so wide outputs use
// P = 2 or 4 as long as that still leaves a workgroup per compute unit.  Loads are issued a
// batch of fragments ahead of the matrix ops that consume them (double buffered).  The partial
// 32 x 32 accumulators of the wavefronts are added through LDS as whole vectors (phase 2 of
// Sec. 3.1: vector adds, no lane tree), one panel after the other.
// ROWSUM_IN: the row sums the zero-point of B needs are formed from the A fragments as they pass
// (a dot product with ones per word of the bytes as loaded, before the shift, so that zero fill
// counts as zero: lane l sees row l % 32, the two halves of a slice sit in lanes l and l ^ 32; the
// shift of an unsigned A is K times 128, taken off in the constants).  At the end every lane
// fetches the sums of the 16 rows its accumulator registers belong to, and each wavefront takes zb
// times its share off its partial sums before they are added up.
template <bool REQUANT, int P, bool ROWSUM_IN = false>
__device__ __forceinline__ void skinny_body(const GemmParams &p0, int pnl0, int nregs, int *red)
{
    GemmParams p = p0;
    if (ROWSUM_IN) {
        const uint32_t shift_sum = p0.a_xor ? 128u * (uint32_t)p0.K : 0u;     // sum_k A' = sum_k A - this
        p.rowsum = nullptr;
        p.kconst = p0.kconst + p0.zb * shift_sum;
        p.rconst = p0.rconst - shift_sum;
    }
    constexpr int BATCH = P >= 4 ? 2 : 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwaves = blockDim.x >> 6;
    const int nslices = p.Kp / 32;
    const int mine = nslices > wave ? (nslices - wave + nwaves - 1) / nwaves : 0;   // fragments of this wavefront

    const int row = lane & 31;
    const bool row_ok = row < p.M;
    const uint8_t *a_row = p.A + (int64_t)(row_ok ? row : 0) * p.lda + (lane >> 5) * 16;
    const uint8_t *b_pan[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        int pn = pnl0 + j;
        pn = pn < p.npanels ? pn : p.npanels - 1;       // panels past N: read a valid one, never stored
        b_pan[j] = p.Bp + ((int64_t)pn * nslices) * kFragBytes + lane * 16;
    }
    auto load_a = [&](int t) {
        v4i af = {0, 0, 0, 0};
        if (row_ok) {
            const int s = wave + t * nwaves;
            const int valid = p.K - (s * 32 + (lane >> 5) * 16);
            const uint8_t *src = a_row + s * 32;
            af = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
        }
        return af;
    };

    v16i acc[P];
#pragma unroll
    for (int j = 0; j < P; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0;

    int rs_lane = 0;
    const bool want_rs = ROWSUM_IN && (p.zb != 0u || p.zb_vec != nullptr);

    v4i bf[2][BATCH][P], af[2][BATCH];
    const v4i zero = {0, 0, 0, 0};
    auto load_batch = [&](int slot, int t0) {
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const bool ok = t0 + u < mine;
#pragma unroll
            for (int j = 0; j < P; ++j)
                bf[slot][u][j] = ok ? __builtin_nontemporal_load((const v4i *)(b_pan[j] + (int64_t)(wave + (t0 + u) * nwaves) * kFragBytes))
                                    : zero;
            af[slot][u] = ok ? load_a(t0 + u) : zero;
        }
    };
    auto mma_batch = [&](int slot) {
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const v4i a = shift_u8_to_s8(af[slot][u], p.a_xor);
#pragma unroll
            for (int j = 0; j < P; ++j)
                acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, bf[slot][u][j], acc[j], 0, 0, 0);
            if (want_rs) {
                const v4i raw = af[slot][u];
                if (p.a_xor) {
                    uint32_t t = (uint32_t)rs_lane;
                    t = __builtin_amdgcn_udot4((uint32_t)raw.x, 0x01010101u, t, false);
                    t = __builtin_amdgcn_udot4((uint32_t)raw.y, 0x01010101u, t, false);
                    t = __builtin_amdgcn_udot4((uint32_t)raw.z, 0x01010101u, t, false);
                    t = __builtin_amdgcn_udot4((uint32_t)raw.w, 0x01010101u, t, false);
                    rs_lane = (int)t;
                } else {
                    rs_lane = __builtin_amdgcn_sdot4(raw.x, 0x01010101, rs_lane, false);
                    rs_lane = __builtin_amdgcn_sdot4(raw.y, 0x01010101, rs_lane, false);
                    rs_lane = __builtin_amdgcn_sdot4(raw.z, 0x01010101, rs_lane, false);
                    rs_lane = __builtin_amdgcn_sdot4(raw.w, 0x01010101, rs_lane, false);
                }
            }
        }
    };
    if (mine > 0) load_batch(0, 0);
    // the column terms: asked for now, needed after the loop (their latency hides under the stream)
    uint32_t cs_early[P];
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int col = (pnl0 + j) * 32 + (lane & 31);
        cs_early[j] = col < p.N ? p.za_term * (uint32_t)p.colsum[col] : 0u;
    }
    for (int t0 = 0; t0 < mine; t0 += 2 * BATCH) {
        if (t0 + BATCH < mine) load_batch(1, t0 + BATCH);
        mma_batch(0);          // a padded slot holds zeros for B: adds nothing
        if (t0 + BATCH < mine) {
            if (t0 + 2 * BATCH < mine) load_batch(0, t0 + 2 * BATCH);
            mma_batch(1);
        }
    }

    if (want_rs) {
        const int rs_row = rs_lane + __shfl_xor(rs_lane, 32, 64);      // this wavefront's share, row lane % 32
        uint32_t rs_out[16];                                          // ... of the row of accumulator register r
#pragma unroll
        for (int r = 0; r < 16; ++r) rs_out[r] = (uint32_t)__shfl(rs_row, 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), 64);
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int col = (pnl0 + j) * 32 + (lane & 31);
            const uint32_t zbj = (p.zb_vec && col < p.N) ? (uint32_t)p.zb_vec[col] : p.zb;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][r] = (int)((uint32_t)acc[j][r] - zbj * rs_out[r]);
        }
    }

#pragma unroll
    for (int j = 0; j < P; ++j) {
        if (pnl0 + j >= p.npanels) break;
        if (nwaves > 1) {
            if (j > 0) __syncthreads();                 // the previous panel's sums have been read
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (r < nregs) red[(wave * nregs + r) * 64 + lane] = acc[j][r];
            __syncthreads();
        }
        const int col = (pnl0 + j) * 32 + (lane & 31);
        const uint32_t cs_term = cs_early[j];
        for (int r = wave; r < nregs; r += nwaves) {
            int v = 0;
            if (nwaves > 1) {
                for (int w = 0; w < nwaves; ++w) v += red[(w * nregs + r) * 64 + lane];
            } else {
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    if (q == r) v = acc[j][q];
            }
            const int orow = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (orow < p.M && col < p.N) store_out<REQUANT>(p, orow, col, v, cs_term);
        }
    }
}

template <bool REQUANT, int P>
__global__ __launch_bounds__(512) void gemm_skinny_kernel(const GemmParams p, int nregs)
{
    extern __shared__ int red[];                       // [nwaves][nregs][64]
    skinny_body<REQUANT, P, true>(p, blockIdx.x * P, nregs, red);     // row sums formed here: no pass before it
}

// Grouped form: unit = one 32-column panel of one problem; always 8 wavefronts and room for 16
// accumulator registers per wavefront in LDS.
__global__ __launch_bounds__(512) void gemm_group_skinny_kernel(const GroupParams g)
{
    extern __shared__ int red[];
    const int q = group_find(g, blockIdx.x);
    const GemmParams p = group_member_params<64, 64>(g.prob[q], g.nxcd);
    skinny_body<false, 1, true>(p, blockIdx.x - g.unit_start[q], 4 * ((p.M + 7) / 8), red);
}

// Both kinds of member in one grid (see GroupParams): four wavefronts; a skinny member's panel is
// summed over K by the four of them, a tile is the 2 x 2 wavefront form of the staged kernel.  The
// skinny members come first in the grid: the longest of them take as long as the whole launch and
// have to start with it.
template <int BM, int BN, int WGM, int WGN, int BK>
__global__ __launch_bounds__(WGM * WGN * 64) void gemm_group_kernel(const GroupParams g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int q = group_find(g, blockIdx.x);
    const GemmParams p = group_member_params<BM, BN>(g.prob[q], g.nxcd);
    const int unit = blockIdx.x - g.unit_start[q];
    if (q < g.first_tile) skinny_body<false, 1, true>(p, unit, 4 * ((p.M + 7) / 8), (int *)lds);
    else tile_body_staged<BM, BN, WGM, WGN, BK, false, true, kGroupRing>(p, unit, lds);
}

// ---- streaming skinny kernel (M <= 32, K short enough for A to sit in LDS) ---------------------
// For outputs of many panels (wide N, or the panels of all members of a grouped call): the unit
// of work is a whole 32-column panel over all of K, one per wavefront, so the partial sums of a
// panel never leave the wavefront's accumulators (no sum across wavefronts, no barrier per
// panel; Sec. 3.1 phases 1-2 at the scale of a wavefront).  A workgroup of four wavefronts takes
// a "chunk" of consecutive panels of one problem (wavefront w the panels w, w + 4, ...): it
// copies the problem's A once into LDS in the order the matrix instruction reads it (slice s =
// 32 values of K: [k-half][row] 16-byte pieces, rows padded to 8, 16 or 32, 16 bytes of padding
// per slice so that neither the fill nor the reads pile up on one bank), and then every
// wavefront streams its panels from memory with kStreamDepth fragments in flight, across panel
// boundaries.  The packed operand is read once and never again: its loads are non-temporal
// (measured on the target: 7.0 TB/s against 6.3 TB/s for plain loads of a read-only stream).
//
// Stores and loads share one in-order counter per wavefront: waiting for the oldest load after a
// panel's stores have been issued also waits for every load issued before those stores, which
// would empty the ring once per panel.  So only a wavefront's last panel is stored from the
// accumulators; the sums of its earlier panels are parked in LDS (the wavefront's own room, no
// barrier) and stored when its stream has ended.  Panels for which there is no room (many panels
// per wavefront, large A) are stored at once.
// Row sums for a zero-point of B: from the A fragments of the wavefront's first panel (the same
// for all its panels), as in skinny_body.
constexpr int kStreamDepth = 8;
constexpr int kStreamWaves = 4;
constexpr int kStreamMaxLds = 64 * 1024;               // what a kernel gets without an attribute
constexpr int kStreamMaxChunk = 64;                    // panels per workgroup at most

__host__ __device__ inline int stream_rows_pad(int M) { return M <= 8 ? 8 : (M <= 16 ? 16 : 32); }
__host__ __device__ inline int stream_slice_bytes(int M) { return 32 * stream_rows_pad(M) + 16; }
// LDS of one workgroup: A, the column terms of `chunk` panels, room to park `park` panels per wavefront
__host__ __device__ inline int stream_park_bytes(int M) { return 4 * ((M + 7) / 8) * 64 * 4; }     // one panel: the registers that hold rows < M
__host__ __device__ inline int64_t stream_lds_bytes(int M, int64_t Kp, int chunk, int park)
{
    return (Kp / 32) * stream_slice_bytes(M) + (int64_t)chunk * 128 + (int64_t)kStreamWaves * park * stream_park_bytes(M);
}

// lds_bytes: the dynamic LDS of the launch (at least stream_lds_bytes(M, Kp, chunk, 0))
template <bool REQUANT>
__device__ __forceinline__ void stream_body(const GemmParams &p0, int pnl_first, int pnl_count, int chunk, int lds_bytes,
                                            uint8_t *lds)
{
    GemmParams p = p0;
    {
        const uint32_t shift_sum = p0.a_xor ? 128u * (uint32_t)p0.K : 0u;     // sum_k A' = sum_k A - this
        p.rowsum = nullptr;
        p.kconst = p0.kconst + p0.zb * shift_sum;
        p.rconst = p0.rconst - shift_sum;
    }
    constexpr int D = kStreamDepth;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = p.Kp / 32;                                   // fragments per panel
    const int RP = stream_rows_pad(p.M), SB = stream_slice_bytes(p.M);

    // A -> LDS: 16-byte pieces in row-major order of (row, piece) over the threads, so that a
    // wavefront reads whole rows from memory; piece c of row r goes to slice c / 2, half c % 2.
    {
        const int cpr = p.Kp / 16, total = p.M * cpr;
        for (int base = 0; base < total; base += 4 * kStreamWaves * 64) {
            v4i v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = base + u * kStreamWaves * 64 + tid;
                v[u] = v4i{0, 0, 0, 0};
                if (idx < total) {
                    const int r = idx / cpr, c = idx - r * cpr;
                    const int valid = p.K - 16 * c;
                    const uint8_t *src = p.A + (int64_t)r * p.lda + 16 * c;
                    if (valid >= 16) v[u] = load16_any(src);
                    else if (valid > 0) v[u] = load16_partial(src, valid);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = base + u * kStreamWaves * 64 + tid;
                if (idx < total) {
                    const int r = idx / cpr, c = idx - r * cpr;
                    *(v4i *)(lds + (c >> 1) * SB + ((c & 1) * RP + r) * 16) = v[u];
                }
            }
        }
    }

    // column terms (128 - za) * colsum[j] of the chunk's panels -> LDS (the array covers the padded
    // columns): read from there when a panel ends, so that no wait on memory falls into the stream
    uint32_t *cs_lds = (uint32_t *)(lds + S * SB);
    for (int i = tid; i < pnl_count * 32; i += kStreamWaves * 64) cs_lds[i] = p.za_term * (uint32_t)p.colsum[pnl_first * 32 + i];

    // this wavefront's panels: pnl_first + wave + 4 i; its fragments form one stream.  Every slot
    // of the ring is loaded and consumed unconditionally (the compiler can then count the loads
    // in flight and wait for exactly the oldest): past the end of the stream a load fetches one
    // 16-byte piece for all lanes and its matrix op adds into sums that are never stored.
    const int my_panels = pnl_count > wave ? (pnl_count - wave + kStreamWaves - 1) / kStreamWaves : 0;
    const int total = my_panels * S;
    const uint8_t *bptr = p.Bp + ((int64_t)(pnl_first + (my_panels > 0 ? wave : 0)) * S) * kFragBytes + lane * 16;
    const int64_t panel_jump = (int64_t)(kStreamWaves - 1) * S * kFragBytes;
    int ld_s = 0, left = total;                               // slice of the next load in its panel; loads still to issue
    v4i buf[D];
    auto issue = [&](v4i &dst) {
        const uint8_t *src = left > 0 ? bptr : p.Bp;
        dst = __builtin_nontemporal_load((const v4i *)src);
        bptr += kFragBytes;
        if (++ld_s == S) {
            ld_s = 0;
            bptr += panel_jump;
        }
        --left;
    };
#pragma unroll
    for (int u = 0; u < D; ++u) issue(buf[u]);
    __syncthreads();                                         // A and the column terms are in LDS

    // room to park finished panels: what the launch's LDS holds beyond A and the column terms
    const int nregs = 4 * ((p.M + 7) / 8);                    // accumulator registers that hold rows < M
    const int park_off = S * SB + chunk * 128;
    int park_cap = (lds_bytes - park_off) / (kStreamWaves * nregs * 256);
    park_cap = park_cap < 0 ? 0 : park_cap;
    const int first_parked = my_panels - 1 - park_cap > 0 ? my_panels - 1 - park_cap : 0;     // panels before it: stored at once
    int *park = (int *)(lds + park_off) + wave * park_cap * nregs * 64 + lane;

    const int row = lane & 31;
    const uint8_t *a_lds = lds + ((lane >> 5) * RP + (row < p.M ? row : 0)) * 16;   // rows past M read row 0: never stored
    const bool want_rs = p.zb != 0u || p.zb_vec != nullptr;
    int rs_lane = 0, rs_row = 0;

    // zero-point terms and stores of one finished panel (index i of this wavefront)
    auto store_panel = [&](const v16i &sum, int i) {
        const int col = (pnl_first + wave + kStreamWaves * i) * 32 + (lane & 31);
        const uint32_t cs_term = cs_lds[(wave + kStreamWaves * i) * 32 + (lane & 31)];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row_lo = 8 * (r >> 2) + (r & 3);          // the lower of the two rows register r holds
            if (row_lo < p.M) {
                const int orow = row_lo + 4 * (lane >> 5);
                if (orow < p.M && col < p.N) store_out<REQUANT>(p, orow, col, sum[r], cs_term);
            }
        }
    };

    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;
    int s = 0, pi = 0;

    for (int f0 = 0; f0 < total; f0 += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const v4i raw = *(const v4i *)(a_lds + s * SB);
            const v4i a = shift_u8_to_s8(raw, p.a_xor);
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, buf[u], acc, 0, 0, 0);
            issue(buf[u]);
            if (want_rs && pi == 0) {
                if (p.a_xor) {
                    uint32_t t = (uint32_t)rs_lane;
                    t = __builtin_amdgcn_udot4((uint32_t)raw.x, 0x01010101u, t, false);
                    t = __builtin_amdgcn_udot4((uint32_t)raw.y, 0x01010101u, t, false);
                    t = __builtin_amdgcn_udot4((uint32_t)raw.z, 0x01010101u, t, false);
                    t = __builtin_amdgcn_udot4((uint32_t)raw.w, 0x01010101u, t, false);
                    rs_lane = (int)t;
                } else {
                    rs_lane = __builtin_amdgcn_sdot4(raw.x, 0x01010101, rs_lane, false);
                    rs_lane = __builtin_amdgcn_sdot4(raw.y, 0x01010101, rs_lane, false);
                    rs_lane = __builtin_amdgcn_sdot4(raw.z, 0x01010101, rs_lane, false);
                    rs_lane = __builtin_amdgcn_sdot4(raw.w, 0x01010101, rs_lane, false);
                }
            }
            if (++s == S) {
                s = 0;
                if (pi < my_panels) {
                    // the panel is complete
                    if (want_rs) {
                        // lane l has summed row l % 32 over its k-half; register r belongs to row
                        // 8 (r / 4) + 4 (l / 32) + r % 4
                        if (pi == 0) rs_row = rs_lane + __shfl_xor(rs_lane, 32, 64);
                        const int col = (pnl_first + wave + kStreamWaves * pi) * 32 + (lane & 31);
                        const uint32_t zbj = (p.zb_vec && col < p.N) ? (uint32_t)p.zb_vec[col] : p.zb;
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            acc[r] = (int)((uint32_t)acc[r] -
                                           zbj * (uint32_t)__shfl(rs_row, 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3), 64));
                    }
                    if (pi >= first_parked && pi < my_panels - 1) {
                        int *dst = park + (pi - first_parked) * nregs * 64;
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (r < nregs) dst[r * 64] = acc[r];
                    } else {
                        store_panel(acc, pi);
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[r] = 0;
                    ++pi;
                }
            }
        }
    }
    // the parked panels (written and read by this wavefront only)
    for (int i = first_parked; i < my_panels - 1; ++i) {
        const int *src = park + (i - first_parked) * nregs * 64;
        v16i sum;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[r] = r < nregs ? src[r * 64] : 0;
        store_panel(sum, i);
    }
}

// Single problem: `chunk` panels per workgroup.
template <bool REQUANT>
__global__ __launch_bounds__(kStreamWaves * 64) void gemm_stream_skinny_kernel(const GemmParams p, int chunk, int lds_bytes)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int first = blockIdx.x * chunk;
    const int count = p.npanels - first < chunk ? p.npanels - first : chunk;
    stream_body<REQUANT>(p, first, count, chunk, lds_bytes, lds);
}

// Grouped form: unit = a chunk of `chunk` consecutive panels of one member.  The launch's fixed
// costs (ramp, tail, the gap to the next launch: some 5 us) are shared by all its members, so the
// argument block is laid out to hold as many as 4 KiB can: 48 bytes per member, field by field
// (no padding), 32-bit pitches, and M, 128 - za and zb in one word.
constexpr int kStreamGroupMax = 84;
struct StreamGroupParams {
    int count;
    int nxcd;
    int chunk;               // panels per unit
    int lds_bytes;           // dynamic LDS of the launch
    int unit_start[kStreamGroupMax + 2];      // first unit of member q; [count] = grid size (one spare entry keeps the pointers aligned)
    const uint8_t *A[kStreamGroupMax];
    const uint8_t *Bp[kStreamGroupMax];
    void *C[kStreamGroupMax];
    int lda[kStreamGroupMax], ldc[kStreamGroupMax], N[kStreamGroupMax], K[kStreamGroupMax];
    uint32_t mzz[kStreamGroupMax];            // M | (128 - za) << 6 (9 bits, signed) | zb << 15 (8 bits, signed)
};
static_assert(sizeof(StreamGroupParams) <= 4096, "kernel argument block");

__host__ __device__ inline uint32_t stream_pack_mzz(int M, uint32_t za_term, uint32_t zb)
{
    return (uint32_t)M | (za_term & 0x1ffu) << 6 | (zb & 0xffu) << 15;
}

__global__ __launch_bounds__(kStreamWaves * 64) void gemm_group_stream_kernel(const StreamGroupParams g)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int unit = blockIdx.x;
    int q = 0;
    for (int t = 1; t < g.count; ++t)
        if (unit >= g.unit_start[t]) q = t;
    GroupMember m;
    m.A = g.A[q]; m.Bp = g.Bp[q]; m.C = g.C[q];
    m.lda = g.lda[q]; m.ldc = g.ldc[q];
    m.N = g.N[q]; m.K = g.K[q];
    const uint32_t mzz = g.mzz[q];
    m.M = (int)(mzz & 63u);
    m.za_term = (int16_t)((int32_t)(mzz << 17) >> 23);        // sign-extend the 9 bits at [6, 15)
    m.zb = (int16_t)((int32_t)(mzz << 9) >> 24);              // ... the 8 bits at [15, 23)
    const GemmParams p = group_member_params<64, 64>(m, g.nxcd);
    const int first = (unit - g.unit_start[q]) * g.chunk;
    const int count = p.npanels - first < g.chunk ? p.npanels - first : g.chunk;
    stream_body<false>(p, first, count, g.chunk, g.lds_bytes, lds);
}

}  // namespace ngemm
