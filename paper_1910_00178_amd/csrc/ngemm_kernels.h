// Device kernels of the gfx950 u8 x s8 -> s32 GEMM.  Included only by ngemm.hip.
//
// Mapping of the paper's method onto CDNA4 (Sec. 3.1 of the paper):
//  * phase 1 (multiply narrow operands, widen, one partial sum per output
//    element held in its own SIMD lane) and phase 2 (accumulate partials
//    straight into the result vector, no horizontal tree reduction) are one
//    v_mfma_i32_32x32x32_i8: 1024 distinct C elements per wavefront, each
//    accumulated in place over the K loop.
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
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kFragBytes = 1024;   // 32 columns x 32 k-values
constexpr int kBK = 64;            // K bytes staged per main-loop step (two fragments deep)

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
    uint32_t za_term;       // 128 - za
    uint32_t zb;            // zb (two's complement)
    uint32_t kconst;        // -zb * (128 - za) * K  (mod 2^32)
    float scale;
    int32_t zc;
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

// u8 -> s8 shift of 16 packed bytes: a xor 0x80 == a - 128 read as signed.
__device__ __forceinline__ v4i shift_u8_to_s8(v4i v)
{
    v.x ^= (int)0x80808080u; v.y ^= (int)0x80808080u;
    v.z ^= (int)0x80808080u; v.w ^= (int)0x80808080u;
    return v;
}

// int32 value of one output element from its shifted-form accumulator.
__device__ __forceinline__ int32_t finish_s32(const GemmParams &p, int32_t acc, uint32_t cs_term, int row)
{
    uint32_t v = (uint32_t)acc + cs_term + p.kconst;
    if (p.rowsum) v -= p.zb * (uint32_t)p.rowsum[row];
    return (int32_t)v;
}

// Requantise-to-u8 sequence of the header: cvt, one multiply, round-half-even, add zc, clamp.
__device__ __forceinline__ uint8_t requant_u8(int32_t c, float scale, int32_t zc)
{
    float f = (float)c;
    float g = __fmul_rn(f, scale);
    float r = rintf(g);
    r = fminf(fmaxf(r, -4294967296.0f), 4294967296.0f);   // keeps the clamp below exact, avoids cvt overflow
    long long q = (long long)r + (long long)zc;
    q = q < 0 ? 0 : (q > 255 ? 255 : q);
    return (uint8_t)q;
}

template <bool REQUANT>
__device__ __forceinline__ void store_out(const GemmParams &p, int row, int col, int32_t acc, uint32_t cs_term)
{
    int32_t c = finish_s32(p, acc, cs_term, row);
    if (REQUANT)
        ((uint8_t *)p.C)[(int64_t)row * p.ldc + col] = requant_u8(c, p.scale, p.zc);
    else
        ((int32_t *)p.C)[(int64_t)row * p.ldc + col] = c;
}

__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ---- pack: column-major B -> fragment order, zero padded ------------------------------------
// One thread per 16-byte chunk of the packed buffer (linear, coalesced writes).
__global__ __launch_bounds__(256) void pack_b_kernel(const int8_t *__restrict__ B, int64_t ldb, int K, int N,
                                                     int Kp, int64_t nchunks, uint8_t *__restrict__ packed)
{
    int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= nchunks) return;
    const int nslices = Kp / 32;
    int64_t frag = c >> 6;
    int lane = (int)(c & 63);
    int pnl = (int)(frag / nslices);
    int s = (int)(frag % nslices);
    int j = pnl * 32 + (lane & 31);
    int k0 = s * 32 + (lane >> 5) * 16;
    v4i v = {0, 0, 0, 0};
    if (j < N && k0 < K) {
        const uint8_t *src = (const uint8_t *)B + (int64_t)j * ldb + k0;
        v = (k0 + 16 <= K) ? load16_any(src) : load16_partial(src, K - k0);
    }
    *(v4i *)(packed + c * 16) = v;
}

// colsum[j] = sum_k B[k][j]; one wavefront per column, cross-lane reduction at the end
// (the only place where a horizontal reduction survives; Sec. 2.1 phase 3).
__global__ __launch_bounds__(256) void colsum_b_kernel(const int8_t *__restrict__ B, int64_t ldb, int K, int N,
                                                       int Np, int32_t *__restrict__ colsum)
{
    int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (j >= Np) return;
    int s = 0;
    if (j < N) {
        const int8_t *col = B + (int64_t)j * ldb;
        for (int k = lane; k < K; k += 64) s += col[k];
        s = wave_sum(s);
    }
    if (lane == 0) colsum[j] = s;
}

// rowsum[i] = sum_k (A[i][k] - 128); needed only when zb != 0.
__global__ __launch_bounds__(256) void rowsum_a_kernel(const uint8_t *__restrict__ A, int64_t lda, int M, int K,
                                                       int32_t *__restrict__ rowsum)
{
    int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (i >= M) return;
    const uint8_t *row = A + (int64_t)i * lda;
    int s = 0;
    for (int k = lane; k < K; k += 64) s += (int)row[k] - 128;
    s = wave_sum(s);
    if (lane == 0) rowsum[i] = s;
}

// ---- tiled MFMA kernel ----------------------------------------------------------------------
// Workgroup tile BM x BN, WGM x WGN wavefronts, each owning (TM*32) x (TN*32) of C in
// accumulators.  A and B stages sit in LDS in fragment order (lane l's 16 bytes at 16*l of
// its fragment), so every fragment read is one conflict-free 16-byte-per-lane LDS load.
template <int BM, int BN, int WGM, int WGN>
struct TileCfg {
    static constexpr int kThreads = WGM * WGN * 64;
    static constexpr int TM = BM / (WGM * 32);
    static constexpr int TN = BN / (WGN * 32);
    static constexpr int kAChunks = BM * kBK / 16;            // 16-byte chunks per A stage
    static constexpr int kBChunks = BN * kBK / 16;
    static constexpr int kAIters = kAChunks / kThreads;
    static constexpr int kBIters = kBChunks / kThreads;
    static constexpr int kStageBytes = (BM + BN) * kBK;
    static_assert(kAChunks % kThreads == 0 && kBChunks % kThreads == 0, "loader shape");
    static_assert(TM >= 1 && TN >= 1, "wave tile");
};

// XCD-aware tile order: consecutive workgroup ids land on different XCDs (8 of them, each with
// its own L2), so give each XCD one contiguous run of the logical tile order, and make that
// order walk groups of GM tile-rows column by column so that the tiles in flight on one XCD
// share A row-panels and B column-panels.
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    const int nb = tiles_m * tiles_n;
    const int q = nb >> 3, r = nb & 7;
    const int xcd = bid & 7, local = bid >> 3;
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

template <int BM, int BN, int WGM, int WGN, bool REQUANT>
__global__ __launch_bounds__(WGM * WGN * 64) void gemm_tile_kernel(const GemmParams p)
{
    using Cfg = TileCfg<BM, BN, WGM, WGN>;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, NT = Cfg::kThreads;
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * Cfg::kStageBytes];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    int tm, tn;
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int nslices = p.Kp / 32;
    const int nkt = p.Kp / kBK;

    // Per-thread source addresses of this thread's chunks (k advances by kBK per step).
    const uint8_t *a_src[Cfg::kAIters];
    int a_koff[Cfg::kAIters];
#pragma unroll
    for (int i = 0; i < Cfg::kAIters; ++i) {
        int c = tid + i * NT;
        int f = c >> 6, l = c & 63;
        int row = (f >> 1) * 32 + (l & 31);
        int kc = (f & 1) * 2 + (l >> 5);
        int grow = m0 + row;
        grow = grow < p.M ? grow : p.M - 1;            // rows past M: read a valid row, never stored
        a_koff[i] = kc * 16;
        a_src[i] = p.A + (int64_t)grow * p.lda + kc * 16;
    }
    const uint8_t *b_src[Cfg::kBIters];
#pragma unroll
    for (int i = 0; i < Cfg::kBIters; ++i) {
        int c = tid + i * NT;
        int nb = c >> 7, within = c & 127;
        int pnl = n0 / 32 + nb;
        pnl = pnl < p.npanels ? pnl : p.npanels - 1;   // panels past N: read a valid panel, never stored
        b_src[i] = p.Bp + ((int64_t)pnl * nslices) * kFragBytes + within * 16;
    }

    v4i ra[Cfg::kAIters], rb[Cfg::kBIters];
    auto load_stage = [&](int kt) {
        const int kbase = kt * kBK;
        const bool full = kbase + kBK <= p.K;
#pragma unroll
        for (int i = 0; i < Cfg::kAIters; ++i) {
            const uint8_t *src = a_src[i] + kbase;
            if (full) {
                ra[i] = load16_any(src);
            } else {
                int valid = p.K - (kbase + a_koff[i]);
                ra[i] = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
            }
        }
#pragma unroll
        for (int i = 0; i < Cfg::kBIters; ++i)
            rb[i] = *(const v4i *)(b_src[i] + (int64_t)kt * (2 * kFragBytes));
    };
    auto store_stage = [&](int buf) {
        uint8_t *As = lds + buf * Cfg::kStageBytes;
        uint8_t *Bs = As + BM * kBK;
#pragma unroll
        for (int i = 0; i < Cfg::kAIters; ++i)
            *(v4i *)(As + (tid + i * NT) * 16) = shift_u8_to_s8(ra[i]);
#pragma unroll
        for (int i = 0; i < Cfg::kBIters; ++i)
            *(v4i *)(Bs + (tid + i * NT) * 16) = rb[i];
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    if (nkt > 0) {
        load_stage(0);
        store_stage(0);
        __syncthreads();
    }
    for (int kt = 0; kt < nkt; ++kt) {
        const bool more = kt + 1 < nkt;
        if (more) load_stage(kt + 1);
        const uint8_t *As = lds + (kt & 1) * Cfg::kStageBytes;
        const uint8_t *Bs = As + BM * kBK;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *(const v4i *)(As + (((wm * TM + i) * 2 + ks) * kFragBytes) + lane * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bf[j] = *(const v4i *)(Bs + (((wn * TN + j) * 2 + ks) * kFragBytes) + lane * 16);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_stage((kt + 1) & 1);
        __syncthreads();
    }

    // Epilogue.  Accumulator register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32] of its
    // 32 x 32 block: consecutive lanes write consecutive columns of one row.
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
        if (col >= p.N) continue;
        const uint32_t cs_term = p.za_term * (uint32_t)p.colsum[col];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int rbase = m0 + (wm * TM + i) * 32 + 4 * (lane >> 5);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = rbase + 8 * (r >> 2) + (r & 3);
                if (row < p.M) store_out<REQUANT>(p, row, col, acc[i][j][r], cs_term);
            }
        }
    }
}

// ---- skinny-M kernel (M <= 32) --------------------------------------------------------------
// Bandwidth-bound: one workgroup per 32-column panel; its wavefronts split K, each streaming
// its fragments of the packed operand straight from memory into registers (no LDS for B) and
// the few rows of A straight from cache.  Partial 32 x 32 accumulators of the wavefronts are
// added through LDS as whole vectors (phase 2 of Sec. 3.1: vector adds, no lane tree).
template <bool REQUANT>
__global__ __launch_bounds__(1024) void gemm_skinny_kernel(const GemmParams p, int nregs)
{
    extern __shared__ int red[];                       // [nwaves][nregs][64]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nwaves = blockDim.x >> 6;
    const int pnl = blockIdx.x;
    const int nslices = p.Kp / 32;
    const int per_wave = (nslices + nwaves - 1) / nwaves;
    const int s0 = wave * per_wave;
    const int s1 = (s0 + per_wave) < nslices ? (s0 + per_wave) : nslices;

    const int row = lane & 31;
    const bool row_ok = row < p.M;
    const uint8_t *a_row = p.A + (int64_t)(row_ok ? row : 0) * p.lda + (lane >> 5) * 16;
    const uint8_t *b_pan = p.Bp + ((int64_t)pnl * nslices) * kFragBytes + lane * 16;

    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;

#pragma unroll 4
    for (int s = s0; s < s1; ++s) {
        v4i bf = *(const v4i *)(b_pan + (int64_t)s * kFragBytes);
        v4i af = {0, 0, 0, 0};
        if (row_ok) {
            int kk = s * 32 + (lane >> 5) * 16;
            int valid = p.K - kk;
            const uint8_t *src = a_row + s * 32;
            af = valid >= 16 ? load16_any(src) : load16_partial(src, valid < 0 ? 0 : valid);
        }
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(shift_u8_to_s8(af), bf, acc, 0, 0, 0);
    }

    if (nwaves > 1) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (r < nregs) red[(wave * nregs + r) * 64 + lane] = acc[r];
        __syncthreads();
    }
    const int col = pnl * 32 + (lane & 31);
    const uint32_t cs_term = col < p.N ? p.za_term * (uint32_t)p.colsum[col] : 0u;
    for (int r = wave; r < nregs; r += nwaves) {
        int v;
        if (nwaves > 1) {
            v = 0;
            for (int w = 0; w < nwaves; ++w) v += red[(w * nregs + r) * 64 + lane];
        } else {
            v = 0;
#pragma unroll
            for (int q = 0; q < 16; ++q)
                if (q == r) v = acc[q];
        }
        const int orow = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (orow < p.M && col < p.N) store_out<REQUANT>(p, orow, col, v, cs_term);
    }
}

}  // namespace ngemm
