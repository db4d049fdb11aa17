// Host side of the C ABI declared in include/ngemm.h: argument validation, kernel
// selection and launches.  Every step of the path runs in the kernels of
// ngemm_kernels.h; there is no CPU fallback.
#include "ngemm.h"
#include "ngemm_kernels.h"

#include <hip/hip_runtime.h>
#include <cmath>
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

using namespace ngemm;

// Scratch memory of ngemm_run_u8s8s32_static, the entry point for callers that cannot allocate:
// the row sums of A that a zero-point of B needs (4 bytes per row), in the device image of the
// library instead of a caller's workspace.  Every GPU the library runs on holds its own copy of
// the array until the process ends.  In host code the name below only stands for the symbol: the
// device address of a GPU's copy comes from hipGetSymbolAddress (ngemm_create keeps it in the
// context), and only that address is ever handed to a kernel.
constexpr int64_t kStaticMaxM = 65536;
constexpr size_t kStaticScratchBytes = (size_t)kStaticMaxM * 4;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct ngemm_ctx {
    uint32_t magic;
    int device;
    int num_cus;
    int num_xcd;             // XCDs (L2 domains) of the device; workgroup ids go round them in turn
    int force_kernel;
    int max_workgroups;      // 0 = one per compute unit
    void *static_scratch;    // device address of this device's copy of `scratch`
    // kernels found fastest by ngemm_tune_u8s8s32, by shape; consulted before the shape heuristic
    struct Tuned {
        int64_t M, N, K;
        int kernel;
    };
    std::vector<Tuned> tuned;
};

struct ngemm_packed_b {
    uint32_t magic;
    int device;
    int64_t K, N, Kp, Np;
    const uint8_t *data;     // device, caller-owned
    size_t bytes;
    int32_t b_shift;         // 0: packed from int8; 128: packed from uint8, stored as B - 128
    int32_t elem_bytes;      // 1: 8-bit operand; 2: int16 operand packed as two byte planes
};

namespace {

constexpr uint32_t kCtxMagic = 0x4e47454du;   // "NGEM"
constexpr uint32_t kPackMagic = 0x4e47504bu;  // "NGPK"
constexpr int64_t kMaxDim = 0x7fffffff - 4096;
constexpr int kSkinnyMaxM = 32;
constexpr int BK256 = 64;                        // stage depth of the 256 x 256 configuration
constexpr int kStages256 = 4;                    // ring depth of its direct-to-LDS form

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// gemm_tile_x64_kernel addresses its copies with 32-bit offsets from the tile's first row (panel,
// column): `rows` rows of `pitch` bytes, `extent` bytes used of the last one
inline bool x64_offsets_fit(int64_t rows, int64_t pitch, int64_t extent)
{
    return pitch < (1ll << 32) && (rows - 1) * pitch + extent + 4096 < (1ll << 32);
}

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        ok = (prev == dev) || (hipSetDevice(dev) == hipSuccess);
        if (prev == dev) prev = -1;
        // the launches below are checked with hipGetLastError(): drop an error that other code on
        // this thread left behind, so that it is not reported as one of ours
        (void)hipGetLastError();
    }
    ~DeviceGuard()
    {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

bool ctx_ok(const ngemm_ctx *c) { return c && c->magic == kCtxMagic; }
bool pack_ok(const ngemm_packed_b *b) { return b && b->magic == kPackMagic; }

template <int BM, int BN, int WGM, int WGN, int BK>
hipError_t launch_tile(const GemmParams &p0, bool requant, hipStream_t st, bool rows = false)
{
    using Cfg = TileCfg<BM, BN, WGM, WGN, BK>;
    GemmParams p = p0;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n)), block(WGM * WGN * 64);
    const size_t smem = Cfg::kLdsBytes;
    if constexpr (BM < 256) {
        // the form that adds up the row sums itself (64 x 64 and 128 x 128 tiles)
        static_assert(Cfg::kLdsBytes <= 64 * 1024, "needs no LDS attribute");
        if (rows) {
            if (requant)
                hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WGM, WGN, BK, true, true>), grid, block, smem, st, p);
            else
                hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WGM, WGN, BK, false, true>), grid, block, smem, st, p);
            return hipGetLastError();
        }
    }
    if (requant)
        hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WGM, WGN, BK, true>), grid, block, smem, st, p);
    else
        hipLaunchKernelGGL((gemm_tile_kernel<BM, BN, WGM, WGN, BK, false>), grid, block, smem, st, p);
    return hipGetLastError();
}

// Kernels whose LDS need exceeds the 64 KiB default must be opted in once per device.
template <int BM, int BN, int WGM, int WGN, int BK>
hipError_t allow_big_lds()
{
    using Cfg = TileCfg<BM, BN, WGM, WGN, BK>;
    if (Cfg::kLdsBytes <= 64 * 1024) return hipSuccess;
    hipError_t e = hipFuncSetAttribute((const void *)gemm_tile_kernel<BM, BN, WGM, WGN, BK, true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void *)gemm_tile_kernel<BM, BN, WGM, WGN, BK, false>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
}

template <int BM, int BN, int WGM, int WGN, int NSTAGE = 4>
hipError_t launch_tile_dma(const GemmParams &p0, bool requant, int num_cus, hipStream_t st,
                           const RawB *rawb = nullptr, bool rows = false)
{
    using Cfg = DmaCfg<BM, BN, WGM, WGN, NSTAGE>;
    GemmParams p = p0;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    // Persistent workgroups: as many as can be resident (the 256 x 256 configuration fills a
    // compute unit's registers and LDS with one workgroup, the smaller ones leave room for more).
    const int ntiles = p.tiles_m * p.tiles_n;
    const int per_cu = BM >= 256 ? 1 : (BM >= 128 ? 2 : 4);
    const int nwg = ntiles < num_cus * per_cu ? ntiles : num_cus * per_cu;
    dim3 grid((unsigned)nwg), block(WGM * WGN * 64);
    const size_t smem = Cfg::kLdsBytes;
    const RawB none{nullptr, 0};
    if (rawb) {      // unpacked B: int32 output only
        hipLaunchKernelGGL((gemm_tile_dma_kernel<BM, BN, WGM, WGN, NSTAGE, false, true>), grid, block, smem, st, p, *rawb);
        return hipGetLastError();
    }
    if constexpr (BM < 256) {
        // the form that adds up the row sums itself (64 x 64 and 128 x 128 tiles)
        static_assert(Cfg::kLdsBytes <= 64 * 1024, "needs no LDS attribute");
        if (rows) {
            if (requant)
                hipLaunchKernelGGL((gemm_tile_dma_kernel<BM, BN, WGM, WGN, NSTAGE, true, false, true>), grid, block, smem, st, p, none);
            else
                hipLaunchKernelGGL((gemm_tile_dma_kernel<BM, BN, WGM, WGN, NSTAGE, false, false, true>), grid, block, smem, st, p, none);
            return hipGetLastError();
        }
    }
    if (requant)
        hipLaunchKernelGGL((gemm_tile_dma_kernel<BM, BN, WGM, WGN, NSTAGE, true>), grid, block, smem, st, p, none);
    else
        hipLaunchKernelGGL((gemm_tile_dma_kernel<BM, BN, WGM, WGN, NSTAGE, false>), grid, block, smem, st, p, none);
    return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN, int NSTAGE = 4>
hipError_t allow_big_lds_dma()
{
    using Cfg = DmaCfg<BM, BN, WGM, WGN, NSTAGE>;
    if (Cfg::kLdsBytes <= 64 * 1024) return hipSuccess;
    hipError_t e = hipFuncSetAttribute((const void *)gemm_tile_dma_kernel<BM, BN, WGM, WGN, NSTAGE, true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)gemm_tile_dma_kernel<BM, BN, WGM, WGN, NSTAGE, false, true>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void *)gemm_tile_dma_kernel<BM, BN, WGM, WGN, NSTAGE, false>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
}

// Small tiles with the long pipeline: one workgroup per compute unit (the ring takes 128 KiB).
// T = 1: 64 x 64 tiles, stages of 256 bytes of K; T = 2: 128 x 128 tiles, stages of 128 bytes.
constexpr int kDeepStages = 4;
template <int T>
constexpr int kDeepSub = T == 1 ? 4 : 2;

// `rows`: the kernel forms the row sums itself (a zero-point of B is there; no row-sum pass ran)
template <int T>
hipError_t launch_tile_deep(const GemmParams &p0, bool requant, bool rows, int num_cus, hipStream_t st)
{
    using Cfg = DeepCfg<T, kDeepSub<T>, kDeepStages>;
    GemmParams p = p0;
    p.tiles_m = (p.M + Cfg::BMN - 1) / Cfg::BMN;
    p.tiles_n = (p.N + Cfg::BMN - 1) / Cfg::BMN;
    const int ntiles = p.tiles_m * p.tiles_n;
    dim3 grid((unsigned)(ntiles < num_cus ? ntiles : num_cus)), block(256);
    if (requant && rows)
        hipLaunchKernelGGL((gemm_tile_deep_kernel<T, kDeepSub<T>, kDeepStages, true, 0, true>), grid, block, Cfg::kLdsBytes, st, p);
    else if (requant)
        hipLaunchKernelGGL((gemm_tile_deep_kernel<T, kDeepSub<T>, kDeepStages, true>), grid, block, Cfg::kLdsBytes, st, p);
    else if (rows)
        hipLaunchKernelGGL((gemm_tile_deep_kernel<T, kDeepSub<T>, kDeepStages, false, 0, true>), grid, block, Cfg::kLdsBytes, st, p);
    else
        hipLaunchKernelGGL((gemm_tile_deep_kernel<T, kDeepSub<T>, kDeepStages, false>), grid, block, Cfg::kLdsBytes, st, p);
    return hipGetLastError();
}

// K split over workgroups for outputs that leave most compute units without a tile (64 x 64 tiles,
// int32 output): S = the number of parts that brings the grid up to the unit count, each part a
// multiple of 256 bytes of K (whole stages of the long pipeline) and at least kSplitMinChunk long.
// With room in the workspace the parts store their partial tiles there and a second kernel sums them
// and finishes the epilogue (any output type); without it C is cleared first and every part adds its
// partial tile with atomic adds (int32 outputs; exact in any order).
constexpr int kSplitMinChunk = 1024;
constexpr int kSplitMaxUnits = 256;        // (tile, part) units of a K split: one per compute unit at most
int splitk_parts(int64_t M, int64_t N, int64_t K, int num_cus, int *kchunk)
{
    const int64_t ntiles = ((M + 63) / 64) * ((N + 63) / 64);
    if (num_cus > kSplitMaxUnits) num_cus = kSplitMaxUnits;
    int64_t S = ntiles > 0 ? num_cus / ntiles : 1;
    if (S * kSplitMinChunk > K) S = K / kSplitMinChunk;
    if (S < 2) return 1;
    const int64_t chunk = round_up((K + S - 1) / S, 256);
    *kchunk = (int)chunk;
    return (int)((K + chunk - 1) / chunk);         // every part holds at least one byte of K
}

// Bytes of the partial results of a K split into `parts`.
size_t splitk_part_bytes(int64_t M, int64_t N, int parts)
{
    return (size_t)round_up((int64_t)parts * M * splitk_part_pitch(N) * 4, 256);
}

// part_ws: room for the partial results (splitk_part_bytes), or nullptr for the atomic form.
hipError_t launch_tile_deep_splitk(const GemmParams &p0, int parts, int kchunk, bool rows, bool requant, int32_t *part_ws,
                                   int num_cus, hipStream_t st)
{
    using Cfg = DeepCfg<1, kDeepSub<1>, kDeepStages>;
    GemmParams p = p0;
    p.tiles_m = (p.M + 63) / 64;
    p.tiles_n = (p.N + 63) / 64;
    p.ksplit = parts;
    p.kchunk = kchunk;
    p.part_ws = part_ws;
    const int nunits = p.tiles_m * p.tiles_n * parts;
    dim3 grid((unsigned)(nunits < num_cus ? nunits : num_cus)), block(256);
    if (part_ws) {
        if (rows)
            hipLaunchKernelGGL((gemm_tile_deep_kernel<1, kDeepSub<1>, kDeepStages, false, 2, true>), grid, block, Cfg::kLdsBytes, st, p);
        else
            hipLaunchKernelGGL((gemm_tile_deep_kernel<1, kDeepSub<1>, kDeepStages, false, 2, false>), grid, block, Cfg::kLdsBytes, st, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const int64_t lanes = (int64_t)p.M * (splitk_part_pitch(p.N) / 4);
        const dim3 rgrid((unsigned)((lanes + 63) / 64)), rblock(64 * (parts < kReduceWaves ? parts : kReduceWaves));
        if (requant)
            hipLaunchKernelGGL(splitk_reduce_kernel<true>, rgrid, rblock, 0, st, p, parts);
        else
            hipLaunchKernelGGL(splitk_reduce_kernel<false>, rgrid, rblock, 0, st, p, parts);
        return hipGetLastError();
    }
    const int64_t segs = (p.N + 1023) / 1024;
    hipLaunchKernelGGL(zero_c_kernel, dim3((unsigned)(p.M * segs)), dim3(256), 0, st, (int32_t *)p.C, p.ldc, p.N, (int)segs);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (rows)
        hipLaunchKernelGGL((gemm_tile_deep_kernel<1, kDeepSub<1>, kDeepStages, false, 1, true>), grid, block, Cfg::kLdsBytes, st, p);
    else
        hipLaunchKernelGGL((gemm_tile_deep_kernel<1, kDeepSub<1>, kDeepStages, false, 1, false>), grid, block, Cfg::kLdsBytes, st, p);
    return hipGetLastError();
}

template <int T>
hipError_t allow_big_lds_deep()
{
    using Cfg = DeepCfg<T, kDeepSub<T>, kDeepStages>;
    const void *forms[] = {
        (const void *)gemm_tile_deep_kernel<T, kDeepSub<T>, kDeepStages, false>,
        (const void *)gemm_tile_deep_kernel<T, kDeepSub<T>, kDeepStages, true>,
        (const void *)gemm_tile_deep_kernel<T, kDeepSub<T>, kDeepStages, false, 0, true>,
        (const void *)gemm_tile_deep_kernel<T, kDeepSub<T>, kDeepStages, true, 0, true>,
        (const void *)gemm_tile_deep_kernel<1, kDeepSub<1>, kDeepStages, false, 1, false>,
        (const void *)gemm_tile_deep_kernel<1, kDeepSub<1>, kDeepStages, false, 1, true>,
        (const void *)gemm_tile_deep_kernel<1, kDeepSub<1>, kDeepStages, false, 2, false>,
        (const void *)gemm_tile_deep_kernel<1, kDeepSub<1>, kDeepStages, false, 2, true>,
    };
    for (const void *f : forms) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::kLdsBytes);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int P>
void launch_skinny_p(const GemmParams &p, bool requant, int nwaves, int nregs, size_t smem, hipStream_t st)
{
    dim3 grid((unsigned)((p.npanels + P - 1) / P)), block(nwaves * 64);
    if (requant)
        hipLaunchKernelGGL((gemm_skinny_kernel<true, P>), grid, block, smem, st, p, nregs);
    else
        hipLaunchKernelGGL((gemm_skinny_kernel<false, P>), grid, block, smem, st, p, nregs);
}

// The streaming kernel (a panel per wavefront, A in LDS) can serve a problem when its A fits the
// 64 KiB of LDS a kernel gets without asking and there is a K to stream.
bool stream_can_serve(int64_t M, int64_t Kp)
{
    return Kp >= 64 && stream_lds_bytes((int)M, Kp, kStreamMaxChunk, 0) <= kStreamMaxLds;
}

// LDS of a streaming launch for one problem: what it needs, plus room to park the sums of all but
// the last panel of each wavefront as far as the 64 KiB allow.
int stream_launch_lds(int M, int64_t Kp, int chunk)
{
    const int per_wave = chunk / kStreamWaves - 1;
    int64_t want = stream_lds_bytes(M, Kp, chunk, per_wave > 0 ? per_wave : 0);
    return (int)(want < kStreamMaxLds ? want : kStreamMaxLds);
}

// Panels per workgroup of the streaming kernel for `panels` panels in all: R per wavefront, one
// as long as that makes no more than eight rounds of resident wavefronts (16 per compute unit):
// short-lived workgroups handed out by the dispatcher even out what a static share cannot
// (measured on 59 x 128 panels: R = 1, 1888 workgroups, 5.6 TB/s; R = 2, 944, one round, 5.45;
// on 84 x 128: R = 1 5.6, R = 2 5.5).
int stream_chunk(int64_t panels, int num_cus)
{
    const int64_t max_waves = (int64_t)num_cus * 128;
    int64_t R = (panels + max_waves - 1) / max_waves;
    R = R < 1 ? 1 : (R > kStreamMaxChunk / kStreamWaves ? kStreamMaxChunk / kStreamWaves : R);
    return (int)(kStreamWaves * R);
}

hipError_t launch_skinny(const GemmParams &p, bool requant, int num_cus, hipStream_t st)
{
    if (p.npanels >= 8 * num_cus && stream_can_serve(p.M, p.Kp)) {
        const int chunk = stream_chunk(p.npanels, num_cus);
        const dim3 grid((unsigned)((p.npanels + chunk - 1) / chunk)), block(kStreamWaves * 64);
        const int smem = stream_launch_lds(p.M, p.Kp, chunk);
        if (requant)
            hipLaunchKernelGGL(gemm_stream_skinny_kernel<true>, grid, block, (size_t)smem, st, p, chunk, smem);
        else
            hipLaunchKernelGGL(gemm_stream_skinny_kernel<false>, grid, block, (size_t)smem, st, p, chunk, smem);
        return hipGetLastError();
    }
    const int nslices = p.Kp / 32;
    int nwaves = 1;
    while (nwaves < 8 && nwaves * 4 <= nslices) nwaves *= 2;    // at least two fragments per wavefront, at most 8 wavefronts
    const int nregs = 4 * ((p.M + 7) / 8);
    const size_t smem = nwaves > 1 ? (size_t)nwaves * nregs * 64 * sizeof(int) : 0;
    // panels per workgroup: share an A fragment between panels when the output is wide enough to
    // still give every compute unit several workgroups (only worth it once A's rows are many)
    // (measured at N = 32768, K = 8192: M = 32 gains 30 % with four panels, M = 16 12 % with two;
    // at N = 16384 a workgroup per panel is still the fastest)
    if (p.M > 16 && p.npanels >= 4 * num_cus)
        launch_skinny_p<4>(p, requant, nwaves, nregs, smem, st);
    else if (p.M > 4 && p.npanels >= 4 * num_cus)
        launch_skinny_p<2>(p, requant, nwaves, nregs, smem, st);
    else
        launch_skinny_p<1>(p, requant, nwaves, nregs, smem, st);
    return hipGetLastError();
}

// Shape heuristic: the 256 x 256 configuration when it fills at least half of the compute units
// (3072^3, 144 tiles: 35 us against 47 us with 128 x 128; 2048 x 4096 x 1024, 128 tiles: a tie),
// the 128 x 128 one when every unit still gets a workgroup, else 64 x 64 (measured on 18 shapes
// from 16 x 512 x 512 to 4096^3: the smallest tile wins as long as the larger ones leave units
// idle; ngemm_tune_u8s8s32 settles the borderline cases by measurement).
constexpr int64_t kSplitMinK = 4096;
int choose_kernel(const ngemm_ctx *ctx, int64_t M, int64_t N, int64_t K)
{
    auto tiles = [&](int64_t b) { return ((M + b - 1) / b) * ((N + b - 1) / b); };
    const int64_t cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
    // Few tiles and a long K: spread K over the idle units.  The launch that clears C and the
    // atomic adds have to pay off: measured on 48 shapes, the split wins from K = 4096 on up to 48
    // tiles of 64 x 64, from 8192 up to 96, from 12288 up to 128; against the streaming kernel
    // (M <= 32) from K = 8192 while the output has at most 32 such tiles (N <= 2048).
    const int64_t t64 = tiles(64), step = 3 * cus / 16;
    if (M <= kSkinnyMaxM) {
        if (K >= 2 * kSplitMinK && t64 * 8 <= cus) return NGEMM_KERNEL_SPLIT_K;
        return NGEMM_KERNEL_SKINNY;
    }
    if (t64 * 2 <= cus && K >= kSplitMinK * ((t64 + step - 1) / step)) return NGEMM_KERNEL_SPLIT_K;
    const int64_t t192 = ((M + 191) / 192) * ((N + 255) / 256);
    // The large tiles pay off from 0.7 of the compute units filled with K >= 512 (4096 x 4096 x 256: 16.5 / 15.0), from 0.5 with K >= 1024,
    // from 0.4 with K >= 2048: their fill and epilogue want stages to spread over (us, large against
    // 128 x 128 tiles: 3072 x 3072 x 512 13.2 / 15.0, 2560 x 2560 x 512 10.8 / 9.6, 2176 x 2176 x 1024
    // 13.4 / 12.1, 2304^3 20.8 / 22.5, 2560^3 24.0 / 26.6).
    const int64_t big = tiles(256) > t192 ? tiles(256) : t192;
    if ((big * 10 >= cus * 7 && K >= 512) || (big * 2 >= cus && K >= 1024) || (big * 5 >= cus * 2 && K >= 2048)) {
        // rounds of resident workgroups times the rows of a tile: 192 x 256 tiles when they fill more of the
        // compute units for less time (3072^3: 144 tiles of 256 rows against 192 of 192, one round each;
        // 2560^3: 100 against 140, 29.3 us against 24.0 us, 128 x 128 tiles 26.6 us)
        const int64_t r256 = (tiles(256) + cus - 1) / cus * 256, r192 = (t192 + cus - 1) / cus * 192;
        return r192 < r256 ? NGEMM_KERNEL_TILE_192 : NGEMM_KERNEL_TILE_256;
    }
    // (1536^3, 144 tiles of 128 x 128: 10.0 us against 10.6 us with 64 x 64 tiles; 1024^3, 64 tiles: 7.9
    // against 5.5; 1536 x 1536 x 512: 6.9 against 6.4)
    if (tiles(128) >= cus || (tiles(128) * 5 >= cus * 2 && K >= 1024)) return NGEMM_KERNEL_TILE_128;
    return NGEMM_KERNEL_TILE_64;
}

int workgroup_budget(const ngemm_ctx *ctx)
{
    const int cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
    return (ctx->max_workgroups > 0 && ctx->max_workgroups < cus) ? ctx->max_workgroups : cus;
}

struct RunArgs {
    int64_t M;
    const uint8_t *A;
    int64_t lda;
    int32_t za, zb;
    const ngemm_packed_b *B;
    void *C;
    int64_t ldc;
    bool requant;
    float scale;
    int32_t zc;
    // per-column epilogue (requantising calls only)
    const float *scale_vec = nullptr;
    const int32_t *bias_vec = nullptr;
    const int32_t *zb_vec = nullptr;
    int relu = 0;
    bool a_signed = false;    // A holds int8 (s8 x s8 variant); za then lies in [-128,127]
    bool b_unsigned = false;  // B was packed from uint8 (u8 x u8 variant); zb is then the caller's zero-point - 128
    bool needs_rowsum() const { return zb != 0 || zb_vec != nullptr; }
};

ngemm_status validate_run(const ngemm_ctx *ctx, const RunArgs &a, int *kernel_out)
{
    if (!ctx_ok(ctx) || !pack_ok(a.B)) return NGEMM_ERR_INVALID_ARG;
    if (a.B->device != ctx->device) return NGEMM_ERR_INVALID_ARG;
    if (a.M < 0 || a.M > kMaxDim) return NGEMM_ERR_BAD_SHAPE;
    if (a.a_signed ? (a.za < -128 || a.za > 127) : (a.za < 0 || a.za > 255)) return NGEMM_ERR_INVALID_ARG;
    if ((a.B->b_shift != 0) != a.b_unsigned) return NGEMM_ERR_INVALID_ARG;   // entry point and pack disagree
    if (a.B->elem_bytes != 1) return NGEMM_ERR_INVALID_ARG;                  // a 16-bit pack: ngemm_run_s16s16s32 only
    if (a.zb < -128 || a.zb > 127) return NGEMM_ERR_INVALID_ARG;   // of the packed (signed) bytes
    if (a.requant && !a.scale_vec) {
        if (!std::isfinite(a.scale) || a.scale < 0x1p-30f || a.scale > 0x1p30f) return NGEMM_ERR_INVALID_ARG;
    }
    if (a.M == 0 || a.B->N == 0) {
        *kernel_out = NGEMM_KERNEL_AUTO;
        return NGEMM_OK;
    }
    if (!a.C || (!a.A && a.B->K > 0)) return NGEMM_ERR_INVALID_ARG;
    if (a.lda < a.B->K || a.ldc < a.B->N) return NGEMM_ERR_BAD_SHAPE;
    int k = ctx->force_kernel;
    if (k == NGEMM_KERNEL_AUTO) {
        for (const ngemm_ctx::Tuned &t : ctx->tuned)
            if (t.M == a.M && t.N == a.B->N && t.K == a.B->K) k = t.kernel;
        if (k == NGEMM_KERNEL_AUTO) k = choose_kernel(ctx, a.M, a.B->N, a.B->K);
    }
    if (k == NGEMM_KERNEL_SKINNY && a.M > kSkinnyMaxM) return NGEMM_ERR_INVALID_ARG;
    *kernel_out = k;
    return NGEMM_OK;
}

size_t rowsum_bytes(int64_t M) { return (size_t)round_up(M * 4, 256); }

// Kernel parameters of one validated GEMM (row sums not yet attached).
GemmParams make_params(const RunArgs &a, int nxcd)
{
    const ngemm_packed_b *B = a.B;
    GemmParams p;
    std::memset(&p, 0, sizeof p);
    p.A = a.A;
    p.lda = a.lda;
    p.Bp = B->data;
    p.colsum = (const int32_t *)(B->data + B->Kp * B->Np);
    p.rowsum = nullptr;
    p.C = a.C;
    p.ldc = a.ldc;
    p.M = (int)a.M;
    p.N = (int)B->N;
    p.K = (int)B->K;
    p.Kp = (int)B->Kp;
    p.npanels = (int)(B->Np / 32);
    const int32_t shift = a.a_signed ? 0 : 128;      // A' = A - shift is what the matrix pipe sees
    p.a_xor = a.a_signed ? 0u : 0x80808080u;
    p.za_term = (uint32_t)(shift - a.za);
    p.zb = (uint32_t)a.zb;
    p.kconst = 0u - (uint32_t)a.zb * (uint32_t)(shift - a.za) * (uint32_t)B->K;
    p.scale = a.scale;
    p.zc = a.zc;
    p.scale_vec = a.scale_vec;
    p.bias_vec = a.bias_vec;
    p.zb_vec = a.zb_vec;
    p.rconst = (uint32_t)(shift - a.za) * (uint32_t)B->K;
    p.relu = a.relu;
    p.ksplit = 1;
    p.kchunk = 0;
    p.nxcd = nxcd;
    return p;
}

// Launches one validated GEMM; `ws` must hold rowsum_bytes(M) when zb != 0.  What lies beyond those
// bytes serves the K split for its partial results when there is enough of it.
ngemm_status launch_run(const RunArgs &a, int kernel, int num_cus, int device_cus, int nxcd, void *ws, size_t ws_bytes,
                        hipStream_t st)
{
    const ngemm_packed_b *B = a.B;
    if (a.M == 0 || B->N == 0) return NGEMM_OK;
    GemmParams p = make_params(a, nxcd);
    const bool dma_ok = (((uintptr_t)a.A | (uintptr_t)a.lda) & 15) == 0;
    int kchunk = 0, parts = 1;
    int32_t *part_ws = nullptr;
    if (kernel == NGEMM_KERNEL_SPLIT_K) {
        // aligned rows of A only; u8 outputs need the workspace form and a zero-point of B per tensor;
        // what it cannot serve goes to the 64 x 64 tiles (to the streaming kernel when M <= 32)
        parts = dma_ok ? splitk_parts(a.M, B->N, B->K, num_cus, &kchunk) : 1;
        // int32 outputs always take the atomic form (never slower: 7.0 against 7.2 us for one tile,
        // 10.4 against 15.2 for 128 tiles at K = 4096); u8 outputs need the partial results in memory
        if (a.requant && parts >= 2 && ws && ws_bytes >= rowsum_bytes(a.M) + splitk_part_bytes(a.M, B->N, parts) && !a.zb_vec)
            part_ws = (int32_t *)((uint8_t *)ws + rowsum_bytes(a.M));
        if (a.requant && !part_ws) parts = 1;
        if (parts < 2) kernel = a.M <= kSkinnyMaxM ? NGEMM_KERNEL_SKINNY : NGEMM_KERNEL_TILE_64;
    }
    // at most one tile per compute unit and a K worth pipelining: the long-pipeline variants
    const bool deep64 = kernel == NGEMM_KERNEL_TILE_64 && dma_ok && B->K >= 512 &&
                        ((a.M + 63) / 64) * ((B->N + 63) / 64) <= (int64_t)device_cus;
    const bool deep128 = kernel == NGEMM_KERNEL_TILE_128 && dma_ok && B->K >= 512 &&
                         ((a.M + 127) / 128) * ((B->N + 127) / 128) <= (int64_t)device_cus;
    // the streaming kernel and every 64 x 64 and 128 x 128 kernel (the K split is one) form the row
    // sums themselves; the 256 x 256 kernels read them from a pass of their own
    const bool rows_in_kernel = kernel == NGEMM_KERNEL_SKINNY || kernel == NGEMM_KERNEL_SPLIT_K ||
                                kernel == NGEMM_KERNEL_TILE_64 || kernel == NGEMM_KERNEL_TILE_128;
    const bool rows_needed = a.needs_rowsum() && B->K > 0;
    if (rows_needed && !rows_in_kernel) {
        int32_t *rs = (int32_t *)ws;
        hipLaunchKernelGGL(rowsum_a_kernel, dim3((unsigned)((a.M + 3) / 4)), dim3(256), 0, st, a.A, a.lda,
                           (int)a.M, (int)B->K, p.a_xor, rs);
        if (hipGetLastError() != hipSuccess) return NGEMM_ERR_DEVICE;
        p.rowsum = rs;
    }
    hipError_t e;
    if (kernel == NGEMM_KERNEL_SPLIT_K)
        return launch_tile_deep_splitk(p, parts, kchunk, rows_needed, a.requant, part_ws, num_cus, st) == hipSuccess ? NGEMM_OK
                                                                                                                : NGEMM_ERR_DEVICE;
    switch (kernel) {
    case NGEMM_KERNEL_SKINNY: e = launch_skinny(p, a.requant, num_cus, st); break;
    // direct-to-LDS copies need 16-byte aligned rows of A; the register-staged kernels take the rest
    case NGEMM_KERNEL_TILE_64:
        if (deep64)
            e = launch_tile_deep<1>(p, a.requant, rows_needed, num_cus, st);
        else
            e = dma_ok ? launch_tile_dma<64, 64, 2, 2>(p, a.requant, num_cus, st, nullptr, rows_needed)
                       : launch_tile<64, 64, 2, 2, 64>(p, a.requant, st, rows_needed);
        break;
    case NGEMM_KERNEL_TILE_128:
        if (deep128)
            e = launch_tile_deep<2>(p, a.requant, rows_needed, num_cus, st);
        else
            e = dma_ok ? launch_tile_dma<128, 128, 2, 2>(p, a.requant, num_cus, st, nullptr, rows_needed)
                       : launch_tile<128, 128, 2, 2, 64>(p, a.requant, st, rows_needed);
        break;
    case NGEMM_KERNEL_TILE_192:
    case NGEMM_KERNEL_TILE_256:
        if (dma_ok && B->K >= X64Cfg::kMinK && x64_offsets_fit(256, a.lda, B->K) && x64_offsets_fit(9, 32 * round_up(B->K, 64), 0)) {
            // the 16 x 16 x 64 form of the matrix instruction; 192 x 256 tiles on request
            const int trows = kernel == NGEMM_KERNEL_TILE_192 ? 192 : 256;
            p.tiles_m = (p.M + trows - 1) / trows;
            p.tiles_n = (p.N + 255) / 256;
            const int ntiles = p.tiles_m * p.tiles_n;
            const dim3 grid((unsigned)(ntiles < num_cus ? ntiles : num_cus));
            const RawB none{nullptr, 0};
            if (trows == 192) {
                if (a.requant)
                    hipLaunchKernelGGL((gemm_tile_x64_kernel<false, true, true, 6>), grid, dim3(256), X64Cfg::kLdsBytes, st, p, none);
                else
                    hipLaunchKernelGGL((gemm_tile_x64_kernel<false, false, true, 6>), grid, dim3(256), X64Cfg::kLdsBytes, st, p, none);
            } else if (a.requant)
                hipLaunchKernelGGL((gemm_tile_x64_kernel<false, true>), grid, dim3(256), X64Cfg::kLdsBytes, st, p, none);
            else if (a.a_signed)      // signed A: the form without the u8 -> s8 shift
                hipLaunchKernelGGL((gemm_tile_x64_kernel<false, false, false>), grid, dim3(256), X64Cfg::kLdsBytes, st, p, none);
            else
                hipLaunchKernelGGL((gemm_tile_x64_kernel<false, false>), grid, dim3(256), X64Cfg::kLdsBytes, st, p, none);
            e = hipGetLastError();
        } else {
            e = dma_ok ? launch_tile_dma<256, 256, 2, 2, kStages256>(p, a.requant, num_cus, st)
                       : launch_tile<256, 256, 2, 2, BK256>(p, a.requant, st);
        }
        break;
    default: return NGEMM_ERR_INVALID_ARG;
    }
    return e == hipSuccess ? NGEMM_OK : NGEMM_ERR_DEVICE;
}

ngemm_status run_common(ngemm_ctx *ctx, const RunArgs &a, void *ws, size_t ws_bytes, void *stream)
{
    int kernel;
    ngemm_status s = validate_run(ctx, a, &kernel);
    if (s != NGEMM_OK) return s;
    if (a.M == 0 || a.B->N == 0) return NGEMM_OK;
    if (a.needs_rowsum() && a.B->K > 0) {
        if (!ws) return NGEMM_ERR_INVALID_ARG;
        if (ws_bytes < rowsum_bytes(a.M)) return NGEMM_ERR_BUFFER_TOO_SMALL;
    }
    // the kernels read and write the workspace in 16-byte pieces
    if (ws && ws_bytes > 0 && ((uintptr_t)ws & 15u) != 0) return NGEMM_ERR_INVALID_ARG;
    DeviceGuard g(ctx->device);
    if (!g.ok) return NGEMM_ERR_DEVICE;
    return launch_run(a, kernel, workgroup_budget(ctx), ctx->num_cus > 0 ? ctx->num_cus : 256, ctx->num_xcd, ws, ws_bytes,
                      (hipStream_t)stream);
}

}  // namespace

extern "C" {

const char *ngemm_status_string(ngemm_status s)
{
    switch (s) {
    case NGEMM_OK: return "ok";
    case NGEMM_ERR_INVALID_ARG: return "invalid argument";
    case NGEMM_ERR_BAD_SHAPE: return "bad shape or leading dimension";
    case NGEMM_ERR_BUFFER_TOO_SMALL: return "buffer too small";
    case NGEMM_ERR_DEVICE: return "HIP device error";
    case NGEMM_ERR_UNSUPPORTED_ARCH: return "unsupported architecture (gfx950 required)";
    case NGEMM_ERR_STATIC_LIMIT: return "problem exceeds the static scratch of the no-allocation entry point (M > 65536)";
    }
    return "unknown status";
}

ngemm_status ngemm_create(ngemm_ctx **out, int device_ordinal)
{
    if (!out) return NGEMM_ERR_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device_ordinal < 0 || device_ordinal >= count) {
        (void)hipGetLastError();
        return NGEMM_ERR_DEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device_ordinal) != hipSuccess) return NGEMM_ERR_DEVICE;
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return NGEMM_ERR_UNSUPPORTED_ARCH;
    ngemm_ctx *c = new (std::nothrow) ngemm_ctx;
    if (!c) return NGEMM_ERR_DEVICE;
    c->magic = kCtxMagic;
    c->device = device_ordinal;
    c->num_cus = prop.multiProcessorCount;
    // XCDs: each has an L2 of its own, and consecutive workgroup ids are dispatched to them in turn
    int nxcc = 0;
    if (hipDeviceGetAttribute(&nxcc, hipDeviceAttributeNumberOfXccs, device_ordinal) != hipSuccess || nxcc < 1) {
        (void)hipGetLastError();
        nxcc = 8;                                    // the MI355X layout
    }
    c->num_xcd = nxcc;
    c->force_kernel = NGEMM_KERNEL_AUTO;
    c->max_workgroups = 0;
    {
        DeviceGuard g(device_ordinal);
        // this device's copy of the static scratch array (every device has its own, at its own address)
        void *sp = nullptr;
        if (!g.ok || hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || !sp) {
            (void)hipGetLastError();
            delete c;
            return NGEMM_ERR_DEVICE;
        }
        c->static_scratch = sp;
        if (allow_big_lds<256, 256, 2, 2, BK256>() != hipSuccess ||
            allow_big_lds_dma<256, 256, 2, 2, kStages256>() != hipSuccess || allow_big_lds_dma<128, 128, 2, 2>() != hipSuccess ||
            allow_big_lds_dma<64, 64, 2, 2>() != hipSuccess || allow_big_lds_deep<1>() != hipSuccess || allow_big_lds_deep<2>() != hipSuccess ||
            hipFuncSetAttribute((const void *)gemm_tile_x64_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                X64Cfg::kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute((const void *)gemm_tile_x64_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                X64Cfg::kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute((const void *)gemm_tile_x64_kernel<false, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                X64Cfg::kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute((const void *)gemm_tile_x64_kernel<false, false, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                X64Cfg::kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute((const void *)gemm_tile_x64_kernel<false, false, true, 6>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                X64Cfg::kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute((const void *)gemm_tile_x64_kernel<false, true, true, 6>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                X64Cfg::kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute((const void *)gemm_s16_tile_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                S16Cfg::kLdsBytes) != hipSuccess) {
            delete c;
            return NGEMM_ERR_DEVICE;
        }
    }
    *out = c;
    return NGEMM_OK;
}

ngemm_status ngemm_destroy(ngemm_ctx *ctx)
{
    if (!ctx) return NGEMM_OK;
    if (!ctx_ok(ctx)) return NGEMM_ERR_INVALID_ARG;
    ctx->magic = 0;
    delete ctx;
    return NGEMM_OK;
}

ngemm_status ngemm_set_kernel(ngemm_ctx *ctx, int kernel)
{
    if (!ctx_ok(ctx)) return NGEMM_ERR_INVALID_ARG;
    if (kernel < NGEMM_KERNEL_AUTO || kernel >= NGEMM_KERNEL_COUNT) return NGEMM_ERR_INVALID_ARG;
    ctx->force_kernel = kernel;
    return NGEMM_OK;
}

ngemm_status ngemm_tune_u8s8s32(ngemm_ctx *ctx, int64_t M, const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                                const ngemm_packed_b *B, int32_t b_zero_point, int32_t *C_dev, int64_t ldc,
                                void *workspace_dev, size_t workspace_bytes, void *hip_stream, int *best_kernel)
{
    if (best_kernel) *best_kernel = NGEMM_KERNEL_AUTO;
    if (!ctx_ok(ctx) || !pack_ok(B)) return NGEMM_ERR_INVALID_ARG;
    RunArgs a{M, A_dev, lda, a_zero_point, b_zero_point, B, C_dev, ldc, false, 1.0f, 0};
    const int saved = ctx->force_kernel;
    int dummy;
    ctx->force_kernel = NGEMM_KERNEL_TILE_64;         // valid for every shape: checks the arguments
    ngemm_status s = validate_run(ctx, a, &dummy);
    ctx->force_kernel = saved;
    if (s != NGEMM_OK) return s;
    if (M == 0 || B->N == 0 || B->K == 0) return NGEMM_OK;   // nothing to measure
    DeviceGuard g(ctx->device);
    if (!g.ok) return NGEMM_ERR_DEVICE;
    hipStream_t st = (hipStream_t)hip_stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return NGEMM_ERR_DEVICE;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return NGEMM_ERR_DEVICE;
    }
    const int candidates[6] = {NGEMM_KERNEL_SKINNY, NGEMM_KERNEL_TILE_64, NGEMM_KERNEL_TILE_128, NGEMM_KERNEL_TILE_256,
                               NGEMM_KERNEL_SPLIT_K, NGEMM_KERNEL_TILE_192};
    int best = NGEMM_KERNEL_AUTO;
    float best_ms = 0.0f;
    s = NGEMM_OK;
    for (int c = 0; c < 6 && s == NGEMM_OK; ++c) {
        const int k = candidates[c];
        if (k == NGEMM_KERNEL_SKINNY && M > kSkinnyMaxM) continue;
        // a tile far larger than the output cannot win: skip what would leave most of it empty
        if ((k == NGEMM_KERNEL_TILE_256 || k == NGEMM_KERNEL_TILE_192) && (M <= 64 || B->N <= 64)) continue;
        if (k == NGEMM_KERNEL_SPLIT_K) {
            // only where it would really split (else it is the 64 x 64 candidate once more)
            int kchunk = 0;
            const bool dma_ok = (((uintptr_t)A_dev | (uintptr_t)lda) & 15) == 0;
            if (!dma_ok || splitk_parts(M, B->N, B->K, workgroup_budget(ctx), &kchunk) < 2) continue;
        }
        ctx->force_kernel = k;
        // three rounds of 50 launches after a warm-up, the fastest round counts: short kernels are
        // within the noise of one another otherwise (clock ramp, first-touch effects)
        const int warm = 5, reps = 50, rounds = 3;
        float ms = 0.0f;
        for (int round = 0; round < rounds && s == NGEMM_OK; ++round) {
            for (int r = (round == 0 ? 0 : warm); r < warm + reps && s == NGEMM_OK; ++r) {
                if (r == warm && hipEventRecord(e0, st) != hipSuccess) s = NGEMM_ERR_DEVICE;
                if (s == NGEMM_OK) s = run_common(ctx, a, workspace_dev, workspace_bytes, hip_stream);
            }
            float t = 0.0f;
            if (s == NGEMM_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                                  hipEventElapsedTime(&t, e0, e1) != hipSuccess))
                s = NGEMM_ERR_DEVICE;
            if (round == 0 || t < ms) ms = t;
        }
        if (s == NGEMM_OK && (best == NGEMM_KERNEL_AUTO || ms < best_ms)) {
            best = k;
            best_ms = ms;
        }
    }
    ctx->force_kernel = saved;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (s != NGEMM_OK) return s;
    bool found = false;
    for (ngemm_ctx::Tuned &t : ctx->tuned)
        if (t.M == M && t.N == B->N && t.K == B->K) {
            t.kernel = best;
            found = true;
        }
    if (!found) {
        try {
            if (ctx->tuned.size() >= 4096) ctx->tuned.erase(ctx->tuned.begin());
            ctx->tuned.push_back(ngemm_ctx::Tuned{M, B->N, B->K, best});
        } catch (...) {
            return NGEMM_ERR_DEVICE;               // out of host memory: measured, but not remembered
        }
    }
    if (best_kernel) *best_kernel = best;
    return NGEMM_OK;
}

ngemm_status ngemm_tuned_kernel(const ngemm_ctx *ctx, int64_t M, int64_t N, int64_t K, int *kernel)
{
    if (!ctx_ok(ctx) || !kernel) return NGEMM_ERR_INVALID_ARG;
    *kernel = NGEMM_KERNEL_AUTO;
    for (const ngemm_ctx::Tuned &t : ctx->tuned)
        if (t.M == M && t.N == N && t.K == K) *kernel = t.kernel;
    return NGEMM_OK;
}

ngemm_status ngemm_set_max_workgroups(ngemm_ctx *ctx, int max_workgroups)
{
    if (!ctx_ok(ctx) || max_workgroups < 0) return NGEMM_ERR_INVALID_ARG;
    ctx->max_workgroups = max_workgroups;
    return NGEMM_OK;
}

size_t ngemm_packed_b_bytes(int64_t K, int64_t N)
{
    if (K < 0 || N < 0 || K > kMaxDim || N > kMaxDim) return 0;
    const int64_t Kp = round_up(K, 64), Np = round_up(N, 32);
    return (size_t)(Kp * Np + 4 * Np);
}

static ngemm_status pack_common(ngemm_ctx *ctx, int64_t K, int64_t N, const int8_t *B_dev, int64_t ldb,
                                void *packed_dev, size_t packed_bytes, void *hip_stream, ngemm_packed_b **out,
                                int32_t b_shift)
{
    if (!out) return NGEMM_ERR_INVALID_ARG;
    *out = nullptr;
    if (!ctx_ok(ctx)) return NGEMM_ERR_INVALID_ARG;
    if (K < 0 || N < 0 || K > kMaxDim || N > kMaxDim) return NGEMM_ERR_BAD_SHAPE;
    if (K > 0 && N > 0 && (!B_dev || ldb < K)) return B_dev ? NGEMM_ERR_BAD_SHAPE : NGEMM_ERR_INVALID_ARG;
    const size_t need = ngemm_packed_b_bytes(K, N);
    if (need > 0 && !packed_dev) return NGEMM_ERR_INVALID_ARG;
    if (packed_bytes < need) return NGEMM_ERR_BUFFER_TOO_SMALL;
    if (((uintptr_t)packed_dev & 15u) != 0) return NGEMM_ERR_INVALID_ARG;
    const int64_t Kp = round_up(K, 64), Np = round_up(N, 32);

    ngemm_packed_b *d = new (std::nothrow) ngemm_packed_b;
    if (!d) return NGEMM_ERR_DEVICE;
    d->magic = kPackMagic;
    d->device = ctx->device;
    d->K = K; d->N = N; d->Kp = Kp; d->Np = Np;
    d->data = (const uint8_t *)packed_dev;
    d->bytes = need;
    d->b_shift = b_shift;
    d->elem_bytes = 1;

    if (Np > 0) {
        DeviceGuard g(ctx->device);
        if (!g.ok) { delete d; return NGEMM_ERR_DEVICE; }
        hipStream_t st = (hipStream_t)hip_stream;
        int32_t *colsum = (int32_t *)((uint8_t *)packed_dev + Kp * Np);
        hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)((Np + 255) / 256)), dim3(256), 0, st, colsum, (int)Np);
        if (hipGetLastError() != hipSuccess) { delete d; return NGEMM_ERR_DEVICE; }
        if (Kp > 0) {
            const int64_t kblocks = (Kp + kPackKBytes - 1) / kPackKBytes;
            const int64_t nwg = (Np / 32) * kblocks;
            if (nwg > 0x7fffffff) { delete d; return NGEMM_ERR_BAD_SHAPE; }
            hipLaunchKernelGGL(pack_b_kernel, dim3((unsigned)nwg), dim3(256), 0, st, B_dev, ldb, (int)K, (int)N,
                               (int)Kp, (int)kblocks, b_shift ? 0x80808080u : 0u, (uint8_t *)packed_dev, colsum);
            if (hipGetLastError() != hipSuccess) { delete d; return NGEMM_ERR_DEVICE; }
        }
    }
    *out = d;
    return NGEMM_OK;
}

ngemm_status ngemm_pack_b(ngemm_ctx *ctx, int64_t K, int64_t N, const int8_t *B_dev, int64_t ldb,
                          void *packed_dev, size_t packed_bytes, void *hip_stream, ngemm_packed_b **out)
{
    return pack_common(ctx, K, N, B_dev, ldb, packed_dev, packed_bytes, hip_stream, out, 0);
}

ngemm_status ngemm_pack_b_u8(ngemm_ctx *ctx, int64_t K, int64_t N, const uint8_t *B_dev, int64_t ldb,
                             void *packed_dev, size_t packed_bytes, void *hip_stream, ngemm_packed_b **out)
{
    return pack_common(ctx, K, N, (const int8_t *)B_dev, ldb, packed_dev, packed_bytes, hip_stream, out, 128);
}

ngemm_status ngemm_packed_b_free(ngemm_packed_b *b)
{
    if (!b) return NGEMM_OK;
    if (!pack_ok(b)) return NGEMM_ERR_INVALID_ARG;
    b->magic = 0;
    delete b;
    return NGEMM_OK;
}

ngemm_status ngemm_packed_b_shape(const ngemm_packed_b *b, int64_t *K, int64_t *N)
{
    if (!pack_ok(b) || !K || !N) return NGEMM_ERR_INVALID_ARG;
    *K = b->K;
    *N = b->N;
    return NGEMM_OK;
}

size_t ngemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || M > kMaxDim) return 0;
    size_t bytes = rowsum_bytes(M);
    // room for the partial results of the K split (outputs of few tiles with a long K: at most 4 MiB)
    if (N > 0 && N <= kMaxDim && K > 0 && K <= kMaxDim) {
        int kchunk = 0;
        const int parts = splitk_parts(M, N, K, kSplitMaxUnits, &kchunk);
        if (parts >= 2) bytes += splitk_part_bytes(M, N, parts);
    }
    return bytes;
}

ngemm_status ngemm_run_u8s8s32(ngemm_ctx *ctx, int64_t M, const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                               const ngemm_packed_b *B, int32_t b_zero_point, int32_t *C_dev, int64_t ldc,
                               void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    RunArgs a{M, A_dev, lda, a_zero_point, b_zero_point, B, C_dev, ldc, false, 1.0f, 0};
    return run_common(ctx, a, workspace_dev, workspace_bytes, hip_stream);
}

ngemm_status ngemm_run_u8s8s32_static(ngemm_ctx *ctx, int64_t M, const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                                      const ngemm_packed_b *B, int32_t b_zero_point, int32_t *C_dev, int64_t ldc,
                                      void *hip_stream)
{
    if (!ctx_ok(ctx)) return NGEMM_ERR_INVALID_ARG;
    if (M > kStaticMaxM) return NGEMM_ERR_STATIC_LIMIT;
    // ngemm_run_u8s8s32 with the row sums in this device's static array (its address, taken at
    // ngemm_create; never the symbol).  The kernel that forms them writes all M entries before
    // the GEMM kernel behind it on the stream reads them, so nothing needs clearing; room for a K
    // split's partial results is not offered (int32 outputs add their parts into C).
    RunArgs a{M, A_dev, lda, a_zero_point, b_zero_point, B, C_dev, ldc, false, 1.0f, 0};
    return run_common(ctx, a, ctx->static_scratch, kStaticScratchBytes, hip_stream);
}

ngemm_status ngemm_run_s8s8s32(ngemm_ctx *ctx, int64_t M, const int8_t *A_dev, int64_t lda, int32_t a_zero_point,
                               const ngemm_packed_b *B, int32_t b_zero_point, int32_t *C_dev, int64_t ldc,
                               void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    RunArgs a{M, (const uint8_t *)A_dev, lda, a_zero_point, b_zero_point, B, C_dev, ldc, false, 1.0f, 0};
    a.a_signed = true;
    return run_common(ctx, a, workspace_dev, workspace_bytes, hip_stream);
}

ngemm_status ngemm_run_u8u8s32(ngemm_ctx *ctx, int64_t M, const uint8_t *A_dev, int64_t lda, int32_t a_zero_point,
                               const ngemm_packed_b *B, int32_t b_zero_point, int32_t *C_dev, int64_t ldc,
                               void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    // (B - zb) == (B - 128) - (zb - 128): the packed bytes are already B - 128
    if (b_zero_point < 0 || b_zero_point > 255) return NGEMM_ERR_INVALID_ARG;
    RunArgs a{M, A_dev, lda, a_zero_point, b_zero_point - 128, B, C_dev, ldc, false, 1.0f, 0};
    a.b_unsigned = true;
    return run_common(ctx, a, workspace_dev, workspace_bytes, hip_stream);
}

ngemm_status ngemm_run_u8s8u8_requant(ngemm_ctx *ctx, int64_t M, const uint8_t *A_dev, int64_t lda,
                                      int32_t a_zero_point, const ngemm_packed_b *B, int32_t b_zero_point,
                                      float scale, int32_t c_zero_point, uint8_t *C_dev, int64_t ldc,
                                      void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    RunArgs a{M, A_dev, lda, a_zero_point, b_zero_point, B, C_dev, ldc, true, scale, c_zero_point};
    return run_common(ctx, a, workspace_dev, workspace_bytes, hip_stream);
}

ngemm_status ngemm_run_u8s8u8_requant_channel(ngemm_ctx *ctx, int64_t M, const uint8_t *A_dev, int64_t lda,
                                              int32_t a_zero_point, const ngemm_packed_b *B, int32_t b_zero_point,
                                              const int32_t *b_zero_points_dev, const float *scales_dev,
                                              const int32_t *bias_dev, int32_t relu, int32_t c_zero_point,
                                              uint8_t *C_dev, int64_t ldc, void *workspace_dev,
                                              size_t workspace_bytes, void *hip_stream)
{
    if (!scales_dev) return NGEMM_ERR_INVALID_ARG;
    RunArgs a{M, A_dev, lda, a_zero_point, b_zero_point, B, C_dev, ldc, true, 1.0f, c_zero_point};
    a.scale_vec = scales_dev;
    a.bias_vec = bias_dev;
    a.zb_vec = b_zero_points_dev;
    a.relu = relu ? 1 : 0;
    return run_common(ctx, a, workspace_dev, workspace_bytes, hip_stream);
}

size_t ngemm_packed_b_bytes_s16(int64_t K, int64_t N)
{
    if (K < 0 || N < 0 || K > kMaxDim / 2 || N > kMaxDim) return 0;
    const int64_t Kp = 2 * round_up(K, 32), Np = round_up(N, 32);
    return (size_t)(Kp * Np + 4 * Np);
}

ngemm_status ngemm_pack_b_s16(ngemm_ctx *ctx, int64_t K, int64_t N, const int16_t *B_dev, int64_t ldb,
                              void *packed_dev, size_t packed_bytes, void *hip_stream, ngemm_packed_b **out)
{
    if (!out) return NGEMM_ERR_INVALID_ARG;
    *out = nullptr;
    if (!ctx_ok(ctx)) return NGEMM_ERR_INVALID_ARG;
    if (K < 0 || N < 0 || K > kMaxDim / 2 || N > kMaxDim) return NGEMM_ERR_BAD_SHAPE;
    if (K > 0 && N > 0 && (!B_dev || ldb < K)) return B_dev ? NGEMM_ERR_BAD_SHAPE : NGEMM_ERR_INVALID_ARG;
    if (((uintptr_t)B_dev & 1u) != 0) return NGEMM_ERR_INVALID_ARG;
    const size_t need = ngemm_packed_b_bytes_s16(K, N);
    if (need > 0 && !packed_dev) return NGEMM_ERR_INVALID_ARG;
    if (packed_bytes < need) return NGEMM_ERR_BUFFER_TOO_SMALL;
    if (((uintptr_t)packed_dev & 15u) != 0) return NGEMM_ERR_INVALID_ARG;
    const int64_t Kp = 2 * round_up(K, 32), Np = round_up(N, 32);
    ngemm_packed_b *d = new (std::nothrow) ngemm_packed_b;
    if (!d) return NGEMM_ERR_DEVICE;
    d->magic = kPackMagic;
    d->device = ctx->device;
    d->K = K; d->N = N; d->Kp = Kp; d->Np = Np;
    d->data = (const uint8_t *)packed_dev;
    d->bytes = need;
    d->b_shift = 0;
    d->elem_bytes = 2;
    if (Np > 0) {
        DeviceGuard g(ctx->device);
        if (!g.ok) { delete d; return NGEMM_ERR_DEVICE; }
        hipStream_t st = (hipStream_t)hip_stream;
        int32_t *colsum = (int32_t *)((uint8_t *)packed_dev + Kp * Np);
        hipLaunchKernelGGL(rowsum_s16_kernel, dim3((unsigned)((Np + 3) / 4)), dim3(256), 0, st, B_dev, ldb, (int)N,
                           (int)Np, (int)K, colsum);
        if (hipGetLastError() != hipSuccess) { delete d; return NGEMM_ERR_DEVICE; }
        if (Kp > 0) {
            const int64_t nslices = Kp / 64;                       // 32-element slices
            const int64_t nchunks = (Np / 32) * nslices * 64;
            const int64_t nwg = (nchunks + 255) / 256;
            if (nwg > 0x7fffffff) { delete d; return NGEMM_ERR_BAD_SHAPE; }
            hipLaunchKernelGGL(pack_b_s16_kernel, dim3((unsigned)nwg), dim3(256), 0, st, B_dev, ldb, (int)K, (int)N,
                               (int)nslices, nchunks, (uint8_t *)packed_dev);
            if (hipGetLastError() != hipSuccess) { delete d; return NGEMM_ERR_DEVICE; }
        }
    }
    *out = d;
    return NGEMM_OK;
}

ngemm_status ngemm_run_s16s16s32(ngemm_ctx *ctx, int64_t M, const int16_t *A_dev, int64_t lda, int32_t a_zero_point,
                                 const ngemm_packed_b *B, int32_t b_zero_point, int32_t *C_dev, int64_t ldc,
                                 void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    if (!ctx_ok(ctx) || !pack_ok(B) || B->elem_bytes != 2 || B->device != ctx->device) return NGEMM_ERR_INVALID_ARG;
    if (M < 0 || M > kMaxDim) return NGEMM_ERR_BAD_SHAPE;
    if (a_zero_point < -32768 || a_zero_point > 32767 || b_zero_point < -32768 || b_zero_point > 32767)
        return NGEMM_ERR_INVALID_ARG;
    if (M == 0 || B->N == 0) return NGEMM_OK;
    if (!C_dev || (!A_dev && B->K > 0)) return NGEMM_ERR_INVALID_ARG;
    if (lda < B->K || ldc < B->N) return NGEMM_ERR_BAD_SHAPE;
    // the kernel copies rows of A straight into LDS in 16-byte pieces
    if ((((uintptr_t)A_dev | (uintptr_t)(lda * 2)) & 15) != 0) return NGEMM_ERR_INVALID_ARG;
    if (B->K > 0) {
        if (!workspace_dev) return NGEMM_ERR_INVALID_ARG;
        if (workspace_bytes < rowsum_bytes(M)) return NGEMM_ERR_BUFFER_TOO_SMALL;
    }
    DeviceGuard g(ctx->device);
    if (!g.ok) return NGEMM_ERR_DEVICE;
    hipStream_t st = (hipStream_t)hip_stream;
    GemmParams p;
    std::memset(&p, 0, sizeof p);
    p.A = (const uint8_t *)A_dev;
    p.lda = lda * 2;
    p.Bp = B->data;
    p.colsum = (const int32_t *)(B->data + B->Kp * B->Np);
    p.C = C_dev;
    p.ldc = ldc;
    p.M = (int)M; p.N = (int)B->N; p.K = (int)B->K; p.Kp = (int)B->Kp;
    p.npanels = (int)(B->Np / 32);
    p.tiles_m = (int)((M + 127) / 128);
    p.tiles_n = (int)((B->N + 127) / 128);
    // sum (a-za)(b-zb) = sum (a-128)(b-128) + (128-za) colsum'[j] - (zb-128) rowsum'[i] - (zb-128)(128-za) K
    p.za_term = (uint32_t)(128 - a_zero_point);
    p.zb = (uint32_t)(b_zero_point - 128);
    p.kconst = 0u - (uint32_t)(b_zero_point - 128) * (uint32_t)(128 - a_zero_point) * (uint32_t)B->K;
    p.nxcd = ctx->num_xcd;
    if (B->K > 0) {
        int32_t *rs = (int32_t *)workspace_dev;
        hipLaunchKernelGGL(rowsum_s16_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, A_dev, lda, (int)M,
                           (int)M, (int)B->K, rs);
        if (hipGetLastError() != hipSuccess) return NGEMM_ERR_DEVICE;
        p.rowsum = rs;
    }
    const int ntiles = p.tiles_m * p.tiles_n, budget = workgroup_budget(ctx);
    hipLaunchKernelGGL(gemm_s16_tile_kernel, dim3((unsigned)(ntiles < budget ? ntiles : budget)), dim3(256),
                       S16Cfg::kLdsBytes, st, p);
    return hipGetLastError() == hipSuccess ? NGEMM_OK : NGEMM_ERR_DEVICE;
}

size_t ngemm_unpacked_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxDim) return 0;
    return (size_t)round_up((int64_t)ngemm_packed_b_bytes(K, N), 256) + rowsum_bytes(M > 0 ? M : 1);
}

ngemm_status ngemm_run_u8s8s32_unpacked(ngemm_ctx *ctx, int64_t M, int64_t N, int64_t K, const uint8_t *A_dev,
                                        int64_t lda, int32_t a_zero_point, const int8_t *B_dev, int64_t ldb,
                                        int32_t b_zero_point, int32_t *C_dev, int64_t ldc, void *workspace_dev,
                                        size_t workspace_bytes, void *hip_stream)
{
    if (!ctx_ok(ctx)) return NGEMM_ERR_INVALID_ARG;
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxDim) return NGEMM_ERR_BAD_SHAPE;
    if (a_zero_point < 0 || a_zero_point > 255 || b_zero_point < -128 || b_zero_point > 127)
        return NGEMM_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return NGEMM_OK;
    if (!C_dev || (K > 0 && (!A_dev || !B_dev))) return NGEMM_ERR_INVALID_ARG;
    if (lda < K || ldb < K || ldc < N) return NGEMM_ERR_BAD_SHAPE;
    if (!workspace_dev || ((uintptr_t)workspace_dev & 15u) != 0) return NGEMM_ERR_INVALID_ARG;
    if (workspace_bytes < ngemm_unpacked_workspace_bytes(M, N, K)) return NGEMM_ERR_BUFFER_TOO_SMALL;
    // Rows of both operands 16-byte aligned and an output that takes a tile kernel: no pack pass.
    // The tile kernel reads B from the caller's storage with the same copies as A; only the column
    // sums are computed beforehand (the row-sum kernel applied to B's [N x K] storage).
    int kernel = ctx->force_kernel == NGEMM_KERNEL_AUTO ? choose_kernel(ctx, M, N, K) : ctx->force_kernel;
    if (kernel == NGEMM_KERNEL_SPLIT_K)                                     // the K split reads a packed B only
        kernel = M <= kSkinnyMaxM ? NGEMM_KERNEL_SKINNY : NGEMM_KERNEL_TILE_64;
    const bool aligned = (((uintptr_t)A_dev | (uintptr_t)lda | (uintptr_t)B_dev | (uintptr_t)ldb) & 15) == 0;
    if (aligned && K > 0 && kernel != NGEMM_KERNEL_SKINNY) {
        DeviceGuard g(ctx->device);
        if (!g.ok) return NGEMM_ERR_DEVICE;
        hipStream_t st = (hipStream_t)hip_stream;
        ngemm_packed_b shape;                         // sizes only: nothing is packed
        shape.magic = kPackMagic; shape.device = ctx->device;
        shape.K = K; shape.N = N; shape.Kp = round_up(K, 64); shape.Np = round_up(N, 32);
        shape.data = nullptr; shape.bytes = 0; shape.b_shift = 0; shape.elem_bytes = 1;
        RunArgs a{M, A_dev, lda, a_zero_point, b_zero_point, &shape, C_dev, ldc, false, 1.0f, 0};
        GemmParams p = make_params(a, ctx->num_xcd);
        int32_t *colsum = (int32_t *)workspace_dev;
        int32_t *rowsum = (int32_t *)((uint8_t *)workspace_dev + round_up(shape.Np * 4, 256));
        p.Bp = nullptr;
        p.colsum = colsum;
        hipLaunchKernelGGL(rowsum_a_kernel, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, st, (const uint8_t *)B_dev,
                           ldb, (int)N, (int)K, 0u, colsum);
        if (hipGetLastError() != hipSuccess) return NGEMM_ERR_DEVICE;
        if (b_zero_point != 0) {
            hipLaunchKernelGGL(rowsum_a_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, A_dev, lda, (int)M,
                               (int)K, p.a_xor, rowsum);
            if (hipGetLastError() != hipSuccess) return NGEMM_ERR_DEVICE;
            p.rowsum = rowsum;
        }
        const RawB rawb{(const uint8_t *)B_dev, ldb};
        const int budget = workgroup_budget(ctx);
        hipError_t e;
        if (kernel == NGEMM_KERNEL_TILE_64) e = launch_tile_dma<64, 64, 2, 2>(p, false, budget, st, &rawb);
        else if (kernel == NGEMM_KERNEL_TILE_128) e = launch_tile_dma<128, 128, 2, 2>(p, false, budget, st, &rawb);
        else if (K >= X64Cfg::kMinK && x64_offsets_fit(256, lda, K) && x64_offsets_fit(256, ldb, K)) {
            p.tiles_m = (int)((M + 255) / 256);
            p.tiles_n = (int)((N + 255) / 256);
            const int ntiles = p.tiles_m * p.tiles_n;
            hipLaunchKernelGGL(gemm_tile_x64_kernel<true>, dim3((unsigned)(ntiles < budget ? ntiles : budget)), dim3(256),
                               X64Cfg::kLdsBytes, st, p, rawb);
            e = hipGetLastError();
        } else e = launch_tile_dma<256, 256, 2, 2, kStages256>(p, false, budget, st, &rawb);
        return e == hipSuccess ? NGEMM_OK : NGEMM_ERR_DEVICE;
    }
    const size_t pb = (size_t)round_up((int64_t)ngemm_packed_b_bytes(K, N), 256);
    ngemm_packed_b *h = nullptr;
    ngemm_status s = ngemm_pack_b(ctx, K, N, B_dev, ldb, workspace_dev, pb, hip_stream, &h);
    if (s != NGEMM_OK) return s;
    s = ngemm_run_u8s8s32(ctx, M, A_dev, lda, a_zero_point, h, b_zero_point, C_dev, ldc,
                          (uint8_t *)workspace_dev + pb, workspace_bytes - pb, hip_stream);
    ngemm_packed_b_free(h);      // the descriptor only: the kernels already hold the device addresses
    return s;
}

size_t ngemm_batched_workspace_bytes(int count, const ngemm_problem *problems)
{
    (void)count;
    (void)problems;
    return 0;                    // the grouped kernels form the row sums they need themselves
}

ngemm_status ngemm_run_batched_u8s8s32(ngemm_ctx *ctx, int count, const ngemm_problem *problems,
                                       void *workspace_dev, size_t workspace_bytes, void *hip_stream)
{
    (void)workspace_dev;
    (void)workspace_bytes;
    if (!ctx_ok(ctx) || count < 0 || (count > 0 && !problems)) return NGEMM_ERR_INVALID_ARG;
    for (int t = 0; t < count; ++t) {
        const ngemm_problem &q = problems[t];
        RunArgs a{q.M, q.A_dev, q.lda, q.a_zero_point, q.b_zero_point, q.B, q.C_dev, q.ldc, false, 1.0f, 0};
        int kernel;
        ngemm_status s = validate_run(ctx, a, &kernel);
        if (s != NGEMM_OK) return s;
    }
    DeviceGuard g(ctx->device);
    if (!g.ok) return NGEMM_ERR_DEVICE;
    hipStream_t st = (hipStream_t)hip_stream;

    // Grouped launches: the members' parameters ride in the kernel argument block, up to
    // kGroupMax per launch; one grid covers the panels of a group's skinny members and the 64 x 64
    // tiles of its members with M > 32.  Launch count, not arithmetic, is what a batch of small odd
    // shapes costs (and two launches run one after the other, however few compute units each can use),
    // so there is no launch for the row sums either: both bodies form them from the A fragments they
    // read anyway.
    GroupParams grp;
    grp.count = 0;
    grp.nxcd = ctx->num_xcd;
    grp.first_tile = 0;
    grp.unit_start[0] = 0;
    const int cus = ctx->num_cus > 0 ? ctx->num_cus : 256;
    using TCfg = TileCfg<64, 64, 2, 2, 64>;
    auto flush = [&]() -> hipError_t {
        if (grp.count == 0) return hipSuccess;
        const unsigned grid = (unsigned)grp.unit_start[grp.count];
        if (grid > 0) {
            if (grp.first_tile == grp.count) {
                // skinny members only.  Wavefronts per panel: eight hide latency when the panels are
                // few; with several panels per compute unit anyway, fewer wavefronts with more
                // fragments each spend less on the final sum across wavefronts
                const unsigned nw = grid >= 8u * cus ? 2 : (grid >= 4u * cus ? 4 : 8);
                hipLaunchKernelGGL(gemm_group_skinny_kernel, dim3(grid), dim3(64 * nw), (size_t)(nw * 16 * 64 * 4), st, grp);
            } else {
                const size_t lds = std::max((size_t)TCfg::kLdsBytes, (size_t)(4 * 16 * 64 * 4));
                hipLaunchKernelGGL((gemm_group_kernel<64, 64, 2, 2, 64>), dim3(grid), dim3(256), lds, st, grp);
            }
        }
        grp.count = 0;
        grp.first_tile = 0;
        grp.unit_start[0] = 0;
        return hipGetLastError();
    };
    // The streaming kernel's group: up to kStreamGroupMax members; unit_start collects panel counts
    // until the launch, which turns them into chunks of panels sized for the whole group.
    StreamGroupParams stream;
    stream.count = 0;
    stream.nxcd = ctx->num_xcd;
    stream.unit_start[0] = 0;
    auto flush_stream = [&]() -> hipError_t {
        if (stream.count == 0) return hipSuccess;
        const int chunk = stream_chunk(stream.unit_start[stream.count], cus);
        int lds = 0, units = 0;
        for (int t = 0; t < stream.count; ++t) {
            const int panels = stream.unit_start[t + 1] - stream.unit_start[t];
            stream.unit_start[t] = units;
            units += (panels + chunk - 1) / chunk;
            lds = std::max(lds, stream_launch_lds((int)(stream.mzz[t] & 63u), round_up(stream.K[t], 64), chunk));
        }
        stream.unit_start[stream.count] = units;
        stream.chunk = chunk;
        stream.lds_bytes = lds;
        if (units > 0)
            hipLaunchKernelGGL(gemm_group_stream_kernel, dim3((unsigned)units), dim3(kStreamWaves * 64), (size_t)lds, st, stream);
        stream.count = 0;
        stream.unit_start[0] = 0;
        return hipGetLastError();
    };
    auto push_stream = [&](const GemmParams &p) {
        const int t = stream.count;
        stream.A[t] = p.A; stream.Bp[t] = p.Bp; stream.C[t] = p.C;
        stream.lda[t] = (int)p.lda; stream.ldc[t] = (int)p.ldc;
        stream.N[t] = p.N; stream.K[t] = p.K;
        stream.mzz[t] = stream_pack_mzz(p.M, p.za_term, p.zb);
        stream.unit_start[t + 1] = stream.unit_start[t] + p.npanels;
        ++stream.count;
    };
    auto push = [&](const GemmParams &p, int64_t units, bool is_skinny) {
        GroupMember &m = grp.prob[grp.count];        // the rest is rebuilt on the device
        m.A = p.A; m.Bp = p.Bp; m.C = p.C;
        m.lda = p.lda; m.ldc = p.ldc;
        m.M = p.M; m.N = p.N; m.K = p.K;
        m.za_term = (int16_t)(int32_t)p.za_term;     // 128 - za and zb: small signed values
        m.zb = (int16_t)(int32_t)p.zb;
        grp.unit_start[grp.count + 1] = grp.unit_start[grp.count] + (int)units;
        ++grp.count;
        if (is_skinny) grp.first_tile = grp.count;   // the skinny members of a group come first
    };
    constexpr int64_t kMaxGrid = 1 << 30;
    // Members with the longest K first: a workgroup's time grows with K, and the grid is handed out
    // in order, so the long ones start at once and the many short ones fill in around them.
    struct Pending { GemmParams p; int64_t units; };
    std::vector<Pending> tile_members, skinny_members, stream_members;
    try {
        tile_members.reserve((size_t)count);
        skinny_members.reserve((size_t)count);
        stream_members.reserve((size_t)count);
    } catch (...) {
        return NGEMM_ERR_DEVICE;                   // out of host memory; nothing was launched
    }
    for (int t = 0; t < count; ++t) {
        const ngemm_problem &q = problems[t];
        if (q.M == 0 || q.B->N == 0) continue;
        RunArgs a{q.M, q.A_dev, q.lda, q.a_zero_point, q.b_zero_point, q.B, q.C_dev, q.ldc, false, 1.0f, 0};
        const GemmParams p = make_params(a, ctx->num_xcd);
        if (q.M <= kSkinnyMaxM && stream_can_serve(p.M, p.Kp) && q.lda <= 0x7fffffff && q.ldc <= 0x7fffffff)
            stream_members.push_back(Pending{p, p.npanels});
        else if (q.M <= kSkinnyMaxM)
            skinny_members.push_back(Pending{p, p.npanels});
        else
            tile_members.push_back(Pending{p, (int64_t)((p.M + 63) / 64) * ((p.N + 63) / 64)});
    }
    // The streaming kernel pays off once its members have panels for every compute unit several
    // times over; a few panels are better served by the kernel that splits K over wavefronts.
    int64_t stream_panels = 0;
    for (const Pending &m : stream_members) stream_panels += m.units;
    if (stream_panels < 4 * (int64_t)cus) {
        skinny_members.insert(skinny_members.end(), stream_members.begin(), stream_members.end());
        stream_members.clear();
    }
    auto longer_k = [](const Pending &x, const Pending &y) { return x.p.K > y.p.K; };
    std::stable_sort(tile_members.begin(), tile_members.end(), longer_k);
    std::stable_sort(skinny_members.begin(), skinny_members.end(), longer_k);
    // skinny members first: in a grid that also holds tiles they start with the launch (the longest
    // of them take as long as all the tiles together)
    for (const Pending &m : skinny_members) {
        if (grp.count == kGroupMax || grp.unit_start[grp.count] + m.units > kMaxGrid)
            if (flush() != hipSuccess) return NGEMM_ERR_DEVICE;
        push(m.p, m.units, true);
    }
    for (const Pending &m : tile_members) {
        if (grp.count == kGroupMax || grp.unit_start[grp.count] + m.units > kMaxGrid)
            if (flush() != hipSuccess) return NGEMM_ERR_DEVICE;
        push(m.p, m.units, false);
    }
    for (const Pending &m : stream_members) {
        if (stream.count == kStreamGroupMax || stream.unit_start[stream.count] + m.units > kMaxGrid)
            if (flush_stream() != hipSuccess) return NGEMM_ERR_DEVICE;
        push_stream(m.p);
    }
    if (flush() != hipSuccess) return NGEMM_ERR_DEVICE;
    if (flush_stream() != hipSuccess) return NGEMM_ERR_DEVICE;
    return NGEMM_OK;
}

}  // extern "C"
