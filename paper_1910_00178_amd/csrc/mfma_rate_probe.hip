// Measurement aid for bench.py, not part of the GEMM library: the rate the int8 matrix pipe
// sustains by itself, in a loop of nothing but matrix instructions on register operands (no LDS,
// no memory traffic), for both instruction shapes and for random or constant operand values.
// On random operands the chip runs at its power cap, and this rate, not the published peak, is
// what a GEMM kernel could approach on such data.
//
// extern "C" int ngemm_probe_mfma_rate(int shape, int random_operands, double *tops_out)
//   shape 0: v_mfma_i32_16x16x64_i8, 1: v_mfma_i32_32x32x32_i8; returns 0 on success, a HIP error
//   code otherwise.  Uses the current device and the null stream; allocates and frees 17 MiB.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <vector>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kSrcEntries = 1 << 20;      // 16-byte operand fragments to pick from
constexpr int kWorkgroups = 256, kIters = 20000;

// One wavefront per SIMD, 256 accumulator registers per lane, as in the 256 x 256 GEMM kernel: per
// iteration 2 * 128 * 128 * 64 operations per wavefront in either shape.
template <int SHAPE>
__global__ __launch_bounds__(256) void mfma_loop(const v4i *__restrict__ src, int *__restrict__ dst, int iters)
{
    const int tid = threadIdx.x + blockIdx.x * 256;
    v4i a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = src[(tid * 16 + i) & (kSrcEntries - 1)];
        b[i] = src[(tid * 16 + 8 + i) & (kSrcEntries - 1)];
    }
    int sum = 0;
    if (SHAPE == 0) {
        v4i acc[8][8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i][j] = v4i{0, 0, 0, 0};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) sum += acc[i][j].x + acc[i][j].y + acc[i][j].z + acc[i][j].w;
    } else {
        v16i acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[2 * i + h], b[2 * j + h], acc[i][j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
    }
    dst[tid] = sum;
}

void launch(int shape, const v4i *src, int *dst)
{
    if (shape == 0) hipLaunchKernelGGL(mfma_loop<0>, dim3(kWorkgroups), dim3(256), 0, 0, src, dst, kIters);
    else hipLaunchKernelGGL(mfma_loop<1>, dim3(kWorkgroups), dim3(256), 0, 0, src, dst, kIters);
}

}  // namespace

extern "C" int ngemm_probe_mfma_rate(int shape, int random_operands, double *tops_out)
{
    if (!tops_out || shape < 0 || shape > 1) return (int)hipErrorInvalidValue;
    *tops_out = 0.0;
    std::vector<uint32_t> h((size_t)kSrcEntries * 4);
    uint64_t s = 0x9E3779B97F4A7C15ull;                   // splitmix64: any fixed random bytes will do
    for (uint32_t &x : h) {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        x = random_operands ? (uint32_t)(z ^ (z >> 31)) : 0x01010101u;
    }
    v4i *src = nullptr;
    int *dst = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipMalloc(&src, h.size() * 4);
    if (e == hipSuccess) e = hipMalloc(&dst, (size_t)kWorkgroups * 256 * sizeof(int));
    if (e == hipSuccess) e = hipMemcpy(src, h.data(), h.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    const int warm = 3, timed = 5;                        // about 20 ms per launch: the clock has settled
    if (e == hipSuccess) {
        for (int w = 0; w < warm; ++w) launch(shape, src, dst);
        e = hipEventRecord(e0, 0);
        for (int w = 0; w < timed; ++w) launch(shape, src, dst);
        if (e == hipSuccess) e = hipEventRecord(e1, 0);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipGetLastError();
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess && ms > 0.0f)
            *tops_out = (double)timed * kWorkgroups * 4 * (double)kIters * 2.0 * 128 * 128 * 64 / (ms * 1e-3) / 1e12;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (src) (void)hipFree(src);
    if (dst) (void)hipFree(dst);
    return (int)e;
}
