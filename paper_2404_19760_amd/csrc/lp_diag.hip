// Diagnostics: how a SIMD of this GPU overlaps matrix and vector instructions (the layout of the
// backward kernels follows from what this measures, see lp_mfma_bwd_ws.h), and how many 64-byte
// lines of fp32 atomic adds the chip retires per second (the ceiling of the gradient scatter).  Not
// part of the method.
#include <hip/hip_runtime.h>

#include "lightplane.h"
#include "lp_mfma.h"

namespace lp {

namespace {

constexpr int kDiagBlocks = 256;   // one workgroup per compute unit
constexpr int kDiagIters = 20000;

// One wave per SIMD: a loop of four independent 32x32x16 bf16 products, each followed by K
// independent vector multiply-adds.
template <int K>
__global__ __launch_bounds__(256) void diag_same_wave_kernel(float* out, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x + i); b[i] = (__bf16)1.0f; }
    f32x16 acc[4];
    for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    float v[16];
    for (int i = 0; i < 16; ++i) v[i] = threadIdx.x * 0.001f + i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < K; ++i) v[i] = v[i] * 1.0001f + 0.5f;
            __builtin_amdgcn_sched_barrier(0);   // keeps the vector work between the products
        }
    }
    float s = 0.f;
    for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) s += acc[j][i];
    for (int i = 0; i < 16; ++i) s += v[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Eight waves per workgroup, two per SIMD.  Waves of the "matrix" role issue 8 products per
// iteration, waves of the "vector" role 64 multiply-adds (256 cycles each on their own).
// pairing 0: waves 0..3 matrix, 4..7 vector; pairing 1: even waves matrix, odd waves vector.
// what: bit 0 = the matrix role works, bit 1 = the vector role works.
template <int PAIRING>
__global__ __launch_bounds__(512) void diag_two_waves_kernel(float* out, int iters, int what)
{
    const int wave = threadIdx.x >> 6;
    const bool matrix = PAIRING == 0 ? wave < 4 : (wave & 1) == 0;
    float s = 0.f;
    if (matrix) {
        if (what & 1) {
            bf16x8 a, b;
            for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x + i); b[i] = (__bf16)1.0f; }
            f32x16 acc[4];
            for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
            for (int it = 0; it < iters; ++it) {
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
            }
            for (int j = 0; j < 4; ++j) for (int i = 0; i < 16; ++i) s += acc[j][i];
        }
    } else if (what & 2) {
        float v[16];
        for (int i = 0; i < 16; ++i) v[i] = threadIdx.x * 0.001f + i;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = v[i] * 1.0001f + 0.5f;
        }
        for (int i = 0; i < 16; ++i) s += v[i];
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Every wave adds 1.0f to LINES whole 64-byte lines per instruction (16 lanes per line, the other
// lanes idle), `iters` times; the lines are drawn by a hash from the n_lines lines of `buf`, or walk
// through neighbouring lines like a ray through a grid.  All addresses are below 16 n_lines floats.
__device__ __forceinline__ unsigned diag_mix(unsigned x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

template <int LINES>
__global__ __launch_bounds__(256) void diag_atomic_kernel(float* buf, unsigned n_lines, int iters, int local)
{
    static_assert(LINES == 1 || LINES == 2 || LINES == 4, "16 lanes per line");
    const unsigned wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
    if (lane >= 16u * LINES) return;
    const unsigned start = diag_mix(wave * 977u + 13u) % n_lines;
    for (int i = 0; i < iters; ++i) {
        const unsigned l = local ? (start + (unsigned)i * 3u + (lane >> 4)) % n_lines
                                 : diag_mix(wave * 7919u + (unsigned)i * 4u + (lane >> 4)) % n_lines;
        atomicAdd(buf + (size_t)l * 16 + (lane & 15), 1.0f);
    }
}

template <class Launch>
hipError_t timed(Launch launch, hipStream_t stream, float* ms)
{
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    launch(10);   // warm-up
    (void)hipEventRecord(e0, stream);
    launch(kDiagIters);
    (void)hipEventRecord(e1, stream);
    e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return e;
}

}  // namespace

}  // namespace lp

extern "C" lp_status lp_diag_coexecution(float* ns_per_iteration, void* stream)
{
    using namespace lp;
    if (!ns_per_iteration) return LP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    float* out = nullptr;
    if (hipMalloc(&out, (size_t)kDiagBlocks * 512 * sizeof(float)) != hipSuccess) return LP_ERR_HIP;
    hipError_t e = hipSuccess;
    int slot = 0;
    auto record = [&](float ms, double per) { ns_per_iteration[slot++] = (float)(ms * 1e6 / per); };
    float ms = 0.f;
#define LP_SAME_WAVE(K)                                                                                          \
    if (e == hipSuccess) {                                                                                       \
        e = timed([&](int it) { hipLaunchKernelGGL(diag_same_wave_kernel<K>, dim3(kDiagBlocks), dim3(256), 0, s, out, it); }, s, &ms); \
        record(ms, 4.0 * kDiagIters);                                                                            \
    }
    LP_SAME_WAVE(0) LP_SAME_WAVE(4) LP_SAME_WAVE(8) LP_SAME_WAVE(12)
#undef LP_SAME_WAVE
#define LP_TWO_WAVES(P, W)                                                                                       \
    if (e == hipSuccess) {                                                                                       \
        e = timed([&](int it) { hipLaunchKernelGGL(diag_two_waves_kernel<P>, dim3(kDiagBlocks), dim3(512), 0, s, out, it, W); }, s, &ms); \
        record(ms, (double)kDiagIters);                                                                          \
    }
    LP_TWO_WAVES(0, 1) LP_TWO_WAVES(0, 2) LP_TWO_WAVES(0, 3) LP_TWO_WAVES(1, 1) LP_TWO_WAVES(1, 2) LP_TWO_WAVES(1, 3)
#undef LP_TWO_WAVES
    (void)hipFree(out);
    return e == hipSuccess ? LP_OK : LP_ERR_HIP;
}

extern "C" lp_status lp_diag_atomic_rate(float* lines_per_second, void* stream)
{
    using namespace lp;
    if (!lines_per_second) return LP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    constexpr unsigned kSmall = 1u << 12, kLarge = 1u << 22;   // 256 KiB (inside one L2) and 256 MiB of lines
    constexpr int kBlocks = 2048, kIters = 2000;
    float* buf = nullptr;
    if (hipMalloc(&buf, (size_t)kLarge * 64) != hipSuccess) return LP_ERR_HIP;
    hipError_t e = hipMemsetAsync(buf, 0, (size_t)kLarge * 64, s);
    int slot = 0;
    auto run = [&](auto kernel, int lines, unsigned n_lines, int local) {
        if (e != hipSuccess) return;
        hipEvent_t e0, e1;
        if ((e = hipEventCreate(&e0)) != hipSuccess) return;
        if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return; }
        hipLaunchKernelGGL(kernel, dim3(kBlocks), dim3(256), 0, s, buf, n_lines, 8, local);   // warm-up
        (void)hipEventRecord(e0, s);
        hipLaunchKernelGGL(kernel, dim3(kBlocks), dim3(256), 0, s, buf, n_lines, kIters, local);
        (void)hipEventRecord(e1, s);
        e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipGetLastError();
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        (void)hipEventDestroy(e0);
        (void)hipEventDestroy(e1);
        lines_per_second[slot++] = ms > 0.f ? (float)((double)kBlocks * 4 * kIters * lines / (ms * 1e-3)) : 0.f;
    };
    run(diag_atomic_kernel<4>, 4, kLarge, 0);
    run(diag_atomic_kernel<2>, 2, kLarge, 0);
    run(diag_atomic_kernel<1>, 1, kLarge, 0);
    run(diag_atomic_kernel<4>, 4, kSmall, 0);
    run(diag_atomic_kernel<4>, 4, kLarge, 1);
    run(diag_atomic_kernel<4>, 4, kSmall, 1);
    (void)hipFree(buf);
    return e == hipSuccess ? LP_OK : LP_ERR_HIP;
}
