// Diagnostics: how a SIMD of this GPU overlaps matrix and vector instructions.  The layout of the
// backward kernels follows from what this measures (see lp_mfma_bwd_ws.h); not part of the method.
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
