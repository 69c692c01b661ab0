// Measurement aid, not part of the convolution path: a loop of independent MFMAs with no operand traffic, so that a
// report can put the rate the matrix cores sustain on this device next to the published peak.
#include <hip/hip_runtime.h>

#include "polysci_conv.h"
#include "ps_internal.h"

namespace ps {
namespace {

typedef float floatx4_p __attribute__((ext_vector_type(4)));
typedef float floatx16_p __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_p __attribute__((ext_vector_type(8)));

constexpr int kProbeAcc = 4;     // independent accumulators per wave
constexpr int kProbeUnroll = 8;  // MFMAs per accumulator per loop iteration

__global__ __launch_bounds__(256) void probe_mfma_f32_kernel(float *sink, int iters, float a0, float b0)
{
    floatx4_p acc[kProbeAcc];
    for (int i = 0; i < kProbeAcc; ++i) acc[i] = floatx4_p{0.f, 0.f, 0.f, 0.f};
    const float a = a0 + threadIdx.x, b = b0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
            for (int i = 0; i < kProbeAcc; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < kProbeAcc; ++i)
        for (int r = 0; r < 4; ++r) s += acc[i][r];
    if (s == 12345.678f) sink[threadIdx.x] = s;  // keeps the loop alive; never true for the arguments passed
}

__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(float *sink, int iters, float a0)
{
    floatx16_p acc[kProbeAcc];
    for (int i = 0; i < kProbeAcc; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    bf16x8_p a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(a0 + (float)(threadIdx.x & 7) + i);
        b[i] = (__bf16)(a0 * i);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
            for (int i = 0; i < kProbeAcc; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < kProbeAcc; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 12345.678f) sink[threadIdx.x] = s;
}

}  // namespace
}  // namespace ps

using namespace ps;

extern "C" int ps_probe_mfma(int dtype, int iters, void *sink, double *flop, void *stream)
{
    if (!sink || iters <= 0 || iters > (1 << 24) || (dtype != PS_F32 && dtype != PS_BF16)) return PS_EINVAL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return hip_status(hipGetLastError());
    const unsigned grid = (unsigned)cus * 4;  // 16 waves per compute unit, 4 per SIMD
    const double mfmas = (double)grid * 4.0 * iters * kProbeUnroll * kProbeAcc;
    if (dtype == PS_F32) {
        hipLaunchKernelGGL(probe_mfma_f32_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (float *)sink, iters,
                           1.0f, 0.5f);
        if (flop) *flop = mfmas * 2.0 * 16 * 16 * 4;
    } else {
        hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (float *)sink, iters,
                           1.0f);
        if (flop) *flop = mfmas * 2.0 * 32 * 32 * 16;
    }
    return hip_status(hipGetLastError());
}
