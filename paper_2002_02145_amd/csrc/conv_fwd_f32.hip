// fp32 kernel shapes of the batch-reduce-GEMM convolution and their launcher.
#include "conv_fwd_kernel.h"
#include "conv_fwd_f32_n16.h"
#include "conv_fwd_f32_n16_kloop.h"

namespace ps {

#define PS_TABLE_ROW(KT, MT, WK, WM, NBUF) PS_F32_SHAPE(KT, MT, WK, WM, NBUF),
static const ShapeEntry kF32Shapes[] = {
    PS_F32_SHAPE_LIST(PS_TABLE_ROW)
    // 64 channels x MT pixels on 16x16x4 MFMA tiles: pixel tiles in steps of 16, for even division over the chip
#define PS_TABLE_ROW_N16(MT, NBUF) PS_F32_N16_SHAPE(MT, NBUF),
    PS_F32_N16_SHAPE_LIST(PS_TABLE_ROW_N16)
    PS_F32_N16_KLOOP_SHAPE(48), PS_F32_N16_KLOOP_SHAPE(96), PS_F32_N16_KLOOP_SHAPE(176),
};

const ShapeEntry *f32_shapes(int *count)
{
    *count = (int)(sizeof(kF32Shapes) / sizeof(kF32Shapes[0]));
    return kF32Shapes;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(floatx4 *p, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) p[i] = floatx4{0.f, 0.f, 0.f, 0.f};
}

// n must be a multiple of 4 floats (blocked outputs are multiples of 16).
int launch_fill_zero(float *p, size_t n, hipStream_t stream)
{
    const size_t n4 = n / 4;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream,
                       reinterpret_cast<floatx4 *>(p), n4);
    return hip_status(hipGetLastError());
}

// out = epilogue(sum over planes of partial[plane][.]); n4 = out elements / 4 (blocked outputs are multiples of 16).
// The output is [N][Kb][PQ][16 k]: element e belongs to channel ((e / (16 * PQ)) % Kb) * 16 + e % 16.
__global__ __launch_bounds__(256) void reduce_planes_kernel(const floatx4 *__restrict__ partial, void *__restrict__ out,
                                                            size_t n4, int planes, const float *__restrict__ bias,
                                                            int epi, unsigned pq4, int Kb)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    floatx4 s = partial[i];
    for (int p = 1; p < planes; ++p) s += partial[(size_t)p * n4 + i];
    if (epi & 1) {
        const int kb = (int)((i / pq4) % (unsigned)Kb);  // pq4 = 16 * PQ / 4 groups of four per channel-block plane
        s += *reinterpret_cast<const floatx4 *>(bias + kb * 16 + (int)(i & 3) * 4);
    }
    if (epi & 2)
        for (int k = 0; k < 4; ++k) s[k] = fmaxf(s[k], 0.f);
    if (epi & 4) {
        const uintx2_t h = {pack_bf16(s[0], s[1]), pack_bf16(s[2], s[3])};
        reinterpret_cast<uintx2_t *>(out)[i] = h;
    } else {
        reinterpret_cast<floatx4 *>(out)[i] = s;
    }
}

int launch_reduce_planes(const float *partial, void *out, size_t n, int planes, const float *bias, int epi, int PQ, int Kb,
                         hipStream_t stream)
{
    const size_t n4 = n / 4;
    hipLaunchKernelGGL(reduce_planes_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, stream,
                       reinterpret_cast<const floatx4 *>(partial), out, n4, planes, bias, epi, (unsigned)(4 * PQ), Kb);
    return hip_status(hipGetLastError());
}

}  // namespace ps
