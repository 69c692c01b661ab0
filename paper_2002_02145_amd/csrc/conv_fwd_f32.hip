// fp32 kernel shapes of the batch-reduce-GEMM convolution and their launcher.
#include "conv_fwd_kernel.h"

namespace ps {

//                       KT   MT  WK WM G
static const ShapeEntry kF32Shapes[] = {
    PS_F32_SHAPE(128, 128, 2, 2, 1), PS_F32_SHAPE(128, 128, 2, 2, 2), PS_F32_SHAPE(128, 128, 2, 2, 4),
    PS_F32_SHAPE(64, 128, 2, 2, 1),  PS_F32_SHAPE(64, 128, 2, 2, 2),  PS_F32_SHAPE(64, 128, 2, 2, 4),
    PS_F32_SHAPE(64, 256, 1, 4, 1),  PS_F32_SHAPE(64, 256, 1, 4, 2),
    PS_F32_SHAPE(128, 64, 2, 2, 1),  PS_F32_SHAPE(128, 64, 2, 2, 2),  PS_F32_SHAPE(128, 64, 2, 2, 4),
    PS_F32_SHAPE(64, 64, 2, 2, 1),   PS_F32_SHAPE(64, 64, 2, 2, 2),   PS_F32_SHAPE(64, 64, 2, 2, 4),
    PS_F32_SHAPE(32, 128, 1, 4, 2),  PS_F32_SHAPE(32, 128, 1, 4, 4),
    PS_F32_SHAPE(32, 64, 1, 2, 2),   PS_F32_SHAPE(32, 64, 1, 2, 4),
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

}  // namespace ps
