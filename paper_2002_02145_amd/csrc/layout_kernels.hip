// Layout transforms between plain (NCHW / KCRS / NKPQ) and blocked tensors.
//
// The blocked layouts are the ones fixed by the index expressions of the paper's Fig. 4
// (Section 5): input[img][ifm_tile][ij][ii][ifm], filter[ofm_tile][ifm_tile][kj][ki][ifm][ofm],
// output[img][ofm_tile][oj][oi][ofm] with a channel block of 16 (Section 5.1).  Every kernel
// here is a pure permutation of bit patterns (plus +0.0 fill of channel lanes past C), so it
// is generic over the element size and bit-exact.
//
// All of them are HBM-bound copies.  Activations go through an LDS transpose so that both
// the read side (a run of pixels of one channel) and the write side (16 channels of a run of
// pixels) are contiguous per wavefront.
#include "ps_internal.h"

namespace ps {
namespace {

constexpr int kPix = 256;  // pixels per workgroup tile (= threads per workgroup)

// plain [n][c][hw] -> blocked [n][cb][hw][16]
template <typename T>
__global__ __launch_bounds__(kPix) void act_to_blocked_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                              int C, int Cb, int HW)
{
    __shared__ T tile[kBlock][kPix + 1];
    const int t = threadIdx.x;
    const int n = blockIdx.y / Cb, cb = blockIdx.y % Cb;
    const int pix0 = blockIdx.x * kPix;
    const int npix = min(kPix, HW - pix0);
#pragma unroll
    for (int c = 0; c < kBlock; ++c) {
        const int ch = cb * kBlock + c;
        T v = 0;
        if (ch < C && t < npix) v = src[((size_t)n * C + ch) * HW + pix0 + t];
        tile[c][t] = v;
    }
    __syncthreads();
    T *out = dst + (((size_t)n * Cb + cb) * HW + pix0) * kBlock;
    const int nel = npix * kBlock;
#pragma unroll
    for (int i = 0; i < kBlock; ++i) {
        const int e = i * kPix + t;
        if (e < nel) out[e] = tile[e % kBlock][e / kBlock];
    }
}

// blocked [n][cb][hw][16] -> plain [n][c][hw]
template <typename T>
__global__ __launch_bounds__(kPix) void blocked_to_act_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                              int C, int Cb, int HW)
{
    __shared__ T tile[kBlock][kPix + 1];
    const int t = threadIdx.x;
    const int n = blockIdx.y / Cb, cb = blockIdx.y % Cb;
    const int pix0 = blockIdx.x * kPix;
    const int npix = min(kPix, HW - pix0);
    const T *in = src + (((size_t)n * Cb + cb) * HW + pix0) * kBlock;
    const int nel = npix * kBlock;
#pragma unroll
    for (int i = 0; i < kBlock; ++i) {
        const int e = i * kPix + t;
        if (e < nel) tile[e % kBlock][e / kBlock] = in[e];
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kBlock; ++c) {
        const int ch = cb * kBlock + c;
        if (ch < C && t < npix) dst[((size_t)n * C + ch) * HW + pix0 + t] = tile[c][t];
    }
}

// plain [k][c][rs] <-> blocked [kb][cb][rs][16 c][16 k]; one thread per blocked element.
// Filters are at most a few MB and transformed once per layer, so this stays a plain gather.
// With kPacked8 (2-byte elements) the block is [c/8][16 k][8 c]: the 8 input channels one bf16 MFMA
// lane consumes are contiguous.
template <typename T, bool kToBlocked, bool kPacked8>
__global__ __launch_bounds__(256) void filt_kernel(const T *__restrict__ src, T *__restrict__ dst, int C,
                                                   int Cb, int RS, size_t nblk)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= nblk) return;
    const int in_blk = (int)(e % (kBlock * kBlock));
    const int kk = kPacked8 ? (in_blk >> 3) & 15 : in_blk & 15;
    const int cc = kPacked8 ? (in_blk >> 7) * 8 + (in_blk & 7) : in_blk >> 4;
    size_t rest = e / (kBlock * kBlock);
    const int rs = rest % RS;
    rest /= RS;
    const int cb = rest % Cb;
    const int kb = rest / Cb;
    const int c = cb * kBlock + cc, k = kb * kBlock + kk;
    if (kToBlocked) {
        T v = 0;
        if (c < C) v = src[((size_t)k * C + c) * RS + rs];
        dst[e] = v;
    } else {
        if (c < C) dst[((size_t)k * C + c) * RS + rs] = src[e];
    }
}

template <typename T>
int run_act(bool to_blocked, const void *src, void *dst, int N, int C, int HW, hipStream_t st)
{
    const int Cb = (C + kBlock - 1) / kBlock;
    dim3 grid((HW + kPix - 1) / kPix, (unsigned)(N * Cb));
    if ((long long)N * Cb > 65535) return PS_EUNSUPPORTED;
    if (to_blocked)
        hipLaunchKernelGGL(act_to_blocked_kernel<T>, grid, dim3(kPix), 0, st, (const T *)src, (T *)dst, C, Cb, HW);
    else
        hipLaunchKernelGGL(blocked_to_act_kernel<T>, grid, dim3(kPix), 0, st, (const T *)src, (T *)dst, C, Cb, HW);
    return hip_status(hipGetLastError());
}

template <typename T>
int run_filt(bool to_blocked, const void *src, void *dst, const Dims &dm, hipStream_t st)
{
    const size_t nblk = (size_t)dm.Kb * dm.Cb * dm.R * dm.S * kBlock * kBlock;
    const unsigned grid = (unsigned)((nblk + 255) / 256);
    if (to_blocked)
        hipLaunchKernelGGL((filt_kernel<T, true, sizeof(T) == 2>), dim3(grid), dim3(256), 0, st, (const T *)src,
                           (T *)dst, dm.C, dm.Cb, dm.R * dm.S, nblk);
    else
        hipLaunchKernelGGL((filt_kernel<T, false, sizeof(T) == 2>), dim3(grid), dim3(256), 0, st, (const T *)src,
                           (T *)dst, dm.C, dm.Cb, dm.R * dm.S, nblk);
    return hip_status(hipGetLastError());
}

int check(const ps_conv_desc *d, const void *a, const void *b, Dims *dm)
{
    int rc = make_dims(d, dm);
    if (rc != PS_OK) return rc;
    if (!a || !b || !aligned16(a) || !aligned16(b)) return PS_EINVAL;
    return PS_OK;
}

}  // namespace
}  // namespace ps

using namespace ps;

extern "C" int ps_nchw_to_blocked(const ps_conv_desc *d, const void *nchw, void *blk, void *stream)
{
    Dims dm;
    int rc = check(d, nchw, blk, &dm);
    if (rc != PS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dm.es == 4 ? run_act<uint32_t>(true, nchw, blk, dm.N, dm.C, dm.H * dm.W, st)
                      : run_act<uint16_t>(true, nchw, blk, dm.N, dm.C, dm.H * dm.W, st);
}

extern "C" int ps_blocked_to_nchw(const ps_conv_desc *d, const void *blk, void *nchw, void *stream)
{
    Dims dm;
    int rc = check(d, blk, nchw, &dm);
    if (rc != PS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dm.es == 4 ? run_act<uint32_t>(false, blk, nchw, dm.N, dm.C, dm.H * dm.W, st)
                      : run_act<uint16_t>(false, blk, nchw, dm.N, dm.C, dm.H * dm.W, st);
}

extern "C" int ps_blocked_to_nkpq(const ps_conv_desc *d, const void *oblk, void *nkpq, void *stream)
{
    Dims dm;
    int rc = check(d, oblk, nkpq, &dm);
    if (rc != PS_OK) return rc;
    return run_act<uint32_t>(false, oblk, nkpq, dm.N, dm.K, dm.P * dm.Q, (hipStream_t)stream);
}

extern "C" int ps_kcrs_to_blocked(const ps_conv_desc *d, const void *kcrs, void *wblk, void *stream)
{
    Dims dm;
    int rc = check(d, kcrs, wblk, &dm);
    if (rc != PS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dm.es == 4 ? run_filt<uint32_t>(true, kcrs, wblk, dm, st) : run_filt<uint16_t>(true, kcrs, wblk, dm, st);
}

extern "C" int ps_blocked_to_kcrs(const ps_conv_desc *d, const void *wblk, void *kcrs, void *stream)
{
    Dims dm;
    int rc = check(d, wblk, kcrs, &dm);
    if (rc != PS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dm.es == 4 ? run_filt<uint32_t>(false, wblk, kcrs, dm, st) : run_filt<uint16_t>(false, wblk, kcrs, dm, st);
}
