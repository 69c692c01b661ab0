// Layout transforms between plain (NCHW / KCRS / NKPQ) and blocked tensors.
//
// The blocked layouts are the ones fixed by the index expressions of the paper's Fig. 4
// (Section 5): input[img][ifm_tile][ij][ii][ifm], filter[ofm_tile][ifm_tile][kj][ki][ifm][ofm],
// output[img][ofm_tile][oj][oi][ofm] with a channel block of 16 (Section 5.1).  Every kernel
// here is a pure permutation of bit patterns (plus +0.0 fill of channel lanes past C), so it
// is generic over the element size and bit-exact.
//
// All of them are HBM-bound copies (2 x tensor bytes).  Activations: a lane moves one VE x VE block (VE = 16 bytes /
// element size: 4 channels x 4 pixels in fp32, 8 x 8 in 16 bits) with 16-byte accesses on both sides and turns it
// around in registers: VE loads of VE consecutive pixels of one channel each (plain side; the 16 lanes that share a
// channel read 256 contiguous bytes), VE stores of VE consecutive channels of one pixel each (blocked side; the
// 16 / VE lanes that share a pixel write its whole 16-channel line, and the VE stores of a wave fill a contiguous
// range without gaps).  No LDS, no barrier, VE independent loads in flight per lane.  Plain cached accesses: with
// non-temporal loads or stores the transforms of tensors that stay in the Infinity Cache got 15-25 % slower and those
// that stream from HBM 2-3 % faster (measured), and a transform's output is normally what the next kernel reads.  Images whose pixel count is
// not a multiple of VE (7x7; 14x14 in 16 bits) have channel rows that do not start on 16-byte boundaries: they go
// through the LDS transpose below with element-sized accesses.
#include "ps_internal.h"

namespace ps {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Work item L -> (image and channel block ncb, pixel group pxv, channel group j); j runs fastest so that the lanes of
// one pixel are neighbours on the blocked side.
template <typename T, bool kToBlocked>
__global__ __launch_bounds__(256) void act_blocks_kernel(const T *__restrict__ src, T *__restrict__ dst, int C, int Cb,
                                                         int HW, unsigned hwv, unsigned magic_hwv, size_t total)
{
    constexpr int VE = 16 / (int)sizeof(T);  // elements per 16-byte access
    constexpr int G = kBlock / VE;           // channel groups per 16-channel block
    const size_t L = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (L >= total) return;
    const unsigned j = (unsigned)(L % G);
    const unsigned rest = (unsigned)(L / G);
    // rest = ncb * hwv + pxv by reciprocal multiplication (exact for rest < 2^31, see fast_divmod in the convolution)
    unsigned ncb = __umulhi(rest, magic_hwv);
    unsigned pxv = rest - ncb * hwv;
    if (pxv >= hwv) { pxv -= hwv; ++ncb; }
    const unsigned n = ncb / (unsigned)Cb, cb = ncb - n * (unsigned)Cb;
    const int c0 = (int)(cb * kBlock + j * VE);                                  // first channel of this lane's group
    const size_t plain_off = ((size_t)n * C + c0) * HW + (size_t)pxv * VE;       // + e * HW per channel
    const size_t blk_off = ((size_t)ncb * HW + (size_t)pxv * VE) * kBlock + j * VE;  // + e * 16 per pixel
    u32x4 v[VE], o[VE];
    if (kToBlocked) {
#pragma unroll
        for (int e = 0; e < VE; ++e) {
            v[e] = u32x4{0u, 0u, 0u, 0u};  // channel lanes past C hold +0.0
            if (c0 + e < C) v[e] = *reinterpret_cast<const u32x4 *>(src + plain_off + (size_t)e * HW);
        }
    } else {
#pragma unroll
        for (int e = 0; e < VE; ++e) v[e] = *reinterpret_cast<const u32x4 *>(src + blk_off + (size_t)e * kBlock);
    }
    // element b of output vector a = element a of input vector b
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int a = 0; a < 4; ++a) o[a] = u32x4{v[0][a], v[1][a], v[2][a], v[3][a]};
    } else {
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const unsigned lo = v[2 * k][a >> 1], hi = v[2 * k + 1][a >> 1];
                o[a][k] = (a & 1) ? (lo >> 16) | (hi & 0xFFFF0000u) : (lo & 0xFFFFu) | (hi << 16);
            }
    }
    if (kToBlocked) {
#pragma unroll
        for (int e = 0; e < VE; ++e) *reinterpret_cast<u32x4 *>(dst + blk_off + (size_t)e * kBlock) = o[e];
    } else {
#pragma unroll
        for (int e = 0; e < VE; ++e)
            if (c0 + e < C) *reinterpret_cast<u32x4 *>(dst + plain_off + (size_t)e * HW) = o[e];
    }
}

constexpr int kPix = 256;  // pixels per workgroup tile of the LDS-transpose kernels (= threads per workgroup)

// plain [n][c][hw] -> blocked [n][cb][hw][16], any pixel count; workgroup = (image and channel block, pixel tile)
template <typename T>
__global__ __launch_bounds__(kPix) void act_to_blocked_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                              int C, int Cb, int HW, unsigned ntile)
{
    __shared__ T tile[kBlock][kPix + 1];
    const int t = threadIdx.x;
    const unsigned ncb = blockIdx.x / ntile;
    const int n = (int)(ncb / (unsigned)Cb), cb = (int)(ncb % (unsigned)Cb);
    const int pix0 = (int)(blockIdx.x % ntile) * kPix;
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

// blocked [n][cb][hw][16] -> plain [n][c][hw], any pixel count
template <typename T>
__global__ __launch_bounds__(kPix) void blocked_to_act_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                              int C, int Cb, int HW, unsigned ntile)
{
    __shared__ T tile[kBlock][kPix + 1];
    const int t = threadIdx.x;
    const unsigned ncb = blockIdx.x / ntile;
    const int n = (int)(ncb / (unsigned)Cb), cb = (int)(ncb % (unsigned)Cb);
    const int pix0 = (int)(blockIdx.x % ntile) * kPix;
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
    constexpr int VE = 16 / (int)sizeof(T);
    const int Cb = (C + kBlock - 1) / kBlock;
    if (HW % VE == 0) {  // every channel row starts on a 16-byte boundary: register-transposed blocks
        const unsigned hwv = (unsigned)(HW / VE);
        const size_t total = (size_t)N * Cb * hwv * (kBlock / VE);  // < 2^31 / 64: the tensors stay below 2 GiB
        const unsigned magic = hwv == 1 ? 0xFFFFFFFFu : (unsigned)((1ULL << 32) / hwv);
        const dim3 grid((unsigned)((total + 255) / 256));
        if (to_blocked)
            hipLaunchKernelGGL((act_blocks_kernel<T, true>), grid, dim3(256), 0, st, (const T *)src, (T *)dst, C, Cb, HW, hwv,
                               magic, total);
        else
            hipLaunchKernelGGL((act_blocks_kernel<T, false>), grid, dim3(256), 0, st, (const T *)src, (T *)dst, C, Cb, HW, hwv,
                               magic, total);
        return hip_status(hipGetLastError());
    }
    const unsigned ntile = (unsigned)((HW + kPix - 1) / kPix);
    const dim3 grid((unsigned)((size_t)N * Cb * ntile));  // <= tensor elements / 16: fits 32 bits
    if (to_blocked)
        hipLaunchKernelGGL(act_to_blocked_kernel<T>, grid, dim3(kPix), 0, st, (const T *)src, (T *)dst, C, Cb, HW, ntile);
    else
        hipLaunchKernelGGL(blocked_to_act_kernel<T>, grid, dim3(kPix), 0, st, (const T *)src, (T *)dst, C, Cb, HW, ntile);
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
