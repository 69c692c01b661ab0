// Forward convolution as a batch-reduce GEMM on the CDNA4 matrix cores.
//
// What is computed (paper, Fig. 4, Section 5): for an output tile of MT pixels x KT output
// channels,
//     Acc[k][m] += sum over batch elements b = (ifm_tile, kj, ki) of  W_b[16 c][KT]^T . A_b[MT][16 c]
// where A_b gathers, for every output pixel m = (img, oj, oi) of the tile, the 16 input channels
// of block ifm_tile at input position (oj*stride + kj - pad, oi*stride + ki - pad) (zero outside the
// image), and W_b is the 16x16 filter blocks filter[ofm_tile][ifm_tile][kj][ki][.][.] of the tile's
// output-channel blocks.  The figure's three innermost "GEMM" loops become MFMA instructions; its
// six outer loops become the grid (img, ofm_tile, oj, oi -> tile index) and the in-kernel
// batch-reduce loop (ifm_tile, kj, ki).
//
// Mapping to the hardware
//   * v_mfma_f32_32x32x2_f32: matrix A = filter (rows = output channels), matrix B = pixels.
//     A lane then owns 4 consecutive output channels of one pixel per 4 accumulator registers,
//     which is one 16-byte store into the [pixel][16 k] blocked output.
//   * The reduction index inside one 16-channel block is permuted: at MFMA step t the lanes
//     0..31 supply channel t and lanes 32..63 channel 8 + t.  A sum does not care, and it lets a
//     lane fetch its 8 channels of a pixel with two 16-byte LDS reads.
//   * LDS holds, per pipeline stage, G batch elements: the gathered pixels [G][MT][16 c (+4 pad)]
//     and the filter rows [G][16 c][KT].  The 80-byte pixel pitch spreads 8 consecutive pixels
//     over all 32 banks for the 16-byte reads.
//   * Two LDS buffers: global loads of stage i+1 are issued into registers before the MFMAs of
//     stage i and written to the other buffer after them; one barrier per stage.
//   * Global loads are raw buffer loads: an out-of-image tap or an exhausted batch range gets an
//     offset past the buffer size and reads as zero, with no branch.
//   * Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the id is remapped so
//     that each XCD works on a contiguous run of tiles and neighbouring tiles share its L2.
#pragma once
#include "ps_internal.h"

namespace ps {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

struct ConvArgs {
    const void *in;
    const void *wt;
    float *out;
    int H, W, Cb, Kb, R, S, stride, pad, Q;
    int PQ;        // P*Q
    int M;         // N*P*Q, flattened output pixels
    int NB;        // Cb*R*S, batch-reduce length
    int nb_split;  // batch elements per split
    int c_split;
    int n_mt, n_kt;
    int raster;
    unsigned in_bytes, wt_bytes;
};

constexpr unsigned kOobOffset = 0x80000000u;  // >= any accepted buffer size: such a load returns 0
constexpr int kNumXcd = 8;

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// Hardware deals workgroup i to XCD i % 8.  Returns a logical tile index such that the
// workgroups resident on one XCD cover one contiguous range of logical indices.
__device__ inline int xcd_contiguous_index(int bid, int nwg)
{
    const int q = nwg / kNumXcd, rem = nwg % kNumXcd;
    const int xcd = bid % kNumXcd, idx = bid / kNumXcd;
    return xcd * q + min(xcd, rem) + idx;
}

struct TileCoord {
    int mtile, ktile, split;
};

__device__ inline TileCoord decode_tile(const ConvArgs &a)
{
    const int nwg = a.n_mt * a.n_kt * a.c_split;
    int L = xcd_contiguous_index((int)blockIdx.x, nwg);
    TileCoord tc;
    tc.split = L % a.c_split;
    L /= a.c_split;
    if (a.raster == 0) {
        tc.ktile = L % a.n_kt;
        tc.mtile = L / a.n_kt;
    } else {
        tc.mtile = L % a.n_mt;
        tc.ktile = L / a.n_mt;
    }
    return tc;
}

template <int KT, int MT, int WK, int WM, int G>
struct F32Shape {
    static constexpr int NT = 64 * WK * WM;
    static constexpr int TK = KT / (WK * 32);
    static constexpr int TM = MT / (WM * 32);
    static constexpr int PIXP = 20;  // floats per staged pixel: 16 channels + 4 pad
    static constexpr int A_ST = G * MT * PIXP;
    static constexpr int W_ST = G * 16 * KT;
    static constexpr int ST = A_ST + W_ST;
    static constexpr int APT = MT * 4 / NT;  // 16-byte input chunks per thread per batch element
    static constexpr int WPT = (KT * 4 + NT - 1) / NT;  // 16-byte filter chunks per thread per batch element
    static constexpr int LDS_BYTES = 2 * ST * 4;
    static_assert(KT % (WK * 32) == 0 && MT % (WM * 32) == 0, "wave tile must be whole 32x32 MFMA tiles");
    static_assert((MT * 4) % NT == 0, "loader needs whole pixel chunks per thread");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

template <int KT, int MT, int WK, int WM, int G>
__global__ __launch_bounds__(64 * WK * WM) void conv_fwd_f32_kernel(const ConvArgs a)
{
    using Sh = F32Shape<KT, MT, WK, WM, G>;
    constexpr int NT = Sh::NT, TK = Sh::TK, TM = Sh::TM, PIXP = Sh::PIXP;
    constexpr int APT = Sh::APT, WPT = Sh::WPT;
    __shared__ __attribute__((aligned(16))) float lds[2 * Sh::ST];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WK, wm = wave / WK;
    const int half = lane >> 5, l32 = lane & 31;

    const TileCoord tc = decode_tile(a);
    const int m0 = tc.mtile * MT;
    const int kb0 = tc.ktile * (KT / 16);
    const int b_begin = tc.split * a.nb_split;
    const int b_end = b_begin + a.nb_split;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rwt = make_rsrc(a.wt, a.wt_bytes);

    // ---- per-thread gather bookkeeping: which pixels this thread stages ------------------
    const int chunk = tid & 3;  // which 16 bytes of the pixel's 64
    int poff[APT], h0[APT], w0[APT];
#pragma unroll
    for (int i = 0; i < APT; ++i) {
        const int m = m0 + (tid >> 2) + i * (NT / 4);
        if (m < a.M) {
            const int n = m / a.PQ;
            const int pq = m - n * a.PQ;
            const int p = pq / a.Q;
            const int q = pq - p * a.Q;
            h0[i] = p * a.stride - a.pad;
            w0[i] = q * a.stride - a.pad;
            poff[i] = (n * a.Cb * a.H + h0[i]) * a.W + w0[i];
        } else {
            h0[i] = -(1 << 24);  // never inside the image: the tail of the last tile reads zeros
            w0[i] = 0;
            poff[i] = 0;
        }
    }

    // position of the next batch element to load, kept as (cb, r, s) counters
    int lb = b_begin;
    int lcb = lb / (a.R * a.S);
    int lr = (lb - lcb * a.R * a.S) / a.S;
    int ls = lb - (lcb * a.R + lr) * a.S;

    uintx4 areg[G][APT], wreg[G][WPT];

    auto issue_loads = [&]() {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const bool bv = lb < b_end;
            const int tapoff = (lcb * a.H + lr) * a.W + ls;
#pragma unroll
            for (int i = 0; i < APT; ++i) {
                const bool ok = bv && (unsigned)(h0[i] + lr) < (unsigned)a.H && (unsigned)(w0[i] + ls) < (unsigned)a.W;
                const unsigned off = ok ? (unsigned)((poff[i] + tapoff) * 64 + chunk * 16) : kOobOffset;
                areg[g][i] = __builtin_amdgcn_raw_buffer_load_b128(rin, off, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < WPT; ++i) {
                const int id = tid + i * NT;
                const bool wv = bv && (KT * 4 % NT == 0 || id < KT * 4) && kb0 + (id >> 6) < a.Kb;
                const unsigned off = wv ? (unsigned)((((kb0 + (id >> 6)) * a.NB + lb) << 10) + ((id & 63) << 4)) : kOobOffset;
                wreg[g][i] = __builtin_amdgcn_raw_buffer_load_b128(rwt, off, 0, 0);
            }
            ++lb;
            if (++ls == a.S) {
                ls = 0;
                if (++lr == a.R) {
                    lr = 0;
                    ++lcb;
                }
            }
        }
    };

    auto store_stage = [&](int buf) {
        float *As = lds + buf * Sh::ST;
        float *Ws = As + Sh::A_ST;
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int i = 0; i < APT; ++i) {
                const int pix = (tid >> 2) + i * (NT / 4);
                *reinterpret_cast<uintx4 *>(As + (g * MT + pix) * PIXP + chunk * 4) = areg[g][i];
            }
#pragma unroll
            for (int i = 0; i < WPT; ++i) {
                const int id = tid + i * NT;
                const int kbl = id >> 6, e = id & 63;
                if (KT * 4 % NT != 0 && id >= KT * 4) continue;
                *reinterpret_cast<uintx4 *>(Ws + (g * 16 + (e >> 2)) * KT + kbl * 16 + (e & 3) * 4) = wreg[g][i];
            }
        }
    };

    floatx16 acc[TK][TM];
#pragma unroll
    for (int tk = 0; tk < TK; ++tk)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tk][tm][r] = 0.f;

    auto compute_stage = [&](int buf) {
        const float *As = lds + buf * Sh::ST;
        const float *Ws = As + Sh::A_ST;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float pf[TM][8], wf[TK][8];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const float *p = As + (g * MT + (wm * TM + tm) * 32 + l32) * PIXP + half * 8;
                const floatx4 v0 = *reinterpret_cast<const floatx4 *>(p);
                const floatx4 v1 = *reinterpret_cast<const floatx4 *>(p + 4);
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    pf[tm][t] = v0[t];
                    pf[tm][4 + t] = v1[t];
                }
            }
#pragma unroll
            for (int tk = 0; tk < TK; ++tk)
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    wf[tk][t] = Ws[(g * 16 + half * 8 + t) * KT + (wk * TK + tk) * 32 + l32];
#pragma unroll
            for (int t = 0; t < 8; ++t)
#pragma unroll
                for (int tk = 0; tk < TK; ++tk)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
                        acc[tk][tm] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[tk][t], pf[tm][t], acc[tk][tm], 0, 0, 0);
        }
    };

    // ---- software pipeline over stages of G batch elements ------------------------------
    const int nstage = (a.nb_split + G - 1) / G;
    issue_loads();
    store_stage(0);
    __syncthreads();
    for (int st = 0; st < nstage; ++st) {
        const bool more = st + 1 < nstage;
        if (more) issue_loads();
        compute_stage(st & 1);
        if (more) store_stage((st + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue: accumulators -> out[n][kb][p][q][16 k] --------------------------------
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int m = m0 + (wm * TM + tm) * 32 + l32;
        if (m >= a.M) continue;
        const int n = m / a.PQ;
        const int pq = m - n * a.PQ;
#pragma unroll
        for (int tk = 0; tk < TK; ++tk) {
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int ofm = tc.ktile * KT + (wk * TK + tk) * 32 + rq * 8 + half * 4;
                if (ofm >= a.Kb * 16) continue;  // K not a multiple of the tile: padded channels are dropped
                float *o = a.out + (((size_t)(n * a.Kb + (ofm >> 4))) * a.PQ + pq) * 16 + (ofm & 15);
                if (a.c_split == 1) {
                    floatx4 v = {acc[tk][tm][rq * 4 + 0], acc[tk][tm][rq * 4 + 1], acc[tk][tm][rq * 4 + 2],
                                 acc[tk][tm][rq * 4 + 3]};
                    *reinterpret_cast<floatx4 *>(o) = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) atomicAdd(o + e, acc[tk][tm][rq * 4 + e]);
                }
            }
        }
    }
}

// One compiled kernel shape and how to launch it.
struct ShapeEntry {
    int dtype, kt, mt, bpp, threads, lds_bytes;
    void (*launch)(const ConvArgs &, unsigned grid, hipStream_t);
};

template <int KT, int MT, int WK, int WM, int G>
void launch_f32(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((conv_fwd_f32_kernel<KT, MT, WK, WM, G>), dim3(grid), dim3(64 * WK * WM), 0, st, a);
}

#define PS_F32_SHAPE(KT, MT, WK, WM, G)                                                               \
    {PS_F32, KT, MT, G, 64 * WK * WM, F32Shape<KT, MT, WK, WM, G>::LDS_BYTES, &launch_f32<KT, MT, WK, WM, G>}

}  // namespace ps
