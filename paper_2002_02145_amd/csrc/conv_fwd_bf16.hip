// bf16-input batch-reduce-GEMM convolution (fp32 accumulate and output) and its kernel shapes.
//
// Same decomposition as the fp32 kernel (see conv_fwd_kernel.h): output tile of MT flattened pixels x KT
// output channels, batch-reduce over (c-block, r, s), LDS ring fed by buffer loads with LDS destination,
// zero fill through out-of-range offsets, fragment double-buffering, guard-free padded loop.  What differs:
//   * v_mfma_f32_32x32x16_bf16: one instruction covers a whole 16-channel block for a 32x32 tile, and a
//     lane supplies 8 consecutive reduction elements (channels 8*(lane/32) .. +7) of its row/column.
//   * A pixel's block is 32 bytes, so a lane's operand is one 16-byte LDS read at pixel*32 + (lane/32)*16;
//     the 64 lanes of a read cover 1 KB contiguously: no swizzle needed.
//   * Filter blocks use the [c/8][16 k][8 c] order: a lane's operand is the 16 bytes at
//     block*512 + (lane/32)*256 + (k%16)*16, again contiguous across lanes.
//   * A batch element is only 32 matrix-core cycles per 32x32 tile, so an iteration (one barrier) handles
//     G batch elements and a ring slot holds G elements.
#include "conv_fwd_bf16_shape.h"
#include "conv_fwd_bf16_halo.h"

namespace ps {

// Loads of ring-slot iteration `it` (counted from the start of the current unrolled block, whose first batch
// element is e0 and first c-block cb0) for the baked-filter path: taps and c-block increments are compile-time
// after unrolling, per-lane offsets come precomputed per tap, the rest is scalar arithmetic.
template <class Sh, int NBUF, int G, int NTAP, int APW, int WPW>
__device__ __forceinline__ void issue_baked_bf16(const ConvArgs &a, char *lds, const unsigned (&vtap)[APW][NTAP],
                                                 const int (&wsoff)[WPW], const bool (&wok)[WPW],
                                                 const unsigned (&vw)[WPW], int wave, int slot, int it, int e0, int cb0)
{
    constexpr int NW = Sh::NW;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int ee = it * G + g;
        const int tap = ee % NTAP, cbi = ee / NTAP;
        const bool valid = e0 + ee < a.nb_split;  // beyond the range: descriptors of size 0 read zeros
        const __amdgpu_buffer_rsrc_t rin_v = make_rsrc(a.in, valid ? a.in_bytes : 0u);
        const int soff = (cb0 + cbi) * a.plane_bytes;
        char *abase = lds + slot * Sh::SLOT + g * Sh::A_EL;
        char *wbase = lds + slot * Sh::SLOT + G * Sh::A_EL + g * Sh::W_EL;
#pragma unroll
        for (int i = 0; i < APW; ++i) {
            const int grp = i * NW + wave;
            char *dst = (Sh::PGRP % NW == 0 || grp < Sh::PGRP) ? abase + grp * 1024 : lds + NBUF * Sh::SLOT;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rin_v, (lds_ptr_t)dst, 16, vtap[i][tap], soff, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int pair = i * NW + wave;
            const __amdgpu_buffer_rsrc_t rwt_v = make_rsrc(a.wt, (valid & wok[i]) ? a.wt_bytes : 0u);
            char *dst = (Sh::WINS % NW == 0 || pair < Sh::WINS) ? wbase + pair * 1024 : lds + NBUF * Sh::SLOT;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt_v, (lds_ptr_t)dst, 16, vw[i], wsoff[i] + ((e0 + ee) << 9), 0, 0);
        }
    }
}

// SIDE > 0: R = S = SIDE baked into the loop (see the fp32 kernel): no vector-ALU work per load.
template <int KT, int MT, int WK, int WM, int NBUF, int G, int SIDE>
__global__ __launch_bounds__(64 * WK * WM) void conv_fwd_bf16_kernel(const ConvArgs a)
{
    constexpr int TAPS = SIDE * SIDE;
    using Sh = Bf16Shape<KT, MT, WK, WM, NBUF, G>;
    constexpr int NW = Sh::NW, TK = Sh::TK, TM = Sh::TM;
    constexpr int APW = Sh::APW, WPW = Sh::WPW, LPS = Sh::LPS, D = Sh::D;
    __shared__ __attribute__((aligned(1024))) char lds[Sh::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave % WK, wm = wave / WK;
    const int half = lane >> 5, l32 = lane & 31;
    const int lhalf = (lane & 1) ^ ((lane >> 4) & 1);  // which half of its pixel this lane loads (see the loader)

    const TileCoord tc = decode_tile(a);
    const int m0 = tc.mtile * MT;
    const int kb0 = tc.ktile * (KT / 16);
    const int b_begin = tc.split * a.nb_split;
    const int b_end = b_begin + a.nb_split;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rwt = make_rsrc(a.wt, a.wt_bytes);

    // ---- loader bookkeeping: one load fills 32 pixels (lane -> pixel lane/2, 16-byte half lane%2).  In every second
    // group of 8 pixels the two halves of a pixel change places in LDS: the 16 lanes an LDS read serves together
    // (16 neighbouring pixels, one half) are 32 bytes apart and would hit every bank twice; with the swap pixels
    // p and p + 8 use different banks.  Neighbouring lanes still fetch one pixel's 32 contiguous bytes. ----
    int poff[APW], h0[APW], w0[APW];
#pragma unroll
    for (int i = 0; i < APW; ++i) {
        const int grp = i * NW + wave;
        const int m = m0 + grp * 32 + (lane >> 1);
        if (grp < Sh::PGRP && m < a.M) {
            int n, pq, p, q;
            fast_divmod(m, a.PQ, a.magic_pq, n, pq);
            fast_divmod(pq, a.Q, a.magic_q, p, q);
            h0[i] = p * a.stride - a.pad;
            w0[i] = q * a.stride - a.pad;
            poff[i] = (n * a.Cb * a.H + h0[i]) * a.W + w0[i];
        } else {
            h0[i] = -(1 << 24);
            w0[i] = 0;
            poff[i] = 0;
        }
    }
    int lb = b_begin;
    int lcb = lb / (a.R * a.S);
    int lr = (lb - lcb * a.R * a.S) / a.S;
    int ls = lb - (lcb * a.R + lr) * a.S;

    auto issue_loads = [&](int slot) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const bool bv = lb < b_end;
            const int tapoff = (lcb * a.H + lr) * a.W + ls;
            char *abase = lds + slot * Sh::SLOT + g * Sh::A_EL;
            char *wbase = lds + slot * Sh::SLOT + G * Sh::A_EL + g * Sh::W_EL;
#pragma unroll
            for (int i = 0; i < APW; ++i) {
                const int grp = i * NW + wave;
                const bool ok = bv & ((unsigned)(h0[i] + lr) < (unsigned)a.H) & ((unsigned)(w0[i] + ls) < (unsigned)a.W);
                const unsigned off = ok ? (unsigned)((poff[i] + tapoff) * 32 + lhalf * 16) : kOobOffset;
                char *dst = (Sh::PGRP % NW == 0 || grp < Sh::PGRP) ? abase + grp * 1024 : lds + NBUF * Sh::SLOT;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rin, (lds_ptr_t)dst, 16, off, 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < WPW; ++i) {
                const int pair = i * NW + wave;           // filter blocks 2*pair and 2*pair + 1
                const int kb = kb0 + 2 * pair + half;
                const bool wv = bv & (Sh::WINS % NW == 0 || pair < Sh::WINS) & (kb < a.Kb);
                const unsigned off = wv ? (unsigned)(((kb * a.NB + lb) << 9) + (l32 << 4)) : kOobOffset;
                char *dst = (Sh::WINS % NW == 0 || pair < Sh::WINS) ? wbase + pair * 1024 : lds + NBUF * Sh::SLOT;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt, (lds_ptr_t)dst, 16, off, 0, 0, 0);
            }
            ++lb;
            ls += 1;
            const int ws = ls == a.S;
            ls = ws ? 0 : ls;
            lr += ws;
            const int wr = lr == a.R;
            lr = wr ? 0 : lr;
            lcb += wr;
        }
    };

    // ---- loader of the baked-filter path: offsets per tap, validity folded in ---------------------
    constexpr int NTAP = TAPS > 0 ? TAPS : 1;
    unsigned vtap[APW][NTAP], vw[WPW];
    int wsoff[WPW];
    bool wok[WPW];
    if constexpr (TAPS > 0) {
#pragma unroll
        for (int i = 0; i < APW; ++i)
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const int r = t / SIDE, sx = t % SIDE;
                const bool ok = ((unsigned)(h0[i] + r) < (unsigned)a.H) & ((unsigned)(w0[i] + sx) < (unsigned)a.W);
                vtap[i][t] = ok ? (unsigned)((poff[i] + r * a.W + sx) * 32 + lhalf * 16) : kOobOffset;
            }
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int pair = i * NW + wave;
            wok[i] = Sh::WINS % NW == 0 || pair < Sh::WINS;
            wsoff[i] = ((kb0 + 2 * pair) * a.NB + b_begin) << 9;
            // lanes 32..63 fetch the next filter block (NB blocks further on), if it exists
            vw[i] = kb0 + 2 * pair + half < a.Kb ? (unsigned)(half * a.NB * 512 + l32 * 16) : kOobOffset;
        }
    }

    // ---- reader bookkeeping -------------------------------------------------------------------
    int paddr[TM], waddr[TK];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) paddr[tm] = ((wm * TM + tm) * 32 + l32) * 32 + (half ^ ((l32 >> 3) & 1)) * 16;
#pragma unroll
    for (int tk = 0; tk < TK; ++tk) {
        const int ofm = (wk * TK + tk) * 32 + l32;
        waddr[tk] = G * Sh::A_EL + (ofm >> 4) * 512 + half * 256 + (ofm & 15) * 16;
    }

    bf16x8 pf[2][G][TM], wf[2][G][TK];
    auto read_frags = [&](int slot, int par) {
        const char *sbase = lds + slot * Sh::SLOT;
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                pf[par][g][tm] = *reinterpret_cast<const bf16x8 *>(sbase + g * Sh::A_EL + paddr[tm]);
#pragma unroll
            for (int tk = 0; tk < TK; ++tk)
                wf[par][g][tk] = *reinterpret_cast<const bf16x8 *>(sbase + g * Sh::W_EL + waddr[tk]);
        }
    };

    floatx16 acc[TK][TM];
#pragma unroll
    for (int tk = 0; tk < TK; ++tk)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tk][tm][r] = 0.f;

    auto mfmas = [&](int par) {
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int tk = 0; tk < TK; ++tk)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    acc[tk][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[par][g][tk], pf[par][g][tm], acc[tk][tm], 0, 0, 0);
    };

    // ---- pipeline over ring slots of G batch elements (range padded with zero elements) -----------
    const int nslot = (a.nb_split + G - 1) / G;
    if constexpr (TAPS > 0) {
        // unrolled so that ring slot, fragment parity and the taps of every element are static
        constexpr int TG = TAPS / ct_gcd(TAPS, G);
        constexpr int U = NBUF / ct_gcd(NBUF, TG) * TG;  // iterations per unrolled block; U * G is a multiple of TAPS
        int cb0 = b_begin / TAPS;
#pragma unroll
        for (int e = 0; e < D; ++e) {
            issue_baked_bf16<Sh, NBUF, G, NTAP, APW, WPW>(a, lds, vtap, wsoff, wok, vw, wave, e, e, 0, cb0);
            __builtin_amdgcn_sched_barrier(0);  // the wait counts assume the elements' loads stay in this order
        }
        wait_vm_and_barrier<(D - 1) * LPS>();
        read_frags(0, 0);
        for (int s0 = 0; s0 < nslot; s0 += U, cb0 += U * G / TAPS) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // a range of whole c-blocks that does not fill the unrolled block ends at a c-block boundary
                if (TAPS > 1 && TAPS % G == 0 && u > 0 && u % TG == 0 && s0 + u >= nslot) break;
                wait_vm_and_barrier<(D - 2) * LPS>();
                read_frags((u + 1) % NBUF, (u + 1) % 2);
                issue_baked_bf16<Sh, NBUF, G, NTAP, APW, WPW>(a, lds, vtap, wsoff, wok, vw, wave, u % NBUF, u + NBUF,
                                                              s0 * G, cb0);
                mfmas(u % 2);
#pragma unroll
                for (int i = 0; i < TK * TM * G; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < D; ++e) {
            issue_loads(e);
            __builtin_amdgcn_sched_barrier(0);  // the wait counts assume the elements' loads stay in this order
        }
        wait_vm_and_barrier<(D - 1) * LPS>();
        read_frags(0, 0);
        for (int s0 = 0; s0 < nslot; s0 += NBUF) {
#pragma unroll
            for (int u = 0; u < NBUF; ++u) {
                wait_vm_and_barrier<(D - 2) * LPS>();
                read_frags((u + 1) % NBUF, (u + 1) % 2);
                issue_loads(u % NBUF);
                mfmas(u % 2);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    write_out<KT, TK, TM, WK, Sh::EPITCH>(a, tc, acc, lds, m0, wave, lane);
}

template <int KT, int MT, int WK, int WM, int NBUF, int G, int SIDE>
void launch_bf16(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((conv_fwd_bf16_kernel<KT, MT, WK, WM, NBUF, G, SIDE>), dim3(grid), dim3(64 * WK * WM), 0, st, a);
}

template <int KT, int MT, int WK, int WM, int NBUF>
void launch_bf16_5x5(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    if constexpr (bf16_5x5_fits<KT, MT, WK, WM, NBUF>())
        hipLaunchKernelGGL((conv_fwd_bf16_kernel<KT, MT, WK, WM, NBUF, 5, 5>), dim3(grid), dim3(64 * WK * WM), 0, st, a);
}

// G batch elements per iteration; the 3x3- and 5x5-baked kernels take one filter row (3 or 5 elements) per iteration
#define PS_BF16_SHAPE(KT, MT, WK, WM, NBUF, G)                                                          \
    {PS_BF16, KT, MT, NBUF, 64 * WK * WM, Bf16Shape<KT, MT, WK, WM, NBUF, G>::LDS_BYTES, G,              \
     &launch_bf16<KT, MT, WK, WM, NBUF, G, 0>, &launch_bf16<KT, MT, WK, WM, NBUF, G, 1>,                 \
     &launch_bf16<KT, MT, WK, WM, NBUF, 3, 3>, &launch_bf16_packed<KT, MT, WK, WM, NBUF, G>,           \
     halo_launch_or_null<KT, MT, WK, WM, NBUF>(),                                                        \
     halo_capacity_bytes<MT>(), 0, Bf16Shape<KT, MT, WK, WM, NBUF, 3>::LDS_BYTES,                        \
     halo_lds_bytes_or_zero<KT, MT, WK, WM, NBUF>(),                                                     \
     bf16_5x5_or_null<KT, MT, WK, WM, NBUF>(), bf16_5x5_lds_or_zero<KT, MT, WK, WM, NBUF>()}
#define PS_TABLE_ROW(KT, MT, WK, WM, G) PS_BF16_SHAPE(KT, MT, WK, WM, 2, G), PS_BF16_SHAPE(KT, MT, WK, WM, 4, G),
static const ShapeEntry kBf16Shapes[] = {PS_BF16_SHAPE_LIST(PS_TABLE_ROW)};

const ShapeEntry *bf16_shapes(int *count)
{
    *count = (int)(sizeof(kBf16Shapes) / sizeof(kBf16Shapes[0]));
    return kBf16Shapes;
}

}  // namespace ps
