// The tap-packed 16-bit kernels (filters over at most 8 input channels), one instance per kernel shape and filter
// side, in a translation unit of their own.
#include "conv_fwd_bf16_shape.h"

namespace ps {

// Loads of ring-slot iteration `it` of the tap-packed loop (elements it*G .. it*G + G-1; compile-time after
// unrolling).  A __device__ function rather than a lambda of the kernel, as issue_baked_fn.
template <class Sh, int NBUF, int G, int NEL, int APW, int WPW>
__device__ __forceinline__ void issue_packed_bf16(const ConvArgs &a, char *lds, const unsigned (&vtap)[APW][NEL],
                                                   const unsigned (&vw)[WPW][2], const int (&wsoff)[WPW],
                                                   const bool (&wok)[WPW], int wave, int slot, int it)
{
    constexpr int NW = Sh::NW;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int t = it * G + g;
        const bool valid = t < NEL;  // iterations past the last element load zeros (descriptors of size 0)
        const int tt = valid ? t : 0;
        const __amdgpu_buffer_rsrc_t rin_v = make_rsrc(a.in, valid ? a.in_bytes : 0u);
        char *abase = lds + slot * Sh::SLOT + g * Sh::A_EL;
        char *wbase = lds + slot * Sh::SLOT + G * Sh::A_EL + g * Sh::W_EL;
#pragma unroll
        for (int i = 0; i < APW; ++i) {
            const int grp = i * NW + wave;
            char *dst = (Sh::PGRP % NW == 0 || grp < Sh::PGRP) ? abase + grp * 1024 : lds + NBUF * Sh::SLOT;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rin_v, (lds_ptr_t)dst, 16, vtap[i][tt], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int pair = i * NW + wave;
            const __amdgpu_buffer_rsrc_t rwt_v = make_rsrc(a.wt, (valid & wok[i]) ? a.wt_bytes : 0u);
            char *dst = (Sh::WINS % NW == 0 || pair < Sh::WINS) ? wbase + pair * 1024 : lds + NBUF * Sh::SLOT;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt_v, (lds_ptr_t)dst, 16, vw[i][tt == NEL - 1 ? 1 : 0],
                                                     wsoff[i] + tt * 2 * 512, 0, 0);
        }
    }
}

// F x F filter (F = 3, 5, 7, 11) over at most 8 input channels (the first layer of an image network) in 16 bits.  One
// 32x32x16 MFMA reduces over 16 values; in the blocked layout a tap of such a layer fills 3 (or up to 8) of them and
// the rest is channel padding, so the general loop runs F * F batch elements with most reduction lanes zero and pulls
// every pixel's 32-byte block through L2 F * F times.  Here a batch element is 2 consecutive taps of the row-major tap
// sequence x channels 0..7 (reduction index 8*j + c for tap 2*t + j): 25 elements for 7x7, and 16 instead of 32 bytes
// per pixel and tap.  The tensors at the boundary keep their blocked layouts; only the gather differs: a tap's eight
// channels are the first 16 bytes of the pixel's block, and the first 256 bytes of a filter block are exactly its
// [16 k][8 c] plane of channels 0..7, so both operands still arrive by 16-byte buffer loads with LDS destination, each
// lane asking for the global bytes that belong at the LDS position it writes.  (Packing four taps x four channels
// needs 8-byte pieces, i.e. 4-byte loads, and measured slower than the general loop: scattered 4-byte loads retire
// at a few lanes per clock.)  LDS layout, fragment reads and MFMAs are those of conv_fwd_bf16_kernel.
template <int KT, int MT, int WK, int WM, int NBUF, int G, int FS>
__global__ __launch_bounds__(64 * WK * WM) void conv_fwd_bf16_packed_kernel(const ConvArgs a)
{
    using Sh = Bf16Shape<KT, MT, WK, WM, NBUF, G>;
    constexpr int NW = Sh::NW, TK = Sh::TK, TM = Sh::TM, D = Sh::D;
    constexpr int APW = Sh::APW, WPW = Sh::WPW, LPS = Sh::LPS;
    constexpr int NEL = (FS * FS + 1) / 2;     // batch elements: taps 2t, 2t+1 (F * F is odd: the last one holds one tap)
    constexpr int NSLOT = (NEL + G - 1) / G;   // ring-slot iterations
    __shared__ __attribute__((aligned(1024))) char lds[Sh::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave % WK, wm = wave / WK;
    const int half = lane >> 5, l32 = lane & 31;
    // a load fills 32 pixels: lane -> pixel lane/2, LDS half lane%2, which holds the logical half (= tap of the pair)
    // lhalf: in every second group of 8 pixels the halves change places, as the fragment reads expect
    const int lhalf = (lane & 1) ^ ((lane >> 4) & 1);

    const TileCoord tc = decode_tile(a);
    const int m0 = tc.mtile * MT;
    const int kb0 = tc.ktile * (KT / 16);

    unsigned vtap[APW][NEL];
#pragma unroll
    for (int i = 0; i < APW; ++i) {
        const int grp = i * NW + wave;
        const int m = m0 + grp * 32 + (lane >> 1);
        const bool live = (Sh::PGRP % NW == 0 || grp < Sh::PGRP) & (m < a.M);
        int n, pq, p, q;
        fast_divmod(min(m, a.M - 1), a.PQ, a.magic_pq, n, pq);
        fast_divmod(pq, a.Q, a.magic_q, p, q);
        const int h0 = p * a.stride - a.pad, w0 = q * a.stride - a.pad;
        const int poff = (n * a.H + h0) * a.W + w0;   // one c-block
#pragma unroll
        for (int t = 0; t < NEL; ++t) {
            const int tap = 2 * t + lhalf;
            const int r = tap / FS;
            const int sx = tap - FS * r;
            const bool ok = live & (tap < FS * FS) & ((unsigned)(h0 + r) < (unsigned)a.H) & ((unsigned)(w0 + sx) < (unsigned)a.W);
            vtap[i][t] = ok ? (unsigned)((poff + r * a.W + sx) * 32) : kOobOffset;
        }
    }
    // filters: a load fills two LDS blocks (output-channel blocks kb, kb+1 of the pair), 512 bytes each: [tap of the
    // pair][16 k][8 c].  Lane -> block lane/32, tap (lane%32)/16, row lane%16; global blocks of consecutive taps are 512
    // bytes apart, those of consecutive output-channel blocks NB * 512.  [1]: the last element, where only the last tap exists.
    unsigned vw[WPW][2];
    int wsoff[WPW];
    bool wok[WPW];
#pragma unroll
    for (int i = 0; i < WPW; ++i) {
        const int pair = i * NW + wave;
        wok[i] = Sh::WINS % NW == 0 || pair < Sh::WINS;
        wsoff[i] = (kb0 + 2 * pair) * a.NB * 512;     // + 2t * 512 per element
        const int j = (l32 >> 4);
        vw[i][0] = kb0 + 2 * pair + half < a.Kb ? (unsigned)(half * a.NB * 512 + j * 512 + (lane & 15) * 16) : kOobOffset;
        vw[i][1] = j == 0 ? vw[i][0] : kOobOffset;
    }

    // ---- reader (as in conv_fwd_bf16_kernel) --------------------------------------------------------------------
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

    // ---- pipeline: NSLOT iterations, fully unrolled (slot, fragment parity and taps are compile-time); iterations past
    // the last element load zeros (descriptors of size 0) so that every iteration issues the same number of loads
#pragma unroll
    for (int e = 0; e < D; ++e) {
        issue_packed_bf16<Sh, NBUF, G, NEL, APW, WPW>(a, lds, vtap, vw, wsoff, wok, wave, e, e);
        __builtin_amdgcn_sched_barrier(0);  // the wait counts assume the elements' loads stay in this order
    }
    wait_vm_and_barrier<(D - 1) * LPS>();
    read_frags(0, 0);
#pragma unroll
    for (int u = 0; u < NSLOT; ++u) {
        wait_vm_and_barrier<(D - 2) * LPS>();
        read_frags((u + 1) % NBUF, (u + 1) % 2);
        issue_packed_bf16<Sh, NBUF, G, NEL, APW, WPW>(a, lds, vtap, vw, wsoff, wok, wave, u % NBUF, u + NBUF);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int tk = 0; tk < TK; ++tk)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    acc[tk][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u % 2][g][tk], pf[u % 2][g][tm], acc[tk][tm], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    write_out<KT, TK, TM, WK, Sh::EPITCH>(a, tc, acc, lds, m0, wave, lane);
}

template <int KT, int MT, int WK, int WM, int NBUF, int G>
void launch_bf16_packed(const ConvArgs &a, unsigned grid, hipStream_t st)
{
#define PS_SIDE(F)                                                                                                   \
    case F:                                                                                                          \
        hipLaunchKernelGGL((conv_fwd_bf16_packed_kernel<KT, MT, WK, WM, NBUF, G, F>), dim3(grid), dim3(64 * WK * WM), 0, st, a); \
        break;
    switch (a.R) {
        PS_SIDE(3) PS_SIDE(5) PS_SIDE(7) PS_SIDE(11)
    default: break;  // not offered by the host (packs_taps)
    }
#undef PS_SIDE
}

#define PS_INSTANTIATE(KT, MT, WK, WM, G)                                                                \
    template void launch_bf16_packed<KT, MT, WK, WM, 2, G>(const ConvArgs &, unsigned, hipStream_t);    \
    template void launch_bf16_packed<KT, MT, WK, WM, 4, G>(const ConvArgs &, unsigned, hipStream_t);
PS_BF16_SHAPE_LIST(PS_INSTANTIATE)
#undef PS_INSTANTIATE

}  // namespace ps
