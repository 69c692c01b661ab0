// fp32 forward convolution on 16x16x4 MFMA tiles: 64 output channels x MT pixels per workgroup, MT any multiple of 16.
//
// Why a second tiling next to the 32x32x2 kernels of conv_fwd_kernel.h: the waves that share a SIMD run their MFMA
// streams one after another, so a launch takes as long as the most loaded SIMD, and with 32-pixel granularity the
// pixel tile can rarely be chosen such that every compute unit gets the same amount (N = 28, 56x56, K = 64: 686
// tiles of 128 pixels on 256 compute units, 3 on most, 2 on the rest: 89 %).  Here the four waves of a workgroup
// split the 64 output channels (16 each) and every wave covers all MT pixels, so MT moves in steps of 16 and the
// host can pick it so that the tiles divide evenly (same layer: 499 tiles of 176 pixels, 2 on nearly every compute
// unit: 97 %), and deep layers need no split of the reduction.
//
// Operands (v_mfma_f32_16x16x4_f32, D = A*B + C with A = filters, B = pixels): lane l supplies A[row l%16][k l/16]
// and B[k l/16][col l%16] and receives D[rows 4*(l/16) .. +3][col l%16].  The reduction index is permuted as in the
// 32x32 kernels: at MFMA step t the lane group g = l/16 contributes channel 4g + t, so a lane's four B values are
// the 16 bytes at pixel*64 + g*16 (one ds_read_b128 per 16-pixel tile, the 64 lanes covering 1 KB contiguously: no
// swizzle) and its four A values are W[c = 4g + t][k] of its channel row (the filter block is re-ordered to [t][g][k] on its
// way into LDS so that these reads are free of bank conflicts).  A lane's four results are four
// consecutive output channels of one pixel: one 16-byte store.
#pragma once
#include "conv_fwd_kernel.h"

namespace ps {

typedef float floatx4_n __attribute__((ext_vector_type(4)));

// (FUSED only tells the two kernels of a shape apart where a helper is instantiated per shape type)
template <int MT, int NBUF, bool FUSED = false>
struct N16Shape {
    static constexpr int KT = 64;
    static constexpr int NW = 4;          // one wave per 16 output channels
    static constexpr int NT = MT / 16;    // 16-pixel tiles, all of them in every wave
    static constexpr int PGRP = MT / 16;  // 1 KB groups of 16 pixels per batch element
    static constexpr int WBLK = KT / 16;
    static constexpr int APW = (PGRP + NW - 1) / NW;
    static constexpr int WPW = 1;
    static constexpr int LPE = APW + WPW;
    static constexpr int WPITCH = 1024 + 64;
    static constexpr int A_BYTES = MT * 64;
    static constexpr int W_BYTES = WBLK * WPITCH;
    static constexpr int SLOT = A_BYTES + W_BYTES;
    static constexpr bool DUMMY = PGRP % NW != 0;
    static constexpr int LDS_BYTES = NBUF * SLOT + (DUMMY ? 1024 : 0);
    static constexpr int D = NBUF;
    static_assert(MT % 16 == 0 && NBUF >= 2 && NBUF % 2 == 0, "tile shape");
    static_assert(LDS_BYTES <= 160 * 1024 && (D - 2) * LPE <= 63, "LDS budget, vmcnt range");
};

// FUSED = false stores the accumulators as they are (output or a split's partial plane); FUSED = true is the kernel
// for an unsplit range with a bias / max(., 0) / bf16 epilogue.  Two kernels rather than a branch: the plain one
// then stores straight from the accumulator registers.
template <int MT, int NBUF, int SIDE, bool FUSED>
__global__ __launch_bounds__(256) void conv_fwd_f32_n16_kernel(const ConvArgs a)
{
    // SIDE = 33, 35, 37, 311: F x F filter over at most 3 input channels, tap-packed as in conv_fwd_kernel.h (a batch
    // element holds 4 consecutive taps x [c0 c1 c2 0]); chunk g of a pixel is then tap g and MFMA step t is channel t,
    // so step 3 would only multiply the padding lane and is left out.
    static_assert(SIDE == 1 || SIDE == 3 || SIDE == 5 || (side_packs(SIDE) && side_skips_c3(SIDE)), "filter sizes with a baked loop");
    constexpr bool PACKED = side_packs(SIDE);
    constexpr int FS = side_filter(SIDE);
    constexpr int TAPS = PACKED ? (FS * FS + 3) / 4 : SIDE * SIDE;
    constexpr int STEPS = PACKED ? 3 : 4;
    using Sh = N16Shape<MT, NBUF, FUSED>;
    constexpr int NW = Sh::NW, NT = Sh::NT, APW = Sh::APW, WPW = Sh::WPW, LPE = Sh::LPE, D = Sh::D;
    constexpr int U = NBUF / ct_gcd(NBUF, TAPS) * TAPS;
    __shared__ __attribute__((aligned(1024))) char lds[Sh::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, l16 = lane & 15;

    const TileCoord tc = decode_tile(a);
    const int m0 = tc.mtile * MT;
    const int kb0 = tc.ktile * (Sh::KT / 16);
    const int b_begin = tc.split * a.nb_split;
    // the fused kernel's bias, asked for before everything else (it is older than every load the loop counts, so the
    // wait counts below hold; asked for in the epilogue it would cost a load's latency there)
    floatx4_n bias = {0.f, 0.f, 0.f, 0.f};
    if constexpr (FUSED) {
        if ((a.epi & 1) && kb0 + wave < a.Kb) bias = *reinterpret_cast<const floatx4_n *>(a.bias + (kb0 + wave) * 16 + g * 4);
    }

    // ---- loader: one instruction fills 16 pixels (lane -> pixel lane/4, 16-byte chunk lane%4), offsets per tap.
    // In two stages: the taps the first D batch elements need, their loads, then the other taps under the latency of
    // those loads (at the start of a launch every wave of the chip does this arithmetic at the same time).
    unsigned vtap[APW][TAPS];
    int ph0[APW], pw0[APW], ppoff[APW];
#pragma unroll
    for (int i = 0; i < APW; ++i) {
        const int grp = i * NW + wave;
        const int m = m0 + grp * 16 + (lane >> 2);
        int n, pq, p, q;
        fast_divmod(m, a.PQ, a.magic_pq, n, pq);
        fast_divmod(pq, a.Q, a.magic_q, p, q);
        const bool inside = (grp < Sh::PGRP) & (m < a.M);
        ph0[i] = inside ? p * a.stride - a.pad : -(1 << 24);
        pw0[i] = q * a.stride - a.pad;
        ppoff[i] = (n * a.Cb * a.H + ph0[i]) * a.W + pw0[i];
    }
#define PS_N16_TAP_OFFSETS(T0_, T1_)                                                                        \
    _Pragma("unroll") for (int i = 0; i < APW; ++i)                                                        \
        _Pragma("unroll") for (int t = (T0_); t < (T1_); ++t) {                                            \
            /* packed: this lane fetches channels 0..3 of tap 4t + lane%4 of the sequence r*F + s */          \
            const int tapidx = 4 * t + (lane & 3);                                                         \
            const int r = PACKED ? tapidx / FS : t / FS, sx = PACKED ? tapidx - FS * r : t % FS;           \
            const bool ok = ((unsigned)(ph0[i] + r) < (unsigned)a.H) & ((unsigned)(pw0[i] + sx) < (unsigned)a.W) & \
                            (!PACKED || tapidx < FS * FS);                                                 \
            vtap[i][t] = ok ? (unsigned)((ppoff[i] + r * a.W + sx) * 64 + (PACKED ? 0 : (lane & 3) * 16)) : kOobOffset; \
        }
    constexpr int FIRST_TAPS = D < TAPS ? D : TAPS;
    PS_N16_TAP_OFFSETS(0, FIRST_TAPS)
    int wsoff[WPW];
    bool wok[WPW];
    wok[0] = kb0 + wave < a.Kb;  // wave w fetches filter block kb0 + w, the one it multiplies with
    wsoff[0] = ((kb0 + wave) * a.NB + b_begin) << 10;
    // The filter block lands in LDS as [t][g][k]: 16-byte position `lane` takes channel 4g + t, channels-out
    // 4q .. 4q+3 with t = lane/16, g = (lane/4)%4, q = lane%4, so that at MFMA step t the four lane groups read four
    // adjacent 64-byte rows (all banks) instead of rows 256 bytes apart (one bank group, four-way conflict).
    const unsigned wsrc = (unsigned)((4 * ((lane >> 2) & 3) + (lane >> 4)) * 64 + (lane & 3) * 16);
    // packed: position (t, g, q) takes row t (channel) of the block of tap 4e + g; channel 3 is never multiplied;
    // [1] is for the last element, where only the last tap exists
    const unsigned wpk = (lane >> 4) == 3 ? kOobOffset : (unsigned)(((lane >> 2) & 3) * 1024 + (lane >> 4) * 64 + (lane & 3) * 16);
    const unsigned vw[2] = {PACKED ? wpk : wsrc, PACKED ? (((lane >> 2) & 3) == 0 ? wpk : kOobOffset) : wsrc};

    const int nb = a.nb_split;
    int cb0 = b_begin / TAPS;
#pragma unroll
    for (int e = 0; e < D; ++e) {
        issue_baked_fn<Sh, NBUF, TAPS, APW, WPW, PACKED>(a, lds, vtap, wsoff, wok, vw, wave, e, e, 0, cb0);
        __builtin_amdgcn_sched_barrier(0);  // the wait counts assume the elements' loads stay in this order
    }
    __builtin_amdgcn_sched_barrier(0);  // the loads above stay in front of the arithmetic below
    PS_N16_TAP_OFFSETS(FIRST_TAPS, TAPS)
#undef PS_N16_TAP_OFFSETS
    // (an empty statement that "uses" every offset: otherwise the compiler sinks this arithmetic to its first use,
    // behind the wait for the first loads)
#pragma unroll
    for (int i = 0; i < APW; ++i)
#pragma unroll
        for (int t = FIRST_TAPS; t < TAPS; ++t) asm volatile("" ::"v"(vtap[i][t]));

    // ---- reader -------------------------------------------------------------------------------------
    const int paddr = l16 * 64 + g * 16;                                  // + tile * 1024
    const int waddr = Sh::A_BYTES + wave * Sh::WPITCH + g * 64 + l16 * 4;  // + t * 256
    floatx4_n pf[2][NT];
    float wf[2][4];
    floatx4_n acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[j] = floatx4_n{0.f, 0.f, 0.f, 0.f};

#define PS_N16_READ(SLOT_, PAR_)                                                                           \
    {                                                                                                      \
        const char *sb_ = lds + (SLOT_) * Sh::SLOT;                                                        \
        _Pragma("unroll") for (int j = 0; j < NT; ++j)                                                     \
            pf[PAR_][j] = *reinterpret_cast<const floatx4_n *>(sb_ + paddr + j * 1024);                    \
        _Pragma("unroll") for (int t = 0; t < 4; ++t)                                                      \
            wf[PAR_][t] = *reinterpret_cast<const float *>(sb_ + waddr + t * 256);                          \
    }

    // ---- pipeline (as the 32x32 kernels: ring of NBUF batch elements, unrolled over lcm(NBUF, taps)) --------
    __builtin_amdgcn_sched_barrier(0);  // ... and all of it in front of the wait for them
    wait_vm_and_barrier<(D - 1) * LPE>();
    PS_N16_READ(0, 0)
    for (int b0 = 0; b0 < nb; b0 += U, cb0 += U / TAPS) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (PACKED && u >= TAPS) break;  // a tap-packed range is exactly TAPS elements (an odd number)
            // a range of whole c-blocks that does not fill the unrolled block ends at a c-block boundary
            if (baked_loop_exits(TAPS, NBUF) && !PACKED && u > 0 && u % TAPS == 0 && b0 + u >= nb) break;
            wait_vm_and_barrier<(D - 2) * LPE>();
            PS_N16_READ((u + 1) % NBUF, (u + 1) % 2)
            issue_baked_fn<Sh, NBUF, TAPS, APW, WPW, PACKED>(a, lds, vtap, wsoff, wok, vw, wave, u % NBUF,
                                                                             u + NBUF, b0, cb0);
#pragma unroll
            for (int t = 0; t < STEPS; ++t)
#pragma unroll
                for (int j = 0; j < NT; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wf[u % 2][t], pf[u % 2][j][t], acc[j], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < NT * 4; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA ...
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // ... one LDS read ...
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // ... one global load
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#undef PS_N16_READ
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- epilogue: lane (g, l16) holds channels 4g .. 4g+3 of this wave's block for pixel tile*16 + l16 -------
    // Kept short on purpose: while another wave of the SIMD streams MFMAs these instructions issue slowly, so
    // their number, not their latency, is what a short-reduction layer pays for.
    const int kb = kb0 + wave;
    if (kb >= a.Kb) return;  // (no barrier follows)
    const int epi = FUSED ? a.epi : 0;
    const bool bf16_out = epi & 4;
    float *const base = a.c_split == 1 ? a.out : a.partial + (size_t)tc.split * (size_t)a.out_elems;
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(base, bf16_out ? a.out_bytes / 2 : a.out_bytes);
    const int esz = bf16_out ? 2 : 4;

// what the fused epilogue does to one accumulator quad before it is stored
#define PS_N16_FUSED_STORE(V_, VOFF_, SOFF_)                                                               \
    {                                                                                                      \
        floatx4_n v_ = (V_) + bias;                                                                        \
        if (epi & 2) {                                                                                     \
            _Pragma("unroll") for (int i_ = 0; i_ < 4; ++i_) v_[i_] = fmaxf(v_[i_], 0.f);                  \
        }                                                                                                  \
        if (bf16_out) {                                                                                    \
            const uintx2_t h_ = {pack_bf16(v_[0], v_[1]), pack_bf16(v_[2], v_[3])};                        \
            __builtin_amdgcn_raw_buffer_store_b64(h_, rout, VOFF_, SOFF_, kStoreWholeLines);               \
        } else {                                                                                           \
            const uintx4_t u_ = __builtin_bit_cast(uintx4_t, v_);                                          \
            __builtin_amdgcn_raw_buffer_store_b128(u_, rout, VOFF_, SOFF_, kStoreWholeLines);              \
            /* keep the four stored registers live across a short pause: a vector-ALU result allocated */  \
            /* into them right after the store could overtake the store's read of them (see write_out) */  \
            asm volatile("s_nop 1" ::"v"(u_));                                                             \
        }                                                                                                  \
    }

    if (a.PQ >= 16) {
        // The 16 pixels of a quad start at the wave-uniform pixel m0 + 16 j = (image n_j, position r_j): everything
        // that depends on j stays in scalar registers (running r_j and the byte offset S_j of (n_j, kb, r_j), which
        // goes into the store's scalar offset), and a lane only has to notice whether its pixel r_j + l16 has run
        // over into the next image, which lies Kb - 1 channel-block planes further on.
        int n0, r;
        fast_divmod(m0, a.PQ, a.magic_pq, n0, r);
        n0 = __builtin_amdgcn_readfirstlane(n0);
        r = __builtin_amdgcn_readfirstlane(r);
        const int plane = a.PQ * 16 * esz;
        const int delta = (a.Kb - 1) * plane;
        int S = (n0 * a.Kb + kb) * plane + r * 16 * esz;
        const unsigned vlane = (unsigned)((l16 * 16 + g * 4) * esz);
        const unsigned vnext = vlane + (unsigned)delta;
        const bool full = m0 + MT <= a.M;
#define PS_N16_STORE_LOOP(PLAIN_, FULL_)                                                                   \
    _Pragma("unroll") for (int j = 0; j < NT; ++j) {                                                       \
        unsigned voff = l16 >= a.PQ - r ? vnext : vlane;                                                   \
        if (!(FULL_)) voff = l16 < a.M - m0 - j * 16 ? voff : kOobOffset;                                  \
        if constexpr (PLAIN_) {                                                                            \
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4_t, acc[j]), rout, voff, S, kStoreWholeLines); \
        } else {                                                                                           \
            PS_N16_FUSED_STORE(acc[j], voff, S)                                                            \
        }                                                                                                  \
        r += 16;                                                                                           \
        S += 256 * esz;                                                                                    \
        if (r >= a.PQ) {                                                                                   \
            r -= a.PQ;                                                                                     \
            S += delta;                                                                                    \
        }                                                                                                  \
    }
        if (full) {
            PS_N16_STORE_LOOP(!FUSED, true)
        } else {
            PS_N16_STORE_LOOP(!FUSED, false)
        }
#undef PS_N16_STORE_LOOP
    } else {
        // images of fewer than 16 pixels: a quad can span several, every lane tracks its own (image, position)
        const int soff = kb * a.PQ * 16 * esz;
        int n, pq;
        fast_divmod(m0 + l16, a.PQ, a.magic_pq, n, pq);
        int row = n * a.Kb * a.PQ + pq;  // pixel row of the [N][Kb][PQ] output, before the channel-block plane
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const int m = m0 + j * 16 + l16;
            const unsigned voff = m < a.M ? (unsigned)((row * 16 + g * 4) * esz) : kOobOffset;
            pq += 16;
            row += 16;
            while (pq >= a.PQ) {
                pq -= a.PQ;
                row += (a.Kb - 1) * a.PQ;
            }
            if constexpr (FUSED) {
                PS_N16_FUSED_STORE(acc[j], voff, soff)
            } else {
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4_t, acc[j]), rout, voff, soff, kStoreWholeLines);
            }
        }
    }
#undef PS_N16_FUSED_STORE
}

template <int MT, int NBUF, int SIDE>
void launch_f32_n16(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    if (a.epi != 0 && a.c_split == 1)
        hipLaunchKernelGGL((conv_fwd_f32_n16_kernel<MT, NBUF, SIDE, true>), dim3(grid), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((conv_fwd_f32_n16_kernel<MT, NBUF, SIDE, false>), dim3(grid), dim3(256), 0, st, a);
}

// the tap-packed kernels of a shape, chosen by the filter side of the arguments (defined and instantiated in
// conv_fwd_f32_packed.hip)
template <int MT, int NBUF>
void launch_f32_n16_packed(const ConvArgs &a, unsigned grid, hipStream_t st);
template <int MT, int NBUF>
void launch_f32_n16_5x5(const ConvArgs &a, unsigned grid, hipStream_t st);

// No loop with a runtime filter size and no atomic epilogue: the enumerator offers these shapes for 1x1, 3x3 and 5x5
// filters and for the tap-packed filters over at most 3 channels, unsplit.
#define PS_F32_N16_SHAPE(MT, NBUF)                                                                  \
    {PS_F32, 64, MT, NBUF, 256, N16Shape<MT, NBUF>::LDS_BYTES, 1, nullptr, &launch_f32_n16<MT, NBUF, 1>, \
     &launch_f32_n16<MT, NBUF, 3>, &launch_f32_n16_packed<MT, NBUF>, nullptr, 0, 0, 0, 0,             \
     &launch_f32_n16_5x5<MT, NBUF>, 0}
#define PS_F32_N16_SHAPE_LIST(X) X(48, 2) X(48, 4) X(96, 2) X(96, 4) X(176, 2) X(176, 4)

}  // namespace ps
