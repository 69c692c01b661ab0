// fp32 1x1 convolution with a short reduction (C = 64: 4 c-blocks) on 16x16x4 MFMA tiles, pixels stationary:
// a workgroup loads its MT pixels with ALL their input channels into LDS once and then walks over 4 consecutive
// 64-channel output tiles (256 output channels), streaming only filter slices.
//
// Why: with 4 batch elements per tile the kernels of conv_fwd_f32_n16.h spend as long starting and ending a
// workgroup (index arithmetic, first loads, store drain until the slot is refilled) as in MFMAs; measured on
// 64 -> 256 channels at 56x56: every tile shape lands at 57 % of the matrix-core peak.  Here the prologue runs once
// per 4 output tiles, the pixels are fetched once instead of 4 times, and a wave never waits for its stores:
//   * the filter slice is private to the wave that multiplies with it (wave w owns output channels 16w .. 16w+15 of
//     each tile), so after the pixels have landed there is no barrier at all;
//   * vector-memory operations of a wave retire in order, so a load issued AFTER a store cannot be waited for
//     without waiting for the store's acknowledgement too.  The slice of tile j+2 is therefore requested BEFORE the
//     stores of tile j are issued, and the wait in front of tile j+1 leaves those stores in flight;
//   * the first MFMA into each accumulator takes a zero C operand, so nothing is cleared between tiles.
#pragma once
#include "conv_fwd_f32_n16.h"

namespace ps {

constexpr int kKloopTiles = 4;  // 64-channel output tiles per workgroup (tile kt = 256)

template <int MT, int CB>
struct N16KShape {
    static constexpr int NW = 4;
    static constexpr int NT = MT / 16;
    static constexpr int PGRP = MT / 16;
    static constexpr int APW = (PGRP + NW - 1) / NW;
    static constexpr int P_ELEM = MT * 64;               // pixels of one c-block
    static constexpr int P_BYTES = CB * P_ELEM;
    static constexpr int W_SLICE = CB * 1024;            // one wave's filter slice for one output tile
    static constexpr int W_BYTES = NW * 2 * W_SLICE;     // double-buffered per wave
    static constexpr bool DUMMY = PGRP % NW != 0;
    static constexpr int LDS_BYTES = P_BYTES + W_BYTES + (DUMMY ? 1024 : 0);
    static_assert(MT % 16 == 0 && CB % 2 == 0, "tile shape");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert(2 * NT + CB <= 63, "vmcnt range");
};

template <int N>
__device__ inline void wait_vm()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));  // vmcnt(N) lgkmcnt(0)
    asm volatile("" ::: "memory");
}

// The LDS-DMA loads live in __device__ functions (the host pass of the compiler cannot see the builtin in kernel
// scope); FUSED only gives each kernel its own instance.
// Slice of one output tile: this wave's 16 channels (block kb) x all c-blocks; nothing beyond the last channel.
template <int MT, int CB, bool FUSED>
__device__ __forceinline__ void kloop_load_slice(const ConvArgs &a, char *dst, int kb, unsigned wsrc)
{
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.wt, kb < a.Kb ? a.wt_bytes : 0u);
#pragma unroll
    for (int e = 0; e < CB; ++e)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr_t)(dst + e * 1024), 16, wsrc, (kb * CB + e) << 10, 0, 0);
}

// All pixels of the tile, c-block by c-block, each followed by its part of the first filter slice.
template <int MT, int CB, bool FUSED>
__device__ __forceinline__ void kloop_load_first(const ConvArgs &a, char *lds, char *wdst, int wave, int kb,
                                                 const unsigned (&vpix)[N16KShape<MT, CB>::APW], unsigned wsrc)
{
    using Sh = N16KShape<MT, CB>;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(a.wt, kb < a.Kb ? a.wt_bytes : 0u);
#pragma unroll
    for (int e = 0; e < CB; ++e) {
#pragma unroll
        for (int i = 0; i < Sh::APW; ++i) {
            const int grp = i * Sh::NW + wave;
            char *dst = (!Sh::DUMMY || grp < Sh::PGRP) ? lds + e * Sh::P_ELEM + grp * 1024 : lds + Sh::P_BYTES + Sh::W_BYTES;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rin, (lds_ptr_t)dst, 16, vpix[i], e * a.plane_bytes, 0, 0);
        }
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr_t)(wdst + e * 1024), 16, wsrc, (kb * CB + e) << 10, 0, 0);
    }
}

template <int MT, int CB, bool FUSED>
__global__ __launch_bounds__(256) void conv_fwd_f32_n16_kloop_kernel(const ConvArgs a)
{
    using Sh = N16KShape<MT, CB>;
    constexpr int NW = Sh::NW, NT = Sh::NT, APW = Sh::APW;
    __shared__ __attribute__((aligned(1024))) char lds[Sh::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, l16 = lane & 15;

    const TileCoord tc = decode_tile(a);
    const int m0 = tc.mtile * MT;
    const int kb0 = tc.ktile * (kKloopTiles * 4) + wave;  // this wave's channel block in output tile 0; +4 per tile

    // ---- pixel loads: one instruction fills 16 pixels of one c-block (lane -> pixel lane/4, chunk lane%4) -------
    unsigned vpix[APW];
#pragma unroll
    for (int i = 0; i < APW; ++i) {
        const int grp = i * NW + wave;
        const int m = m0 + grp * 16 + (lane >> 2);
        int n, pq, p, q;
        fast_divmod(m, a.PQ, a.magic_pq, n, pq);
        fast_divmod(pq, a.Q, a.magic_q, p, q);
        const int h0 = p * a.stride - a.pad, w0 = q * a.stride - a.pad;
        const bool ok = (grp < Sh::PGRP) & (m < a.M) & ((unsigned)h0 < (unsigned)a.H) & ((unsigned)w0 < (unsigned)a.W);
        vpix[i] = ok ? (unsigned)(((n * a.Cb * a.H + h0) * a.W + w0) * 64 + (lane & 3) * 16) : kOobOffset;
    }
    // filter block -> LDS in the order [t][g][k] (see conv_fwd_f32_n16.h)
    const unsigned wsrc = (unsigned)((4 * ((lane >> 2) & 3) + (lane >> 4)) * 64 + (lane & 3) * 16);
    char *const wbase = lds + Sh::P_BYTES + wave * 2 * Sh::W_SLICE;
    kloop_load_first<MT, CB, FUSED>(a, lds, wbase, wave, kb0, vpix, wsrc);
    __builtin_amdgcn_sched_barrier(0);  // slice 1 after everything the first wait is for
    kloop_load_slice<MT, CB, FUSED>(a, wbase + Sh::W_SLICE, kb0 + 4, wsrc);

    // ---- output offsets, once for all tiles (as in conv_fwd_f32_n16.h: scalar running position, lanes only
    // notice a run-over into the next image); images of fewer than 16 pixels are not offered this kernel -------
    const int epi = FUSED ? a.epi : 0;
    const bool bf16_out = epi & 4;
    const int esz = bf16_out ? 2 : 4;
    const int plane = a.PQ * 16 * esz;
    unsigned voff[NT];
    int soff[NT];
    {
        int n0, r;
        fast_divmod(m0, a.PQ, a.magic_pq, n0, r);
        n0 = __builtin_amdgcn_readfirstlane(n0);
        r = __builtin_amdgcn_readfirstlane(r);
        const int delta = (a.Kb - 1) * plane;
        int S = (n0 * a.Kb + kb0) * plane + r * 16 * esz;
        const unsigned vlane = (unsigned)((l16 * 16 + g * 4) * esz);
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            const unsigned v = l16 >= a.PQ - r ? vlane + (unsigned)delta : vlane;
            voff[j] = l16 < a.M - m0 - j * 16 ? v : kOobOffset;
            soff[j] = S;
            r += 16;
            S += 256 * esz;
            if (r >= a.PQ) {
                r -= a.PQ;
                S += delta;
            }
        }
    }
    floatx4_n bias[kKloopTiles];
    if constexpr (FUSED) {
#pragma unroll
        for (int j = 0; j < kKloopTiles; ++j) {
            bias[j] = floatx4_n{0.f, 0.f, 0.f, 0.f};
            if ((epi & 1) && kb0 + j * 4 < a.Kb)
                bias[j] = *reinterpret_cast<const floatx4_n *>(a.bias + (kb0 + j * 4) * 16 + g * 4);
        }
    }

    // ---- reader ---------------------------------------------------------------------------------------------
    const int paddr = l16 * 64 + g * 16;  // + c-block * P_ELEM + tile * 1024
    const int waddr = g * 64 + l16 * 4;   // + buffer * W_SLICE + c-block * 1024 + t * 256
    floatx4_n pf[2][NT];
    float wf[2][4];
    floatx4_n acc[NT];
#define PS_KLOOP_READ(E_, BUF_, PAR_)                                                                       \
    {                                                                                                      \
        const char *pb_ = lds + (E_) * Sh::P_ELEM + paddr;                                                 \
        const char *wb_ = wbase + (BUF_) * Sh::W_SLICE + (E_) * 1024 + waddr;                              \
        _Pragma("unroll") for (int j = 0; j < NT; ++j)                                                     \
            pf[PAR_][j] = *reinterpret_cast<const floatx4_n *>(pb_ + j * 1024);                            \
        _Pragma("unroll") for (int t = 0; t < 4; ++t)                                                      \
            wf[PAR_][t] = *reinterpret_cast<const float *>(wb_ + t * 256);                                 \
    }
#define PS_KLOOP_MFMA(E_, PAR_)                                                                             \
    {                                                                                                      \
        _Pragma("unroll") for (int t = 0; t < 4; ++t)                                                      \
            _Pragma("unroll") for (int j = 0; j < NT; ++j)                                                 \
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(                                             \
                    wf[PAR_][t], pf[PAR_][j][t], ((E_) == 0 && t == 0) ? floatx4_n{0.f, 0.f, 0.f, 0.f} : acc[j], 0, 0, 0); \
        /* the NT + 4 fragment reads of the next element spread evenly over the 4 NT MFMAs */              \
        _Pragma("unroll") for (int i = 0; i < NT + 4; ++i) {                                               \
            __builtin_amdgcn_sched_group_barrier(0x008, (4 * NT) / (NT + 4), 0);                           \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                             \
        }                                                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                                                 \
    }

    const unsigned out_bytes = bf16_out ? a.out_bytes / 2 : a.out_bytes;

    // One stream of CB * kKloopTiles batch elements: the fragments of the next element are fetched under the MFMAs
    // of the current one, across tile boundaries too.
    wait_vm_and_barrier<CB>();  // pixels (loaded by all four waves) and slice 0 have landed; slice 1 may not
    PS_KLOOP_READ(0, 0, 0)
#pragma unroll
    for (int J = 0; J < kKloopTiles; ++J) {
        const int buf = J % 2;
#pragma unroll
        for (int e = 0; e < CB; ++e) {
            if (e + 1 < CB) {
                PS_KLOOP_READ(e + 1, buf, (e + 1) % 2)
            } else if (J + 1 < kKloopTiles) {
                // slice J+1 was requested before the stores of tile J-1, which may stay in flight
                if (J == 0)
                    wait_vm<0>();
                else
                    wait_vm<NT>();
                PS_KLOOP_READ(0, 1 - buf, 0)
            }
            PS_KLOOP_MFMA(e, e % 2)
        }
        // the slice after next goes into the buffer just read (all its reads have been consumed by the MFMAs above)
        if (J + 2 < kKloopTiles) kloop_load_slice<MT, CB, FUSED>(a, wbase + buf * Sh::W_SLICE, kb0 + (J + 2) * 4, wsrc);
        // The wait counts above rely on this order: every load of the slice in front of every store of the tile.
        // Without the fence the instruction scheduler interleaves the two groups.
        __builtin_amdgcn_sched_barrier(0);
        {
            const int kb = kb0 + J * 4;
            const __amdgpu_buffer_rsrc_t rout = make_rsrc(a.out, kb < a.Kb ? out_bytes : 0u);  // nothing beyond K
            const int kstep = J * 4 * plane;
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                if constexpr (!FUSED) {
                    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4_t, acc[j]), rout, voff[j],
                                                           soff[j] + kstep, kStoreWholeLines);
                } else {
                    floatx4_n v = acc[j] + bias[J];
                    if (epi & 2) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
                    }
                    if (bf16_out) {
                        const uintx2_t h = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
                        __builtin_amdgcn_raw_buffer_store_b64(h, rout, voff[j], soff[j] + kstep, kStoreWholeLines);
                    } else {
                        const uintx4_t u = __builtin_bit_cast(uintx4_t, v);
                        __builtin_amdgcn_raw_buffer_store_b128(u, rout, voff[j], soff[j] + kstep, kStoreWholeLines);
                        asm volatile("s_nop 1" ::"v"(u));  // store-data guard, see conv_fwd_f32_n16.h
                    }
                }
            }
            // the next tile's first MFMAs overwrite the accumulators just stored: same guard
            asm volatile("s_nop 1" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);  // ... and the stores in front of whatever memory operation comes next
        }
    }
#undef PS_KLOOP_READ
#undef PS_KLOOP_MFMA
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// compiled for 4 c-blocks (C = 64); the host offers these shapes to nothing else (with C = 128 the pixels and the
// double-buffered slices leave room for one workgroup per compute unit only, which gains nothing)
template <int MT>
void launch_f32_n16_kloop(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    const bool fused = a.epi != 0 && a.c_split == 1;
    if (a.Cb == 4) {
        if (fused)
            hipLaunchKernelGGL((conv_fwd_f32_n16_kloop_kernel<MT, 4, true>), dim3(grid), dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL((conv_fwd_f32_n16_kloop_kernel<MT, 4, false>), dim3(grid), dim3(256), 0, st, a);
    }
}

#define PS_F32_N16_KLOOP_SHAPE(MT)                                                                      \
    {PS_F32, 64 * kKloopTiles, MT, 2, 256, N16KShape<MT, 4>::LDS_BYTES, 1, nullptr, &launch_f32_n16_kloop<MT>, \
     nullptr, nullptr, nullptr, 0, 1}

}  // namespace ps
