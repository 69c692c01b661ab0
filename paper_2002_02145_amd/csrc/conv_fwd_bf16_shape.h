// Tile-shape arithmetic of the 16-bit kernels and the list of compiled shapes.
#pragma once
#include "conv_fwd_kernel.h"

namespace ps {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int KT, int MT, int WK, int WM, int NBUF, int G>
struct Bf16Shape {
    static constexpr int NW = WK * WM;
    static constexpr int TK = KT / (WK * 32);
    static constexpr int TM = MT / (WM * 32);
    static constexpr int PGRP = MT / 32;  // 1 KB groups of 32 pixels per batch element
    static constexpr int WINS = KT / 32;  // 1 KB pairs of filter blocks per batch element
    static constexpr int APW = (PGRP + NW - 1) / NW;
    static constexpr int WPW = (WINS + NW - 1) / NW;
    static constexpr int LPS = G * (APW + WPW);  // load instructions per wave per ring slot
    static constexpr int A_EL = MT * 32;
    static constexpr int W_EL = KT * 32;
    static constexpr int SLOT = G * (A_EL + W_EL);
    static constexpr bool DUMMY = (PGRP % NW != 0) || (WINS % NW != 0);
    static constexpr int EPITCH = 36;
    static constexpr int RING_BYTES = NBUF * SLOT + (DUMMY ? 1024 : 0);
    static constexpr int EPI_BYTES = NW * 32 * EPITCH * 4;
    static constexpr int LDS_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
    static constexpr int D = NBUF;
    static_assert(KT % (WK * 32) == 0 && MT % (WM * 32) == 0, "wave tile must be whole 32x32 MFMA tiles");
    static_assert(NBUF >= 2 && NBUF % 2 == 0, "ring size must be even (fragment register parity)");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert((D - 2) * LPS <= 63, "vmcnt range");
};

// the tap-packed kernels of a shape, chosen by the filter side of the arguments (defined and instantiated in
// conv_fwd_bf16_packed.hip)
template <int KT, int MT, int WK, int WM, int NBUF, int G>
void launch_bf16_packed(const ConvArgs &a, unsigned grid, hipStream_t st);
// the loop with a 5x5 filter baked in, one filter row (5 batch elements) per iteration (conv_fwd_bf16.hip); not
// compiled where that ring does not fit LDS or the wait counter's range
template <int KT, int MT, int WK, int WM, int NBUF>
void launch_bf16_5x5(const ConvArgs &a, unsigned grid, hipStream_t st);
template <int KT, int MT, int WK, int WM, int NBUF>
constexpr bool bf16_5x5_fits()
{
    constexpr int NW = WK * WM, LPS = 5 * ((MT / 32 + NW - 1) / NW + (KT / 32 + NW - 1) / NW);
    // (eight-wave shapes have 256 registers per lane: five elements' fragments next to 64 accumulators do not fit)
    return NW <= 4 && NBUF * 5 * (MT + KT) * 32 + 1024 <= 160 * 1024 && (NBUF - 2) * LPS <= 63;
}
template <int KT, int MT, int WK, int WM, int NBUF>
constexpr LaunchFn bf16_5x5_or_null()
{
    if constexpr (bf16_5x5_fits<KT, MT, WK, WM, NBUF>())
        return &launch_bf16_5x5<KT, MT, WK, WM, NBUF>;
    else
        return nullptr;
}
template <int KT, int MT, int WK, int WM, int NBUF>
constexpr int bf16_5x5_lds_or_zero()
{
    if constexpr (bf16_5x5_fits<KT, MT, WK, WM, NBUF>())
        return Bf16Shape<KT, MT, WK, WM, NBUF, 5>::LDS_BYTES;
    else
        return 0;
}

// Every shape is compiled with rings of 2 and 4 slots.
//                      KT   MT  WK WM  G        wave tile (channels x pixels)
#define PS_BF16_SHAPE_LIST(X)                         \
    X(256, 128, 4, 2, 2) /* 64 x 64, 8 waves */       \
    X(128, 128, 2, 2, 2) /* 64 x 64 */                \
    X(64, 256, 1, 4, 2)  /* 64 x 64 */                \
    X(128, 64, 2, 2, 4)  /* 64 x 32 */                \
    X(64, 128, 2, 2, 4)  /* 32 x 64 */                \
    X(64, 64, 2, 2, 4)   /* 32 x 32 */                \
    X(32, 128, 1, 4, 4)  /* 32 x 32 */                \
    X(128, 32, 4, 1, 4)  /* 32 x 32 */                \
    X(64, 32, 2, 1, 4)   /* 32 x 32, 2 waves */       \
    X(32, 64, 1, 2, 4)   /* 32 x 32, 2 waves */

}  // namespace ps
