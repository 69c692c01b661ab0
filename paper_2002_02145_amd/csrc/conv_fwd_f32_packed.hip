// The tap-packed fp32 kernels (filters over at most 4 input channels, e.g. the first layer of an image network) and
// the loops with a 5x5 filter baked in: one instance per kernel shape and filter side, in a translation unit of their
// own.
#include "conv_fwd_kernel.h"
#include "conv_fwd_f32_n16.h"

namespace ps {

template <int KT, int MT, int WK, int WM, int NBUF>
void launch_f32_packed(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    switch (packed_side_code(a.R, a.cin)) {
    case 7: launch_f32<KT, MT, WK, WM, NBUF, 7>(a, grid, st); break;
    case 33: launch_f32<KT, MT, WK, WM, NBUF, 33>(a, grid, st); break;
    case 35: launch_f32<KT, MT, WK, WM, NBUF, 35>(a, grid, st); break;
    case 37: launch_f32<KT, MT, WK, WM, NBUF, 37>(a, grid, st); break;
    case 311: launch_f32<KT, MT, WK, WM, NBUF, 311>(a, grid, st); break;
    default: break;  // not offered by the host (packs_taps)
    }
}

template <int MT, int NBUF>
void launch_f32_n16_packed(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    switch (packed_side_code(a.R, a.cin)) {
    case 33: launch_f32_n16<MT, NBUF, 33>(a, grid, st); break;
    case 35: launch_f32_n16<MT, NBUF, 35>(a, grid, st); break;
    case 37: launch_f32_n16<MT, NBUF, 37>(a, grid, st); break;
    case 311: launch_f32_n16<MT, NBUF, 311>(a, grid, st); break;
    default: break;  // four channels: the enumerator keeps these shapes away
    }
}

template <int KT, int MT, int WK, int WM, int NBUF>
void launch_f32_5x5(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    launch_f32<KT, MT, WK, WM, NBUF, 5>(a, grid, st);
}
template <int MT, int NBUF>
void launch_f32_n16_5x5(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    launch_f32_n16<MT, NBUF, 5>(a, grid, st);
}

#define PS_INSTANTIATE(KT, MT, WK, WM, NBUF)                                                        \
    template void launch_f32_packed<KT, MT, WK, WM, NBUF>(const ConvArgs &, unsigned, hipStream_t); \
    template void launch_f32_5x5<KT, MT, WK, WM, NBUF>(const ConvArgs &, unsigned, hipStream_t);
PS_F32_SHAPE_LIST(PS_INSTANTIATE)
#undef PS_INSTANTIATE
#define PS_INSTANTIATE(MT, NBUF)                                                              \
    template void launch_f32_n16_packed<MT, NBUF>(const ConvArgs &, unsigned, hipStream_t);  \
    template void launch_f32_n16_5x5<MT, NBUF>(const ConvArgs &, unsigned, hipStream_t);
PS_F32_N16_SHAPE_LIST(PS_INSTANTIATE)
#undef PS_INSTANTIATE

}  // namespace ps
