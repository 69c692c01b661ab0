// 3x3, stride 1, pad 1 convolution on 16-bit inputs with the input patch staged once per c-block.
//
// With 16-bit operands a batch element is only 32 matrix-pipe cycles per 32x32 tile, and the kernel that gathers
// the pixels of every tap separately (conv_fwd_bf16_kernel) is bound by the bytes it pulls from L2 into LDS: each
// pixel block nine times.  Here a ring slot holds one whole c-block: the rows of the input that the tile's pixels
// and their neighbours lie in (with the zero border materialised), fetched once, plus the nine filter taps.  The
// matrix-core operand of tap (r, s) is then the same LDS patch read at a shifted address, which costs nothing:
// the nine shifted addresses per lane are computed once per tile.
//
// Patch layout: "extended rows".  Image n owns extended rows n*(H+2) .. n*(H+2)+H+1: a zero row, its H rows, a
// zero row.  A tile of consecutive (n, p, q) pixels covers a contiguous range of extended rows e0 .. e1 (one more
// on either side of its first and last pixel), also across image boundaries, and patch row e - e0 holds
// extended row e with a zero column on either side: pitch W + 2 pixels.  Pixel (n, p, q) has its
// centre at row n*(H+2) + p + 1 - e0, column q + 1, and tap (r, s) at (r - 1) rows and (s - 1) columns from it.
// Patch pixels are numbered row by row, 32 bytes each; in every second group of 8 pixels the two 16-byte channel
// halves of a pixel change places.  (The 16 lanes that an LDS read serves in one go -- 16 neighbouring pixels, one
// channel half -- are 32 bytes apart and would hit every bank twice: the bank-conflict counter read 39 % of the LDS
// cycles.  With the swap, pixels p and p + 8 use different banks, and neighbouring lanes of a load still fetch one
// pixel's 32 contiguous bytes.)
// The loads place 16 bytes per lane at consecutive LDS addresses, so the layout is produced by choosing each
// lane's global address (out of range = zero fill) for the LDS position it writes.
#pragma once
#include "conv_fwd_kernel.h"

namespace ps {

typedef __bf16 bf16x8_h __attribute__((ext_vector_type(8)));

template <int KT, int MT, int WK, int WM>
struct HaloShape {
    static constexpr int NW = WK * WM;
    static constexpr int TK = KT / (WK * 32);
    static constexpr int TM = MT / (WM * 32);
    static constexpr int HALO_BYTES = (MT >= 256 ? 20 : 14) * 1024;  // capacity of the patch; checked on the host
    static constexpr int KBPITCH = 9 * 512 + 512;                   // one 16-channel filter block row: 9 taps + pad
    static constexpr int W_BYTES = (KT / 16) * KBPITCH;
    static constexpr int SLOT = HALO_BYTES + W_BYTES;
    static constexpr int NSLOT = 2;
    static constexpr int HI = HALO_BYTES / 1024, WI = W_BYTES / 1024;  // 1 KB load instructions per c-block
    static constexpr int HPW = (HI + NW - 1) / NW, WPW = (WI + NW - 1) / NW;
    static constexpr bool DUMMY = (HI % NW != 0) || (WI % NW != 0);
    static constexpr int EPITCH = 36;
    static constexpr int RING_BYTES = NSLOT * SLOT + (DUMMY ? 1024 : 0);
    static constexpr int EPI_BYTES = NW * 32 * EPITCH * 4;
    static constexpr int LDS_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
    static_assert(KT % (WK * 32) == 0 && MT % (WM * 32) == 0, "wave tile must be whole 32x32 MFMA tiles");
    static_assert(W_BYTES % 1024 == 0 && LDS_BYTES <= 160 * 1024, "LDS budget");
};

// Loads of c-block `cb` of the workgroup's range into ring slot `slot` (kernel scope only, see issue_baked_fn).
template <class Sh>
__device__ __forceinline__ void issue_halo_cblock(const ConvArgs &a, char *lds, const unsigned (&vh)[Sh::HPW],
                                                  const unsigned (&vw)[Sh::WPW], int wave, int slot, int cb, bool valid)
{
    constexpr int NW = Sh::NW;
    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, valid ? a.in_bytes : 0u);
    const __amdgpu_buffer_rsrc_t rwt = make_rsrc(a.wt, valid ? a.wt_bytes : 0u);
    char *sbase = lds + slot * Sh::SLOT;
    const int in_soff = cb * a.plane_bytes, wt_soff = cb * (9 * 512);
#pragma unroll
    for (int i = 0; i < Sh::HPW; ++i) {
        const int k = i * NW + wave;
        char *dst = (Sh::HI % NW == 0 || k < Sh::HI) ? sbase + k * 1024 : lds + Sh::NSLOT * Sh::SLOT;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rin, (lds_ptr_t)dst, 16, vh[i], in_soff, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < Sh::WPW; ++i) {
        const int k = i * NW + wave;
        char *dst = (Sh::WI % NW == 0 || k < Sh::WI) ? sbase + Sh::HALO_BYTES + k * 1024 : lds + Sh::NSLOT * Sh::SLOT;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt, (lds_ptr_t)dst, 16, vw[i], wt_soff, 0, 0);
    }
}

template <int KT, int MT, int WK, int WM>
__global__ __launch_bounds__(64 * WK * WM) void conv_fwd_bf16_halo_kernel(const ConvArgs a)
{
    using Sh = HaloShape<KT, MT, WK, WM>;
    constexpr int NW = Sh::NW, TK = Sh::TK, TM = Sh::TM, HPW = Sh::HPW, WPW = Sh::WPW;
    constexpr int LPC = HPW + WPW;  // load instructions per wave per c-block
    static_assert(LPC <= 63, "vmcnt range");
    __shared__ __attribute__((aligned(1024))) char lds[Sh::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave % WK, wm = wave / WK;
    const int half = lane >> 5, l32 = lane & 31;

    const TileCoord tc = decode_tile(a);
    const int m0 = tc.mtile * MT;
    const int kb0 = tc.ktile * (KT / 16);
    const int ncb = a.nb_split / 9;  // c-blocks of this workgroup's range
    const int cb_begin = tc.split * ncb;
    const int pitch = a.W + 2, h2 = a.H + 2;

    // extended-row range of the tile
    int n0, pq0, p0, q0, n1, pq1, p1, q1;
    fast_divmod(m0, a.PQ, a.magic_pq, n0, pq0);
    fast_divmod(pq0, a.Q, a.magic_q, p0, q0);
    const int ml = min(m0 + MT, a.M) - 1;
    fast_divmod(ml, a.PQ, a.magic_pq, n1, pq1);
    fast_divmod(pq1, a.Q, a.magic_q, p1, q1);
    const int e0 = n0 * h2 + p0, e1 = n1 * h2 + p1 + 2;
    const int nrows = e1 - e0 + 1;

    // ---- loader: which input chunk belongs at the LDS position a lane writes --------------------------
    unsigned vh[HPW], vw[WPW];
#pragma unroll
    for (int i = 0; i < HPW; ++i) {
        // 16-byte position inside the patch: pixel j / 2; in every second group of 8 pixels the two halves of a
        // pixel change places (see the layout note at the top)
        const int j = (i * NW + wave) * 64 + lane;
        const int px = j >> 1, sub = (j & 1) ^ ((px >> 3) & 1);
        int hr, hc, n, pe;
        fast_divmod(px, pitch, a.magic_pitch, hr, hc);
        fast_divmod(e0 + hr, h2, a.magic_h2, n, pe);
        pe -= 1;
        const bool ok = (hr < nrows) & ((unsigned)pe < (unsigned)a.H) & ((unsigned)(hc - 1) < (unsigned)a.W);
        vh[i] = ok ? (unsigned)(((n * a.Cb * a.H + pe) * a.W + hc - 1) * 32 + sub * 16) : kOobOffset;
    }
#pragma unroll
    for (int i = 0; i < WPW; ++i) {
        const int j = (i * NW + wave) * 64 + lane;  // 16-byte position inside the filter area
        const int kb = j / (Sh::KBPITCH / 16), within = j % (Sh::KBPITCH / 16);
        const bool ok = (kb < KT / 16) & (kb0 + kb < a.Kb) & (within < 9 * 32);
        vw[i] = ok ? (unsigned)((kb0 + kb) * a.NB * 512 + within * 16) : kOobOffset;  // the c-block goes into the scalar offset
    }

    // The first two c-blocks are requested now; the reader's addresses and the cleared accumulators are computed
    // under their latency (all workgroups of a launch start at once, so nothing else would hide that arithmetic).
    issue_halo_cblock<Sh>(a, lds, vh, vw, wave, 0, cb_begin, 0 < ncb);
    __builtin_amdgcn_sched_barrier(0);  // the wait counts assume the elements' loads stay in this order
    issue_halo_cblock<Sh>(a, lds, vh, vw, wave, 1, cb_begin + 1, 1 < ncb);
    __builtin_amdgcn_sched_barrier(0);

    // ---- reader: patch address of every tap for this lane's pixels, filter rows ---------------------------
    int paddr[TM][9], waddr[TK];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int m = min(m0 + (wm * TM + tm) * 32 + l32, a.M - 1);  // lanes past the end read some valid place
        int n, pq, p, q;
        fast_divmod(m, a.PQ, a.magic_pq, n, pq);
        fast_divmod(pq, a.Q, a.magic_q, p, q);
        const int centre = (n * h2 + p + 1 - e0) * pitch + q + 1;  // patch pixel
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int px = centre + (t / 3 - 1) * pitch + (t % 3 - 1);
            paddr[tm][t] = px * 32 + (half ^ ((px >> 3) & 1)) * 16;
        }
    }
#pragma unroll
    for (int tk = 0; tk < TK; ++tk) {
        const int ofm = (wk * TK + tk) * 32 + l32;
        waddr[tk] = Sh::HALO_BYTES + (ofm >> 4) * Sh::KBPITCH + half * 256 + (ofm & 15) * 16;
    }

    bf16x8_h pf[2][TM], wf[2][TK];
    floatx16 acc[TK][TM];
#pragma unroll
    for (int tk = 0; tk < TK; ++tk)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tk][tm][r] = 0.f;

#define PS_HALO_READ(SLOT_, TAP_, PAR_)                                                                          \
    {                                                                                                            \
        const char *sb_ = lds + (SLOT_) * Sh::SLOT;                                                              \
        _Pragma("unroll") for (int tm = 0; tm < TM; ++tm)                                                        \
            pf[PAR_][tm] = *reinterpret_cast<const bf16x8_h *>(sb_ + paddr[tm][TAP_]);                           \
        _Pragma("unroll") for (int tk = 0; tk < TK; ++tk)                                                        \
            wf[PAR_][tk] = *reinterpret_cast<const bf16x8_h *>(sb_ + waddr[tk] + (TAP_) * 512);                  \
    }

    // ---- pipeline: one c-block per ring slot, two slots, the next c-block in flight while this one computes
    // (every address the loop needs exists before the wait: the compiler would otherwise sink that arithmetic to its
    // first use, behind the arrival of the first c-block)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int t = 0; t < 9; ++t) asm volatile("" ::"v"(paddr[tm][t]));
    __builtin_amdgcn_sched_barrier(0);
    wait_vm_and_barrier<LPC>();
    PS_HALO_READ(0, 0, 0)
    for (int c0 = 0; c0 < ncb; c0 += 2) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if (c > 0 && c0 + c >= ncb) break;  // an odd number of c-blocks ends here
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int par = (c * 9 + t) % 2;
                if (t < 8) {
                    PS_HALO_READ(c, t + 1, par ^ 1)
                } else {
                    // every wave is done with slot c, and the other slot's loads (issued a c-block ago) have landed
                    wait_vm_and_barrier<0>();
                    PS_HALO_READ(c ^ 1, 0, par ^ 1)
                    issue_halo_cblock<Sh>(a, lds, vh, vw, wave, c, cb_begin + c0 + c + 2, c0 + c + 2 < ncb);
                }
#pragma unroll
                for (int tk = 0; tk < TK; ++tk)
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
                        acc[tk][tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[par][tk], pf[par][tm], acc[tk][tm], 0, 0, 0);
            }
        }
    }
#undef PS_HALO_READ
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // loads switched off at the end of the range still land (zeros)

    write_out<KT, TK, TM, WK, Sh::EPITCH>(a, tc, acc, lds, m0, wave, lane);
}

template <int KT, int MT, int WK, int WM>
void launch_bf16_halo(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((conv_fwd_bf16_halo_kernel<KT, MT, WK, WM>), dim3(grid), dim3(64 * WK * WM), 0, st, a);
}

// The patch kernel of a tile shape, where two ring slots fit into LDS; listed once per shape (ring 2 rows).
template <int KT, int MT, int WK, int WM, int NBUF>
constexpr LaunchFn halo_launch_or_null()
{
    if constexpr (NBUF == 2 && 2 * ((MT >= 256 ? 20 : 14) * 1024 + (KT / 16) * 5120) <= 160 * 1024)
        return &launch_bf16_halo<KT, MT, WK, WM>;
    else
        return nullptr;
}
template <int KT, int MT, int WK, int WM, int NBUF>
constexpr int halo_lds_bytes_or_zero()
{
    if constexpr (NBUF == 2 && 2 * ((MT >= 256 ? 20 : 14) * 1024 + (KT / 16) * 5120) <= 160 * 1024)
        return HaloShape<KT, MT, WK, WM>::LDS_BYTES;
    else
        return 0;
}
template <int MT>
constexpr int halo_capacity_bytes() { return (MT >= 256 ? 20 : 14) * 1024; }

}  // namespace ps
