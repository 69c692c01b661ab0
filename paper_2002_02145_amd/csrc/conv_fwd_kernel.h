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
//   * LDS is a ring of NBUF slots, one batch element each: the gathered pixels [MT][16 c] and the
//     filter blocks [KT/16][16 c][16 k].  Global memory is copied straight into LDS by buffer loads
//     with the LDS modifier (no staging registers, no LDS store instructions).  Such a load places
//     lane i's 16 bytes at base + 16*i, so the layout in LDS is decided by which global address each
//     lane asks for: the four 16-byte chunks of a pixel are stored at position chunk ^ ((pixel>>1)&3),
//     which spreads 8 consecutive pixels over all 32 banks for the 16-byte fragment reads, and each
//     1 KB filter block gets a 64-byte pad so that the two blocks a 32-channel fragment spans do
//     not share banks.
//   * A load whose tap falls outside the image, whose pixel is past the end of the tensor or whose
//     batch element is past the end of the range asks for an offset beyond the buffer size: the
//     hardware returns zeros, so padding needs no branch and no separate fill.
//   * Pipeline, per batch element b: wait for this wave's loads of element b+1, barrier (everyone's
//     b+1 is in LDS, and everyone holds element b's fragments in registers, so slot b is free), issue
//     the loads of element b+NBUF into slot b, read the fragments of b+1 into the other register set,
//     run the MFMAs of b.  LDS reads, loads and address arithmetic interleave with the MFMAs of the
//     same iteration; a load has NBUF-1 iterations to land.
//   * The batch range is padded to a multiple of NBUF with all-zero elements (out-of-range loads),
//     which keeps the unrolled loop free of guards.
//   * Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the id is remapped so
//     that each XCD works on a contiguous run of tiles and neighbouring tiles share its L2.
#pragma once
#include <type_traits>
#include "ps_internal.h"

namespace ps {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_ptr_t;

struct ConvArgs {
    const void *in;
    const void *wt;
    float *out;
    int H, W, Cb, Kb, R, S, stride, pad, Q;
    int cin;       // input channels before padding to whole 16-blocks
    int PQ;        // P*Q
    int M;         // N*P*Q, flattened output pixels
    int NB;        // Cb*R*S, batch-reduce length
    int nb_split;  // batch elements per split
    int c_split;
    int n_mt, n_kt;
    unsigned magic_split, magic_inner;
    unsigned magic_pitch, magic_h2;     // floor(2^32 / (W + 2)), floor(2^32 / (H + 2)): patch rows of the 3x3 kernels  // floor(2^32 / c_split), floor(2^32 / (raster == 0 ? n_kt : n_mt))
    const float *bias;  // per output channel, added before the store (epi & 1)
    int epi;            // fused epilogue: 1 = add bias, 2 = max(x, 0), 4 = store bf16 (round to nearest even)
    int raster;
    unsigned in_bytes, wt_bytes;
    int plane_bytes;       // bytes of one [H][W][16] c-block plane of the input
    unsigned magic_pq, magic_q;  // floor(2^32 / PQ), floor(2^32 / Q) for divisions without the long VALU sequence
    unsigned out_bytes;
    float *partial;        // split reduction with a workspace: [c_split][out elements], else nullptr (atomics)
    long long out_elems;   // N*K*P*Q
};

constexpr unsigned kOobOffset = 0x80000000u;  // >= any accepted buffer size: such a load returns 0
constexpr int kNumXcd = 8;

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// n / d for 0 <= n < 2^31 with magic = floor(2^32 / d) (0xFFFFFFFF for d = 1): the estimate
// mulhi(n, magic) is the quotient or one less, so one correction step makes it exact.  Six VALU
// instructions instead of the ~35 of a generic 32-bit division; every VALU instruction stalls the matrix
// pipe of its SIMD, so the prologue and epilogue arithmetic is kept short too.
__device__ inline void fast_divmod(int n, int d, unsigned magic, int &q, int &r)
{
    q = (int)__umulhi((unsigned)n, magic);
    r = n - q * d;
    const int adj = r >= d;
    q += adj;
    r -= adj ? d : 0;
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
    // divisions by reciprocal multiplication: a generic 32-bit division is ~35 instructions, and everything a
    // workgroup issues before its first MFMA competes with the MFMA streams of its neighbours on the SIMD
    tc.split = 0;
    if (a.c_split > 1) fast_divmod(L, a.c_split, a.magic_split, L, tc.split);
    if (a.raster == 0)
        fast_divmod(L, a.n_kt, a.magic_inner, tc.mtile, tc.ktile);
    else
        fast_divmod(L, a.n_mt, a.magic_inner, tc.ktile, tc.mtile);
    return tc;
}

// s_waitcnt vmcnt(N) lgkmcnt(0), then s_barrier.  The wait is emitted through the builtin so that the
// compiler's own wait-count bookkeeping sees it (it cannot look inside inline assembly and would
// otherwise add redundant waits in front of the MFMAs).
template <int N>
__device__ inline void wait_vm_and_barrier()
{
    // gfx9 immediate: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14]; expcnt 7 = no wait
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (0 << 8) | ((N >> 4) << 14));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

typedef unsigned uintx2_t __attribute__((ext_vector_type(2)));

// Two fp32 values rounded to bf16 (nearest, ties to even), packed low | high << 16: the hardware's packed conversion
// (v_cvt_pk_bf16_f32, one instruction; a NaN stays a quiet NaN).  Done with integer arithmetic it took seven
// instructions per value, a microsecond on a launch that stores 64 values per lane.
typedef float floatx2_cvt __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_cvt __attribute__((ext_vector_type(2)));
__device__ inline unsigned pack_bf16(float lo, float hi)
{
    const floatx2_cvt v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_cvt));
}

// Cache policy (auxiliary operand of the buffer-store builtins; bit 4 = sc1) of output stores whose every instruction
// covers whole 64-byte lines, as in the 16x16-tile kernels: the line is written through L2 at once instead of
// staying there dirty until it is evicted, which leaves the L2 to the operands.  Measured at N = 28: 3x3 64 -> 64 at
// 56x56 48.9 -> 47.2 us, the pixel-stationary 1x1 64 -> 256 27.8 -> 24.2 us, 1x1 256 -> 64 25.8 -> 25.6 us; the
// non-temporal hint (bit 1) gives the same on the first and less on the second.  It only pays for whole lines: half
// lines written through one by one no longer merge in L2 and everything gets slower (16-bit stem 39 -> 47 us, 16-bit
// 1x1 64 -> 256 21 -> 37 us with the 32x32-tile kernels' stores as the accumulator layout has them), which is why
// write_out below turns its tiles around first.
constexpr int kStoreWholeLines = 16;

// Epilogue shared by the fp32 and bf16 kernels: accumulators -> out[n][kb][p][q][16 k].
// acc[tk][tm] is the 32x32 tile (output channels x pixels) number (tk, tm) of this wave in the MFMA
// result layout: register r of lane l holds channel 8*(r/4) + 4*(l/32) + r%4 of pixel l%32.
template <int KT, int TK, int TM, int WK, int EPITCH>
__device__ inline void write_out(const ConvArgs &a, const TileCoord &tc, floatx16 (&acc)[TK][TM], char *lds, int m0,
                                 int wave, int lane)
{
    const int wk = wave % WK, wm = wave / WK;
    const int half = lane >> 5, l32 = lane & 31;
    float *const stage = reinterpret_cast<float *>(lds) + wave * (32 * EPITCH);  // this wave's 32x32 patch
    const int rp = lane >> 3, c4 = lane & 7;
    if (a.c_split == 1 || a.partial != nullptr) {
        // From the accumulator layout a store instruction would write 32 bytes of each of 32 pixels: half a 64-byte
        // line, the other half following with the next instruction.  Each wave therefore turns its 32x32 tile around
        // in a private LDS patch, so that 4 consecutive lanes cover one pixel's 16-channel line (lanes 4..7 of the
        // group: the next channel block's) and an instruction writes 16 whole lines, with the write-through policy
        // that whole lines allow (kStoreWholeLines).  Measured at N = 28 with 16-bit inputs: 3x3 64 -> 64 at 56x56
        // 14.4 -> 11.5 us, 1x1 64 -> 256 21.4 -> 17.1 us, 1x1 128 -> 512 14.3 -> 11.1 us; same bits.
        // With a workspace, split s stores its partial tile into plane s; a second kernel adds the planes.
        // Buffer stores: the per-lane part of the address (pixel, channel quad) is computed once per pixel
        // tile, the tile's channel-block part is a scalar offset, and lanes past the end of the tensor get an
        // out-of-range offset, which drops their store.
        float *const base = a.c_split == 1 ? a.out : a.partial + (size_t)tc.split * (size_t)a.out_elems;
        const int epi = a.c_split == 1 ? a.epi : 0;  // a split's partial planes stay raw; the adding pass applies it
        // The bias of this lane's channel quads, asked for once and before the wait below (TK loads, which that wait
        // leaves in flight: vector-memory operations retire in order, and everything older has to have landed).
        floatx4 bias_q[TK];
#pragma unroll
        for (int tk = 0; tk < TK; ++tk) bias_q[tk] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (epi & 1) {
#pragma unroll
            for (int tk = 0; tk < TK; ++tk) {
                const int ofm = tc.ktile * KT + (wk * TK + tk) * 32 + c4 * 4;
                if (ofm < a.Kb * 16) bias_q[tk] = *reinterpret_cast<const floatx4 *>(a.bias + ofm);
            }
            wait_vm_and_barrier<TK>();
        } else {
            wait_vm_and_barrier<0>();  // every wave has read its last fragments: the ring may be overwritten
        }
        // Two instances of the loop: the plain one has no branch between the LDS reads and the stores of a tile, so
        // the four reads are issued together and the stores follow as the data return.
        auto store_tiles = [&](auto fused_tag) {
            constexpr bool FUSED = decltype(fused_tag)::value;
            const bool bf16_out = FUSED && (epi & 4);
            const int esz = bf16_out ? 2 : 4;
            const __amdgpu_buffer_rsrc_t rout = make_rsrc(base, bf16_out ? a.out_bytes / 2 : a.out_bytes);
            const int plane = a.PQ * 16 * esz;  // bytes from one 16-channel block plane to the next
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                unsigned vpix[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = m0 + (wm * TM + tm) * 32 + rp + 8 * i;
                    int n, pq;
                    fast_divmod(m, a.PQ, a.magic_pq, n, pq);
                    vpix[i] = m < a.M ? (unsigned)(((n * a.Kb * a.PQ + pq) * 16 + (c4 & 3) * 4) * esz + (c4 >> 2) * plane) : kOobOffset;
                }
#pragma unroll
                for (int tk = 0; tk < TK; ++tk) {
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq) {
                        const floatx4 v = {acc[tk][tm][rq * 4 + 0], acc[tk][tm][rq * 4 + 1], acc[tk][tm][rq * 4 + 2],
                                           acc[tk][tm][rq * 4 + 3]};
                        *reinterpret_cast<floatx4 *>(stage + l32 * EPITCH + rq * 8 + half * 4) = v;
                    }
                    const int ofm0 = tc.ktile * KT + (wk * TK + tk) * 32;  // uniform; this lane: + c4 * 4
                    const bool kok = ofm0 + c4 * 4 < a.Kb * 16;            // K not a multiple of the tile: padded channels are dropped
                    const int soff = (ofm0 >> 4) * plane;
                    const floatx4 bias = bias_q[tk];  // (zero and unused in the plain instance)
                    // fused: all four reads first, so that the branches on the epilogue flags do not sit between a read
                    // and its store (the plain instance has no such branches and is left to the scheduler)
                    floatx4 vq[4];
                    if constexpr (FUSED) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) vq[i] = *reinterpret_cast<const floatx4 *>(stage + (rp + 8 * i) * EPITCH + c4 * 4);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        floatx4 v;
                        if constexpr (FUSED)
                            v = vq[i];
                        else
                            v = *reinterpret_cast<const floatx4 *>(stage + (rp + 8 * i) * EPITCH + c4 * 4);
                        const unsigned voff = kok ? vpix[i] : kOobOffset;
                        if constexpr (FUSED) {
                            // bias, max(., 0), optional rounding to bf16
                            v += bias;
                            if (epi & 2) {
#pragma unroll
                                for (int j = 0; j < 4; ++j) v[j] = fmaxf(v[j], 0.f);
                            }
                        }
                        // A vector-ALU write to the data registers of a multi-dword store issued just before it can
                        // overtake the store's read of them on this hardware (the compiler only guards the form without
                        // a scalar offset).  The empty asm keeps the stored registers live across a short s_nop, so
                        // nothing can be scheduled or allocated into that window.
                        if (bf16_out) {
                            const uintx2_t h = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
                            __builtin_amdgcn_raw_buffer_store_b64(h, rout, voff, soff, kStoreWholeLines);
                            asm volatile("s_nop 1" ::"v"(h[0]), "v"(h[1]));
                        } else {
                            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4_t, v), rout, voff, soff, kStoreWholeLines);
                            asm volatile("s_nop 1" ::"v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]));
                        }
                    }
                }
            }
        };
        if (epi == 0)
            store_tiles(std::false_type{});
        else
            store_tiles(std::true_type{});
        return;
    }
    // Split reduction without a workspace: partial tiles are added into the cleared output with fp32 atomics.  Issued from
    // the accumulator layout, one atomic instruction would touch 64 different 64-byte lines; each wave
    // therefore turns its 32x32 tile around in a private LDS patch so that 16 consecutive lanes cover
    // one pixel's 16-channel line and an instruction adds into 4 whole lines.
    wait_vm_and_barrier<0>();  // zero-fill loads of the padded iterations may still be landing in the ring
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
        for (int tk = 0; tk < TK; ++tk) {
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const floatx4 v = {acc[tk][tm][rq * 4 + 0], acc[tk][tm][rq * 4 + 1], acc[tk][tm][rq * 4 + 2],
                                   acc[tk][tm][rq * 4 + 3]};
                *reinterpret_cast<floatx4 *>(stage + l32 * EPITCH + rq * 8 + half * 4) = v;
            }
            const int ofm = tc.ktile * KT + (wk * TK + tk) * 32 + c4 * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int pr = rp + 8 * i;
                const floatx4 v = *reinterpret_cast<const floatx4 *>(stage + pr * EPITCH + c4 * 4);
                const int m = m0 + (wm * TM + tm) * 32 + pr;
                if (m < a.M && ofm < a.Kb * 16) {
                    int n, pq;
                    fast_divmod(m, a.PQ, a.magic_pq, n, pq);
                    float *o = a.out + (((size_t)(n * a.Kb + (ofm >> 4))) * a.PQ + pq) * 16 + (ofm & 15);
#pragma unroll
                    for (int e = 0; e < 4; ++e) atomicAdd(o + e, v[e]);
                }
            }
        }
    }
}

template <int KT, int MT, int WK, int WM, int NBUF>
struct F32Shape {
    static constexpr int NW = WK * WM;
    static constexpr int NT = 64 * NW;
    static constexpr int TK = KT / (WK * 32);  // 32x32 MFMA tiles per wave, output-channel direction
    static constexpr int TM = MT / (WM * 32);  // ... pixel direction
    static constexpr int PGRP = MT / 16;       // 1 KB groups of 16 pixels per batch element
    static constexpr int WBLK = KT / 16;       // 1 KB filter blocks per batch element
    static constexpr int APW = (PGRP + NW - 1) / NW;
    static constexpr int WPW = (WBLK + NW - 1) / NW;
    static constexpr int LPE = APW + WPW;      // load instructions per wave per batch element (same for all waves)
    static constexpr int WPITCH = 1024 + 64;   // bytes from one filter block to the next in LDS
    static constexpr int A_BYTES = MT * 64;
    static constexpr int W_BYTES = WBLK * WPITCH;
    static constexpr int SLOT = A_BYTES + W_BYTES;
    // waves with no real group/block left still issue their load (keeps vmcnt uniform) into a dump area
    static constexpr bool DUMMY = (PGRP % NW != 0) || (WBLK % NW != 0);
    static constexpr int EPITCH = 36;  // floats per pixel row of the epilogue patch: 32 channels + 4 pad
    static constexpr int RING_BYTES = NBUF * SLOT + (DUMMY ? 1024 : 0);
    static constexpr int EPI_BYTES = NW * 32 * EPITCH * 4;
    static constexpr int LDS_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
    static constexpr int D = NBUF;  // prefetch distance in batch elements
    static_assert(KT % (WK * 32) == 0 && MT % (WM * 32) == 0, "wave tile must be whole 32x32 MFMA tiles");
    static_assert(NBUF >= 2 && NBUF % 2 == 0, "ring size must be even (fragment register parity)");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert((D - 2) * LPE <= 63, "vmcnt range");
};

// Loads of batch element e (counted from the start of the workgroup's range, b0 already added by the
// caller's loop) into ring slot `slot`, for the baked-filter path: the tap (e % NTAP) and c-block increment
// (e / NTAP) are compile-time after unrolling, per-lane offsets come precomputed per tap, everything else is
// scalar arithmetic.  An element beyond the range gets descriptors of size 0, i.e. reads zeros.
// (A __device__ function rather than a lambda of the kernel: lambdas are also compiled for the host,
// where buffer descriptors cannot be built.  TAG only gives kernels that agree in every other argument an
// instance of their own.)
template <class Sh, int NBUF, int NTAP, int APW, int WPW, bool PACK4, int TAG = 0>
__device__ __forceinline__ void issue_baked_fn(const ConvArgs &a, char *lds, const unsigned (&vtap)[APW][NTAP],
                                               const int (&wsoff)[WPW], const bool (&wok)[WPW],
                                               const unsigned (&vw)[2], int wave, int slot, int e, int b0, int cb0)
{
    constexpr int NW = Sh::NW;
    const int tap = e % NTAP, cbi = e / NTAP;
    const bool valid = b0 + e < a.nb_split;
    const __amdgpu_buffer_rsrc_t rin_v = make_rsrc(a.in, valid ? a.in_bytes : 0u);
    const int soff = PACK4 ? 0 : (cb0 + cbi) * a.plane_bytes;
    char *sbase = lds + slot * Sh::SLOT;
#pragma unroll
    for (int i = 0; i < APW; ++i) {
        const int grp = i * NW + wave;
        char *dst = (Sh::PGRP % NW == 0 || grp < Sh::PGRP) ? sbase + grp * 1024 : lds + NBUF * Sh::SLOT;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rin_v, (lds_ptr_t)dst, 16, vtap[i][tap], soff, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < WPW; ++i) {
        const int blk = i * NW + wave;
        const __amdgpu_buffer_rsrc_t rwt_v = make_rsrc(a.wt, (valid & wok[i]) ? a.wt_bytes : 0u);
        char *dst = (Sh::WBLK % NW == 0 || blk < Sh::WBLK) ? sbase + Sh::A_BYTES + blk * Sh::WPITCH
                                                           : lds + NBUF * Sh::SLOT;
        // tap-packed mode: the blocks of taps 4*tap .. 4*tap+3, per-lane offsets pick tap and channel row
        const int wso = PACK4 ? wsoff[i] + tap * 4 * 1024 : wsoff[i] + ((b0 + e) << 10);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt_v, (lds_ptr_t)dst, 16, vw[PACK4 && tap == NTAP - 1 ? 1 : 0], wso, 0, 0);
    }
}

constexpr int ct_gcd(int x, int y) { return y == 0 ? x : ct_gcd(y, x % y); }
// Whether the unrolled block of a baked loop (lcm(ring, taps) batch elements) can be left at a c-block boundary: the
// compiler unrolls a loop with such an exit only up to a certain length (the host's padded_elems mirrors this).
constexpr bool baked_loop_exits(int taps, int ring) { return taps > 1 && ring / ct_gcd(ring, taps) * taps <= 50; }

// Codes of the loops with the filter baked in (template argument SIDE of the fp32 kernels):
//   1, 3, 5     R = S = SIDE, 16 channels of one tap per batch element;
//   7           tap-packed 7x7 over at most 4 input channels (4 taps x 4 channels per batch element);
//   30 + F      tap-packed F x F over at most 3 input channels, F = 3, 5, 7 (the zero fourth lane is never multiplied);
//   311         the same for 11 x 11.
constexpr bool side_packs(int side) { return side == 7 || side >= 30; }
constexpr bool side_skips_c3(int side) { return side >= 30; }
constexpr int side_filter(int side) { return side >= 300 ? side - 300 : side >= 30 ? side - 30 : side; }
// the code for an F x F filter over `cin` input channels, 0 if that combination has no tap-packed loop
inline int packed_side_code(int F, int cin)
{
    if (F == 7 && cin == 4) return 7;
    if (cin > 3) return 0;
    return F == 3 || F == 5 || F == 7 ? 30 + F : F == 11 ? 311 : 0;
}

// SIDE > 0 bakes a square SIDE x SIDE filter into the loop (R = S = SIDE, split ranges on c-block
// boundaries): every load's per-lane offset, validity included, is then precomputed per tap, and the loop
// issues no vector-ALU instruction at all.  That matters because on this hardware each VALU instruction
// takes about 4 cycles away from the SIMD's matrix pipe (measured: one VALU op per MFMA costs 6 %).
// SIDE = 0 is the general path (any R, S), which computes offsets and predicates per load.
template <int KT, int MT, int WK, int WM, int NBUF, int SIDE>
__global__ __launch_bounds__(64 * WK * WM) void conv_fwd_f32_kernel(const ConvArgs a)
{
    // Tap-packed mode (codes above) for inputs with at most 4 channels (one c-block whose lanes 4..15 are
    // zero padding, e.g. an RGB network stem): a batch element then holds channels 0..3 of four
    // consecutive taps of the row-major tap sequence (4 taps x 4 channels = the 16 reduction lanes) instead of 16
    // channels of one tap, so a 7x7 filter takes ceil(49 / 4) = 13 elements instead of 49, an 11x11 one 31 instead of
    // 121.  Pixels and filter blocks are gathered accordingly from the ordinary blocked tensors: only the per-lane load
    // offsets differ.  (F * F is odd for every F offered, so the last element always holds exactly one tap.)
    constexpr bool PACK4 = side_packs(SIDE);
    // With at most 3 input channels lane 3 of every tap's 4-channel group is zero padding, and with the reduction
    // index permuted as below it is MFMA steps 3 and 7 that would multiply it: they are left out, a quarter of the
    // matrix-core work.
    constexpr bool SKIP_C3 = side_skips_c3(SIDE);
    constexpr int FS = side_filter(SIDE);  // filter side
    constexpr int FSD = FS > 0 ? FS : 1;
    constexpr int TAPS = PACK4 ? (FS * FS + 3) / 4 : SIDE * SIDE;
    using Sh = F32Shape<KT, MT, WK, WM, NBUF>;
    constexpr int NW = Sh::NW, TK = Sh::TK, TM = Sh::TM;
    constexpr int APW = Sh::APW, WPW = Sh::WPW, LPE = Sh::LPE, D = Sh::D;
    __shared__ __attribute__((aligned(1024))) char lds[Sh::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave % WK, wm = wave / WK;
    const int half = lane >> 5, l32 = lane & 31;

    const TileCoord tc = decode_tile(a);
    const int m0 = tc.mtile * MT;
    const int kb0 = tc.ktile * (KT / 16);
    const int b_begin = tc.split * a.nb_split;
    const int b_end = b_begin + a.nb_split;

    const __amdgpu_buffer_rsrc_t rin = make_rsrc(a.in, a.in_bytes);
    const __amdgpu_buffer_rsrc_t rwt = make_rsrc(a.wt, a.wt_bytes);

    // ---- loader bookkeeping ---------------------------------------------------------------------
    // One load instruction fills one 1 KB pixel group: lane -> pixel group*16 + lane/4, LDS chunk
    // position lane%4, which holds global chunk (lane%4) ^ ((pixel >> 1) & 3) = (lane%4) ^ ((lane>>3)&3).
    const int gchunk = (lane & 3) ^ ((lane >> 3) & 3);
    int poff[APW], h0[APW], w0[APW];
#pragma unroll
    for (int i = 0; i < APW; ++i) {
        const int grp = i * NW + wave;
        const int m = m0 + grp * 16 + (lane >> 2);
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
        const bool bv = lb < b_end;
        const int tapoff = (lcb * a.H + lr) * a.W + ls;
        char *sbase = lds + slot * Sh::SLOT;
#pragma unroll
        for (int i = 0; i < APW; ++i) {
            const int grp = i * NW + wave;
            const bool ok = bv & ((unsigned)(h0[i] + lr) < (unsigned)a.H) & ((unsigned)(w0[i] + ls) < (unsigned)a.W);
            const unsigned off = ok ? (unsigned)((poff[i] + tapoff) * 64 + gchunk * 16) : kOobOffset;
            char *dst = (Sh::PGRP % NW == 0 || grp < Sh::PGRP) ? sbase + grp * 1024 : lds + NBUF * Sh::SLOT;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rin, (lds_ptr_t)dst, 16, off, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int blk = i * NW + wave;
            const bool wv = bv & (Sh::WBLK % NW == 0 || blk < Sh::WBLK) & (kb0 + blk < a.Kb);
            const unsigned off = wv ? (unsigned)((((kb0 + blk) * a.NB + lb) << 10) + (lane << 4)) : kOobOffset;
            char *dst = (Sh::WBLK % NW == 0 || blk < Sh::WBLK) ? sbase + Sh::A_BYTES + blk * Sh::WPITCH
                                                               : lds + NBUF * Sh::SLOT;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rwt, (lds_ptr_t)dst, 16, off, 0, 0, 0);
        }
        ++lb;
        // branch-free (r, s, c-block) odometer: keeps the whole iteration one basic block
        ls += 1;
        const int ws = ls == a.S;
        ls = ws ? 0 : ls;
        lr += ws;
        const int wr = lr == a.R;
        lr = wr ? 0 : lr;
        lcb += wr;
    };

    // ---- loader of the baked-filter path: offsets per tap, validity folded in ----------------------
    constexpr int NTAP = TAPS > 0 ? TAPS : 1;
    unsigned vtap[APW][NTAP];
    int wsoff[WPW];      // byte offset of filter block (kb0 + blk, batch element 0), uniform per wave
    bool wok[WPW];
    if constexpr (TAPS > 0) {
#pragma unroll
        for (int i = 0; i < APW; ++i)
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                // ordinary: tap (r, sx), this lane fetches chunk `gchunk` of the pixel's 16 channels;
                // tap-packed: element t holds taps 4t .. 4t+3 of the sequence r*F + s, this lane fetches channels
                // 0..3 of tap 4t + gchunk
                const int tapidx = 4 * t + gchunk;
                const int r = PACK4 ? tapidx / FSD : t / FSD;
                const int sx = PACK4 ? tapidx - FS * r : t % FSD;
                const bool ok = ((unsigned)(h0[i] + r) < (unsigned)a.H) & ((unsigned)(w0[i] + sx) < (unsigned)a.W) &
                                (!PACK4 || tapidx < FS * FS);
                vtap[i][t] = ok ? (unsigned)((poff[i] + r * a.W + sx) * 64 + (PACK4 ? 0 : gchunk * 16)) : kOobOffset;
            }
#pragma unroll
        for (int i = 0; i < WPW; ++i) {
            const int blk = i * NW + wave;
            wok[i] = (Sh::WBLK % NW == 0 || blk < Sh::WBLK) & (kb0 + blk < a.Kb);
            wsoff[i] = ((kb0 + blk) * a.NB + b_begin) << 10;
        }
    }
    // per-lane offset of a filter load inside its 1 KB block: lane*16 normally; tap-packed, LDS row
    // c' = lane/4 = 4*j + c is row c of the block of tap 4t + j (blocks follow the tap sequence; [1]: the last
    // element, where only the last tap exists)
    unsigned vw[2];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        const int cp = lane >> 2, j = cp >> 2, c = cp & 3;
        vw[g] = !PACK4 ? (unsigned)lane << 4 : (g == 0 || j == 0) ? (unsigned)(j * 1024 + c * 64 + (lane & 3) * 16) : kOobOffset;
    }
    // ---- reader bookkeeping -------------------------------------------------------------
    int paddr[TM], waddr[TK];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int p = (wm * TM + tm) * 32 + l32;
        const int pos0 = (2 * half) ^ ((p >> 1) & 3);
        paddr[tm] = p * 64 + pos0 * 16;
    }
#pragma unroll
    for (int tk = 0; tk < TK; ++tk) {
        const int ofm = (wk * TK + tk) * 32 + l32;
        waddr[tk] = Sh::A_BYTES + (ofm >> 4) * Sh::WPITCH + half * 8 * 64 + (ofm & 15) * 4;
    }

    float pf[2][TM][8], wf[2][TK][8];
    auto read_frags = [&](int slot, int par) {
        const char *sbase = lds + slot * Sh::SLOT;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const floatx4 v0 = *reinterpret_cast<const floatx4 *>(sbase + paddr[tm]);
            const floatx4 v1 = *reinterpret_cast<const floatx4 *>(sbase + (paddr[tm] ^ 16));
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                pf[par][tm][t] = v0[t];
                pf[par][tm][4 + t] = v1[t];
            }
        }
#pragma unroll
        for (int tk = 0; tk < TK; ++tk)
#pragma unroll
            for (int t = 0; t < 8; ++t)
                wf[par][tk][t] = *reinterpret_cast<const float *>(sbase + waddr[tk] + t * 64);
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
        for (int t = 0; t < 8; ++t) {
            if (SKIP_C3 && (t & 3) == 3) continue;  // channel 3 of both taps of this lane's half: zeros
#pragma unroll
            for (int tk = 0; tk < TK; ++tk)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
                    acc[tk][tm] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[par][tk][t], pf[par][tm][t], acc[tk][tm], 0, 0, 0);
        }
    };

    // ---- pipeline ---------------------------------------------------------------------------
    const int nb = a.nb_split;
    if constexpr (TAPS > 0) {
        // unrolled over lcm(NBUF, TAPS) iterations so that ring slot, fragment parity and tap are static
        constexpr int U = NBUF / ct_gcd(NBUF, TAPS) * TAPS;
        int cb0 = b_begin / TAPS;
#pragma unroll
        for (int e = 0; e < D; ++e) {
            issue_baked_fn<Sh, NBUF, NTAP, APW, WPW, PACK4, SIDE>(a, lds, vtap, wsoff, wok, vw, wave, e, e, 0, cb0);
            __builtin_amdgcn_sched_barrier(0);  // the wait counts assume the elements' loads stay in this order
        }
        wait_vm_and_barrier<(D - 1) * LPE>();
        read_frags(0, 0);
        for (int b0 = 0; b0 < nb; b0 += U, cb0 += U / TAPS) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (PACK4 && u >= TAPS) break;  // a tap-packed range is exactly TAPS elements (an odd number)
                // a range of whole c-blocks that does not fill the unrolled block ends at a c-block boundary (one
                // scalar compare per c-block; 1x1 ranges, and blocks too long to unroll with an exit, stay padded)
                if (baked_loop_exits(TAPS, NBUF) && !PACK4 && u > 0 && u % TAPS == 0 && b0 + u >= nb) break;
                wait_vm_and_barrier<(D - 2) * LPE>();
                read_frags((u + 1) % NBUF, (u + 1) % 2);
                issue_baked_fn<Sh, NBUF, NTAP, APW, WPW, PACK4, SIDE>(a, lds, vtap, wsoff, wok, vw, wave, u % NBUF, u + NBUF,
                                                         b0, cb0);
                mfmas(u % 2);
                // order within the iteration: after each of the first MFMAs one LDS read and one load, so
                // that the next fragments are requested early and into the other register set
#pragma unroll
                for (int i = 0; i < TK * TM * 8; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < D; ++e) {  // elements 0..D-1 (zero-filled beyond the range)
            issue_loads(e);
            __builtin_amdgcn_sched_barrier(0);  // the wait counts assume the elements' loads stay in this order
        }
        wait_vm_and_barrier<(D - 1) * LPE>();        // element 0 has landed everywhere
        read_frags(0, 0);
        // iteration b: slot b % NBUF, fragment parity b % 2; unrolled by NBUF (even) so both are static.
        // The range is padded up to a multiple of NBUF with zero elements (loads past b_end read zeros).
        for (int b0 = 0; b0 < nb; b0 += NBUF) {
#pragma unroll
            for (int u = 0; u < NBUF; ++u) {
                wait_vm_and_barrier<(D - 2) * LPE>();
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

// One compiled kernel shape and how to launch it.
typedef void (*LaunchFn)(const ConvArgs &, unsigned grid, hipStream_t);
struct ShapeEntry {
    int dtype, kt, mt, ring, threads, lds_bytes;
    int group;            // batch elements per loop iteration of the general kernel (fp32: 1)
    LaunchFn launch;      // any filter size
    LaunchFn launch_1x1;  // R = S = 1 baked in (nullptr if not compiled)
    LaunchFn launch_3x3;  // R = S = 3 baked in
    LaunchFn launch_packed; // tap-packed loops (R = S = 3, 5, 7, 11 over at most 3 channels; 7x7 over 4), by the arguments
    LaunchFn launch_halo; // 3x3, stride 1, pad 1 with the input patch staged once per c-block (nullptr if none)
    int halo_bytes;       // capacity of that kernel's patch
    int stationary;       // 1: pixels with all their input channels stay in LDS (1x1 filters, C = 64 only)
    int lds_3x3;          // LDS bytes of launch_3x3 / launch_halo where they differ from lds_bytes (0 = the same):
    int lds_halo;         // the tile model prices occupancy with the footprint of the loop that will run
    LaunchFn launch_5x5;  // R = S = 5 baked in (nullptr if not compiled)
    int lds_5x5;          // LDS bytes of launch_5x5 where they differ from lds_bytes (0 = the same)
};

template <int KT, int MT, int WK, int WM, int NBUF, int SIDE>
void launch_f32(const ConvArgs &a, unsigned grid, hipStream_t st)
{
    hipLaunchKernelGGL((conv_fwd_f32_kernel<KT, MT, WK, WM, NBUF, SIDE>), dim3(grid), dim3(64 * WK * WM), 0, st, a);
}

// the tap-packed kernels of a shape, chosen by filter side and channel count of the arguments (defined and
// instantiated in conv_fwd_f32_packed.hip)
template <int KT, int MT, int WK, int WM, int NBUF>
void launch_f32_packed(const ConvArgs &a, unsigned grid, hipStream_t st);
// the loop with a 5x5 filter baked in (same translation unit)
template <int KT, int MT, int WK, int WM, int NBUF>
void launch_f32_5x5(const ConvArgs &a, unsigned grid, hipStream_t st);

#define PS_F32_SHAPE(KT, MT, WK, WM, NBUF)                                                              \
    {PS_F32, KT, MT, NBUF, 64 * WK * WM, F32Shape<KT, MT, WK, WM, NBUF>::LDS_BYTES, 1,                   \
     &launch_f32<KT, MT, WK, WM, NBUF, 0>, &launch_f32<KT, MT, WK, WM, NBUF, 1>,                        \
     &launch_f32<KT, MT, WK, WM, NBUF, 3>, &launch_f32_packed<KT, MT, WK, WM, NBUF>, nullptr, 0, 0, 0, 0,    \
     &launch_f32_5x5<KT, MT, WK, WM, NBUF>, 0}

//               KT   MT  WK WM NBUF       wave tile (channels x pixels)
// Ring depths: a load has (NBUF - 1) iterations to land, and an iteration lasts 512 matrix-core cycles
// per 32x32 tile a wave owns, so the small wave tiles get the deeper rings.
#define PS_F32_SHAPE_LIST(X)                                     \
    X(256, 128, 4, 2, 2) X(256, 128, 4, 2, 4) /* 64 x 64, 8 waves */ \
    X(256, 64, 4, 1, 2) X(256, 64, 4, 1, 4)   /* 64 x 64 */          \
    X(128, 128, 2, 2, 2) X(128, 128, 2, 2, 4) /* 64 x 64 */          \
    X(64, 256, 1, 4, 2) X(64, 256, 1, 4, 4)   /* 64 x 64 */          \
    X(128, 64, 2, 2, 2) X(128, 64, 2, 2, 4) X(128, 64, 2, 2, 8) /* 64 x 32 */ \
    X(64, 128, 2, 2, 2) X(64, 128, 2, 2, 4) X(64, 128, 2, 2, 8) /* 32 x 64 */ \
    X(64, 64, 2, 2, 2) X(64, 64, 2, 2, 4) X(64, 64, 2, 2, 8)    /* 32 x 32 */ \
    X(128, 32, 4, 1, 4) X(128, 32, 4, 1, 8)   /* 32 x 32 */          \
    X(32, 128, 1, 4, 4) X(32, 128, 1, 4, 8)   /* 32 x 32 */          \
    X(64, 32, 2, 1, 4) X(64, 32, 2, 1, 8)     /* 32 x 32, 2 waves */ \
    X(32, 64, 1, 2, 4) X(32, 64, 1, 2, 8)     /* 32 x 32, 2 waves */


}  // namespace ps
