// Outer-loop variant space and its analytic ranking.
//
// The paper generates n variants of the loops around the microkernel by tiling and
// interchange with varied tile sizes (Section 4.2), sizes the working set of every data
// reuse (Algorithm 1), assigns each working set to the fastest memory level it fits
// (Algorithm 2) and ranks variants by the sum over levels of data volume x latency / bandwidth
// (Eq. 1); the top k are then run (k = 1 in the paper).
//
// The GPU analogue below enumerates workgroup tiles (output-channel tile, pixel tile, batch
// elements per LDS stage, split of the batch-reduce range, launch order) and scores each one:
// the tile's reuses have closed-form working sets (rectangular tiles), each is assigned to the
// level whose capacity holds it (registers/LDS by construction, then one XCD's L2, then the
// Infinity Cache, else HBM), the bytes that have to move at each level are divided by that
// level's bandwidth, and the matrix-core time carries the wave-quantisation of the grid.
// The constants are per-chip figures (one Chip struct and a handful of cycle counts in model_cost), not per-layer
// factors.  Bandwidths and capacities are measured or published; the cycle counts (per-iteration and per-tile
// overheads, fill, stall coefficients) were calibrated on exhaustive sweeps of the ResNet-50-shaped layers at batch
// 28, 8 and 1, so on those layers the agreement with the sweeps is in-sample; the out-of-sample check is the second
// layer set of workloads.heldout_layers (other widths, 5x5 and 11x11 filters, strided 3x3), swept with the constants
// frozen.
#include <algorithm>
#include <cmath>
#include <utility>
#include <vector>

#include "ps_internal.h"

namespace ps {

struct ShapeInfo {
    int kt, mt, ring, threads, lds_bytes, group, halo_bytes, baked_only, stationary, lds_3x3, lds_halo, has_5x5, lds_5x5;
};
int list_shapes(int dtype, ShapeInfo *out, int cap);  // api.hip
bool halo_applies(const Dims &dm, const ps_tile &t, int capacity_bytes);  // api.hip
bool kt_admissible(int K, int kt);                                         // api.hip

namespace {

// Per-chip constants (MI355X: 256 CUs in 8 XCDs).  Bandwidths are sustained figures measured with
// streaming microbenchmarks on the device, not spec-sheet peaks.
struct Chip {
    double cus = 256, xcds = 8;
    double clock_hz = 2.4e9;
    double lds_bytes = 160 * 1024;
    double regs_per_simd = 512;               // VGPRs + AGPRs per lane
    double l2_bytes = 4.0 * 1024 * 1024;      // per XCD
    double mall_bytes = 256.0 * 1024 * 1024;  // Infinity Cache
    double hbm_bw = 5.0e12;                   // read+write streaming beyond the Infinity Cache
    double mall_bw = 9.0e12;                  // working set resident in the Infinity Cache
    double l2_bw = 14.0e12;                   // L2 -> LDS, all XCDs
    double atomic_bw = 0.35e12;               // fp32 atomic adds (resolved memory-side across XCDs), payload bytes/s
    double mfma_flop_clk_cu[2] = {256.0, 4096.0};  // f32, bf16
    double steady_eff_general[2] = {0.84, 0.45};  // matrix-core issue efficiency of the general loop (VALU address work)
    double steady_eff_baked = 0.97;           // ... of the loops with a baked filter size (no VALU work)
    double load_latency_clk = 1150.0;         // global load to LDS under load, served from beyond one XCD's L2
    double l2_hit_latency_clk = 700.0;        // ... when the layer stays resident in L2 between launches
    double fill_clk = 4500.0;                 // first loads of a workgroup (nothing to overlap with)
    double fill_clk_16 = 6750.0;              // ... per round of resident workgroups in the 16-bit kernels (with the epilogue's barrier and pass through LDS)
    double launch_us = 1.5;
    double dependent_launch_us = 3.5;         // a kernel that has to wait for the previous one to drain (measured gap)
    double plane_latency_us = 0.3;            // per partial plane: the adding pass reads them one after another
    double reduce_ineff = 2.0;                // the plane-adding pass against streaming bandwidth
};

const Chip kChip;

// The kernels with a baked 1x1, 3x3 or 5x5 filter issue no vector-ALU work in their loop; their loop is unrolled
// over lcm(ring, R*S) batch elements and the range is padded to a multiple of that.  (A 16-bit shape whose ring of
// filter rows does not fit LDS has no 5x5 loop and runs the general one.)
bool baked_filter(const Dims &dm, const ShapeInfo &sh, int nb_split)
{
    if (packs_taps(dm)) return nb_split == dm.NB;  // unsplit only
    if (dm.R == 5 && !sh.has_5x5) return false;
    return dm.R == dm.S && (dm.R == 1 || dm.R == 3 || dm.R == 5) && nb_split % (dm.R * dm.S) == 0;
}

// The pixel-stationary fp32 kernels: 1x1 filters over exactly 4 c-blocks (everything a pixel needs fits in LDS next
// to double-buffered filter slices), images of at least 16 pixels.
bool stationary_applies(const Dims &dm)
{
    return dm.dtype == PS_F32 && dm.R == 1 && dm.S == 1 && dm.Cb == 4 && (long long)dm.P * dm.Q >= 16;
}

// The tap-packed loop runs: an unsplit range of a layer it exists for, unless the 16-bit patch loop takes the tile.
bool packed_runs(const Dims &dm, int nb_split, bool patch) { return packs_taps(dm) && nb_split == dm.NB && !patch; }

// batch elements one loop iteration of the kernel consumes (the 16-bit kernels group several per ring slot;
// their 3x3 variant takes one filter row)
int group_of(const Dims &dm, const ShapeInfo &sh, int nb_split, bool patch = false)
{
    if (dm.dtype == PS_F32) return 1;
    if (packed_runs(dm, nb_split, patch)) return sh.group;
    return baked_filter(dm, sh, nb_split) && dm.R >= 3 ? dm.R : sh.group;  // one filter row (the patch kernel: see model_cost)
}

// batch elements the kernel really iterates over for a range of nb_split (c-block, r, s) triples

int padded_elems(const Dims &dm, const ShapeInfo &sh, int nb_split, bool patch = false)
{
    const int ring = sh.ring;
    int unit = ring;
    if (dm.dtype != PS_F32) {
        const int g = group_of(dm, sh, nb_split, patch);
        // tap-packed: two taps per element, g elements per iteration
        if (packed_runs(dm, nb_split, patch)) return ((dm.R * dm.S + 1) / 2 + g - 1) / g * g;
        // baked 3x3 / 5x5 and the patch loop: whole filter rows per iteration, the loop leaves at a c-block boundary
        if (g == 3 || g == 5) return nb_split;
        unit = ring * g;
    } else if (baked_filter(dm, sh, nb_split)) {
        if (packs_taps(dm)) return (dm.R * dm.S + 3) / 4;  // four taps per element, in one pass of exactly that many iterations
        const int taps = dm.R * dm.S;
        int g = ring, h = taps;
        while (h) { const int r = g % h; g = h; h = r; }
        unit = ring / g * taps;                             // lcm(ring, taps): the unrolled block
        if (taps > 1 && unit <= 50) return nb_split;        // ... which the kernel leaves at a c-block boundary where it is short enough
    }
    return (nb_split + unit - 1) / unit * unit;
}

// batch elements the range holds as the kernel counts them: the tap-packed loops run their elements (in whole
// iterations) whatever the ring depth
int logical_elems(const Dims &dm, const ShapeInfo &sh, int nb_split, bool patch = false)
{
    return packed_runs(dm, nb_split, patch) ? padded_elems(dm, sh, nb_split, patch) : nb_split;
}

// Working sets of the tile's data reuses, and the level each one is served from (the analogue of
// Algorithms 1 and 2): accumulators -> registers, one batch element of pixels and filters -> LDS
// (both by construction of the kernel), the filter slice and input slab shared by the workgroups of
// one XCD -> that XCD's L2 if they fit, else the Infinity Cache, else HBM.  The cost is the time the
// slowest level needs for the bytes it has to move (Eq. 1 with latency folded into per-workgroup
// fill and launch terms), plus a fraction of the second-slowest for imperfect overlap.
// terms, if given, receives the parts the total is made of (us): matrix cores with their per-workgroup overheads,
// traffic into the compute units, traffic beyond L2, and launches plus extra passes.
double model_cost(const Dims &dm, const ps_tile &t, const ShapeInfo &sh, bool with_ws, double *terms = nullptr)
{
    const Chip &c = kChip;
    const double M = (double)dm.M;
    const double n_mt = std::ceil(M / t.mt), n_kt = std::ceil((double)dm.K / t.kt);
    const double nwg = n_mt * n_kt * t.c_split;
    const double nb_split = (double)dm.NB / t.c_split;
    // 16-bit 3x3 / stride 1 / pad 1: the ring-2 rows of a shape run the kernel that stages the input patch once per
    // c-block (two slots of one c-block each) instead of gathering every tap
    const bool patch = sh.halo_bytes > 0 && halo_applies(dm, t, sh.halo_bytes);
    const bool packed = packed_runs(dm, dm.NB / t.c_split, patch);
    const double nb_pad = padded_elems(dm, sh, dm.NB / t.c_split, patch);  // zero elements pad the range
    const bool baked = baked_filter(dm, sh, dm.NB / t.c_split);
    const double es = dm.es;
    const double waves_wg = sh.threads / 64.0;

    // ---- residency --------------------------------------------------------------------------------
    const double tiles_wave = (double)t.kt * t.mt / (waves_wg * 1024.0);  // 32x32 MFMA tiles per wave
    const double regs = 16.0 * tiles_wave + 2.0 * 8.0 * 2.0 * std::sqrt(tiles_wave) + 48.0;
    const double waves_simd = std::max(1.0, std::min(8.0, std::floor(c.regs_per_simd / regs)));
    // LDS footprint of the loop that will run: the 16-bit 3x3 loops (one filter row per ring slot, or the patch
    // kernel's two c-block slots) differ from the general loop's
    double lds_used = sh.lds_bytes;
    if (patch && sh.lds_halo > 0)
        lds_used = sh.lds_halo;
    else if (dm.dtype != PS_F32 && baked && dm.R == 3 && !packed && sh.lds_3x3 > 0)
        lds_used = sh.lds_3x3;
    else if (dm.dtype != PS_F32 && baked && dm.R == 5 && !packed && sh.lds_5x5 > 0)
        lds_used = sh.lds_5x5;
    double occ = std::floor(c.lds_bytes / lds_used);
    occ = std::max(1.0, std::min(occ, std::floor(waves_simd * 4.0 / waves_wg)));

    // ---- matrix cores -----------------------------------------------------------------------------
    // Work is quantised per SIMD: a CU gets ceil(nwg / CUs) workgroups, each SIMD of it a quarter of
    // their waves, and a wave owns `tiles_wave` 32x32 accumulator tiles for the whole batch range.
    const double per_cu = std::ceil(nwg / c.cus);
    // Waves per SIMD.  The hardware hands a workgroup consecutive SIMDs of its cyclic order [0, 2, 1, 3] and starts the
    // next workgroup of the compute unit ONE position further, not one workgroup's width: four- and eight-wave
    // workgroups fill all SIMDs evenly, but two-wave workgroups overlap by one SIMD (measured by recording the
    // hardware id of every wave: two such workgroups on a compute unit put two waves on one SIMD and none on another;
    // six put 4, 3, 3, 2).  A SIMD runs its waves' MFMA streams one after another, so the fullest SIMD decides.
    double per_simd = std::ceil(per_cu * waves_wg / 4.0);
    if (waves_wg == 2.0) {
        const double rem = std::fmod(per_cu, 4.0);
        per_simd = std::floor(per_cu / 4.0) * 2.0 + std::min(2.0, rem);
    }
    const double mfma_clk = dm.dtype == PS_F32 ? 64.0 * 8.0 : 32.0;  // per 32x32 tile per batch element
    const double eff = baked ? c.steady_eff_baked : c.steady_eff_general[dm.dtype == PS_F32 ? 0 : 1];
    // tap-packed over at most 3 channels: the MFMA steps of the zero lane are left out
    const double lane_skip = dm.dtype == PS_F32 && packed && dm.C <= 3 ? 0.75 : 1.0;
    const double clk_wave = tiles_wave * mfma_clk * lane_skip * nb_pad / eff;
    // per batch element a wave also pays a barrier and the issue of its loads and LDS reads; with a
    // single resident wave per SIMD nothing hides that
    const double waves_res = std::min(per_simd, std::max(1.0, std::floor(occ * waves_wg / 4.0)));
    const double grp = patch ? 9.0 : group_of(dm, sh, dm.NB / t.c_split, patch);  // batch elements per loop iteration
    const double n_iter = nb_pad / grp;
    // (a lone 16-bit wave cannot hide its barrier behind its own short MFMA stream; an fp32 one can)
    const bool f32 = dm.dtype == PS_F32;
    double clk_iter_overhead = (f32 ? 40.0 : waves_res >= 2 ? 150.0 : 220.0) * n_iter;
    // a load issued in iteration b must have landed (ring - 1) iterations later: the part of the latency
    // the ring does not cover stalls every wave of the SIMD, and latency varies, so a thin margin still costs
    const double clk_iter = tiles_wave * mfma_clk * grp / eff * waves_res;  // wall clock of one iteration
    // Latency of a global load into LDS.  Under repeated launches (how layers are timed, and how an inference loop runs
    // them) a layer whose per-XCD share -- an eighth of input and output, all filters -- fits the XCD's L2 is served
    // from L2 on every launch after the first; larger layers come from beyond L2 under load.  fp32 only: the 16-bit
    // cost below folds latency into a coefficient that was calibrated together with the one constant.
    const double in_b0 = (double)dm.N * dm.Cb * dm.H * dm.W * 16.0 * dm.es;
    const double wt_b0 = (double)dm.Kb * 16.0 * dm.Cb * 16.0 * dm.R * dm.S * dm.es;
    const bool l2_resident = (in_b0 + M * dm.K * 4.0) / c.xcds + wt_b0 <= c.l2_bytes;
    double latency = f32 && l2_resident ? c.l2_hit_latency_clk : c.load_latency_clk;
    if (packed) {
        // A tap-packed gather uses 16 bytes of every pixel it touches, so one load instruction (1 KB into LDS) passes
        // more 64-byte lines through the unit's L1, which takes one line per clock, than the 16 of an ordinary load:
        // the input pixels between its first and last (pixel, tap), i.e. up to 64 at stride 4.  The loads of one batch
        // element from all resident workgroups queue there, and what the queue takes beyond fully used lines is
        // latency the ring has to cover.
        const double px_instr = f32 ? 16.0 : 32.0, taps_instr = f32 ? 4.0 : 2.0, px_line = f32 ? 1.0 : 2.0;
        const double lines = std::min(64.0, ((px_instr - 1.0) * dm.stride + taps_instr) / px_line);
        latency += std::min(occ, per_cu) * std::max(0.0, lines - 16.0) * (t.mt / px_instr);
    }
    const double cover = (t.ring - 1) * clk_iter / latency;
    const double stall = std::max(0.0, latency / (t.ring - 1) - clk_iter) + (f32 ? 0.10 : 0.50) * clk_iter * std::exp(-cover);
    if (patch) {
        // one barrier per c-block (9 taps) and the next c-block requested a whole iteration ahead: the hard part of
        // the stall (latency the ring does not cover) does not arise; a lone wave still pays for its barrier
        clk_iter_overhead = (waves_res >= 2 ? 40.0 : 220.0) * n_iter + (stall - std::max(0.0, latency / (t.ring - 1) - clk_iter)) * n_iter / waves_res;
    } else {
        clk_iter_overhead += stall * n_iter / waves_res;
    }
    // Per workgroup, outside its MFMA stream: address set-up, first fragment reads and the stores of its tile.  The
    // waves of a SIMD run their streams one after another and a pending MFMA holds the SIMD's issue port, so this
    // work is not hidden by the other workgroups on the compute unit; it grows with the accumulator tiles a wave
    // has to store (atomics cost more per tile), and in the 16x16-tile kernels with the pixel tiles every wave
    // walks over.  The first loads of a launch have nothing to overlap with at all (fill_clk, once).
    const double clk_tile = t.c_split > 1 && !with_ws ? 1900.0 : (sh.baked_only ? 900.0 : 1250.0);
    const double clk_wg = (tiles_wave * clk_tile + (sh.baked_only ? 200.0 * (t.mt / 16.0) : 0.0)) * waves_wg / 4.0;  // per SIMD
    double t_mfma;
    if (sh.stationary) {
        // One workgroup walks over kt / 64 output tiles with its pixels resident: set-up and the first loads (all
        // pixels, two filter slices; every workgroup of the launch asks at once) are paid once per launch, and a
        // tile boundary costs the issue of its stores (measured 3.2 us, and 0.3 us per 176-pixel tile).
        const double tiles = t.kt / 64.0;
        const double clk_boundary = tiles * (150.0 + 90.0 * t.mt / 16.0);
        t_mfma = (per_simd * (clk_wave + clk_iter_overhead) + 7700.0 + per_cu * clk_boundary) / c.clock_hz;
    } else if (f32) {
        // Workgroups that share a compute unit hide part of each other's set-up and stores.
        const double hidden = 1.0 + 0.5 * (std::min(occ, per_cu) - 1.0);
        // (a deeper ring takes longer to fill, per workgroup: 150 clk per extra slot, hidden like the rest of the set-up)
        t_mfma = (per_simd * (clk_wave + clk_iter_overhead) + c.fill_clk +
                  per_cu * (clk_wg + (t.ring - 2) * 150.0) / hidden) / c.clock_hz;
    } else {
        // 16-bit tiles are short enough that their set-up and stores mostly hide behind other workgroups; what
        // shows is the fill of every round of resident workgroups
        const double rounds = std::ceil(per_cu / occ);
        const double clk_epi = tiles_wave * (t.c_split > 1 && !with_ws ? 900.0 : 250.0);
        t_mfma = (per_simd * (clk_wave + clk_iter_overhead + clk_epi) + rounds * c.fill_clk_16 +
                  per_cu * (t.ring - 2) * 250.0) / c.clock_hz;
    }

    // ---- bytes that cross each level --------------------------------------------------------------
    const double in_bytes = (double)dm.N * dm.Cb * dm.H * dm.W * 16.0 * es;
    const double wt_bytes = (double)dm.Kb * 16.0 * dm.Cb * 16.0 * dm.R * dm.S * es;
    const double out_bytes = M * dm.K * 4.0;
    // into the CUs: every workgroup gathers its pixels and its filter slice once per batch element
    double cu_bytes = nwg * nb_pad * 16.0 * es * (t.mt + t.kt);
    if (patch) {
        // rows of the tile plus a row above and below, pitch W + 2, once per c-block; filters as before
        const double rows = std::ceil((double)t.mt / dm.Q) + 3.0;
        cu_bytes = nwg * (nb_pad / 9.0) * (rows * (dm.W + 2) * 16.0 * es + 9.0 * 16.0 * es * t.kt);
    }
    // what one XCD's resident workgroups touch between two uses of the same data
    const double wg_xcd = std::min(nwg, c.cus * occ) / c.xcds;
    double xcd_ws;
    if (t.raster == 0)  // k tiles fastest: neighbours share pixels, all of them need every filter
        xcd_ws = wt_bytes + in_bytes * std::min(1.0, wg_xcd / n_kt / n_mt);
    else                // pixel tiles fastest: neighbours share one filter slice
        xcd_ws = wt_bytes * std::min(1.0, std::ceil(wg_xcd / n_mt) / n_kt) + in_bytes * std::min(1.0, wg_xcd / n_mt);
    const double total = in_bytes + wt_bytes + out_bytes;
    double hbm = total + wt_bytes * (c.xcds - 1);  // compulsory: every XCD pulls the filters once
    double beyond_l2 = hbm;
    if (xcd_ws > c.l2_bytes) {
        // re-reads miss L2: the operand that is not shared by neighbours is refetched per workgroup
        const double refetch = (t.raster == 0 ? nwg * nb_pad * 16.0 * es * t.kt : nwg * nb_pad * 16.0 * es * t.mt);
        beyond_l2 += refetch * std::min(1.0, (xcd_ws - c.l2_bytes) / xcd_ws);
    }
    const double far_bw = total <= 0.7 * c.mall_bytes ? c.mall_bw : c.hbm_bw;
    // L2 -> LDS is a per-compute-unit rate (the chip-wide figure over all of them): the compute unit with the most
    // workgroups decides, which on an under-filled grid is far more than an even share.
    const double t_near = (cu_bytes / nwg) * std::max(1.0, nwg / c.cus) / (c.l2_bw / c.cus), t_far = beyond_l2 / far_bw;
    double t_mem = std::max(t_near, t_far);
    double t_extra = 0.0;
    if (t.c_split > 1 && !with_ws) {
        t_mem += out_bytes * t.c_split / c.atomic_bw;   // atomic accumulation of partial tiles
        t_extra = out_bytes / c.hbm_bw * 1e6 + c.launch_us;  // the clearing pass
    } else if (t.c_split > 1) {
        t_mem += out_bytes * t.c_split / far_bw;  // partial planes written once ...
        t_extra = out_bytes * (t.c_split + 1.0) / far_bw * 1e6 * c.reduce_ineff + c.dependent_launch_us +
                  c.plane_latency_us * t.c_split;  // ... and added by a second pass
    }
    // Filters larger than one XCD's L2: with the channel tiles fastest every XCD streams all of them through its L2
    // over and over, with the pixel tiles fastest it stays on the slices of a few channel tiles.  Where the two
    // orders otherwise cost the same this decides (measured 3x3, 512 channels, 7x7 images, bf16: 19.3 against 16.2 us).
    const double order_bias = (wt_bytes > c.l2_bytes && t.raster == 0 && n_kt >= c.xcds && n_mt > 1) ? 1.02 : 1.0;
    if (terms) {
        terms[0] = t_mfma * 1e6;
        terms[1] = t_near * 1e6;
        terms[2] = (t_far + (t_mem - std::max(t_near, t_far))) * 1e6;  // with the partial tiles of a split reduction
        terms[3] = c.launch_us + t_extra;
    }
    return (std::max(t_mfma, t_mem) + 0.12 * std::min(t_mfma, t_mem)) * 1e6 * order_bias + c.launch_us + t_extra;
}

struct Cand {
    ps_tile t;
    ShapeInfo sh;
};

void enumerate(const Dims &dm, std::vector<Cand> &out)
{
    ShapeInfo shapes[128];
    const int ns = list_shapes(dm.dtype, shapes, 128);
    static const int splits[] = {1, 2, 3, 4, 6, 8, 9, 12, 16};
    for (int i = 0; i < ns; ++i) {
        const ShapeInfo &s = shapes[i];
        if (!kt_admissible(dm.K, s.kt)) continue;
        if (s.mt > 64 && s.mt >= 2 * dm.M) continue;
        const long long n_mt = (dm.M + s.mt - 1) / s.mt;
        const long long base_wg = n_mt * ((dm.K + s.kt - 1) / s.kt);
        if (s.baked_only && !((dm.R == dm.S && (dm.R == 1 || dm.R == 3 || dm.R == 5)) || (packs_taps(dm) && dm.C <= 3 && !s.stationary)))
            continue;
        if (s.stationary && !stationary_applies(dm)) continue;
        for (int sp : splits) {
            if (dm.NB % sp != 0) continue;
            if (s.baked_only && sp > 1) continue;  // no atomic epilogue in these kernels
            const int nbs = dm.NB / sp;
            // stage depth: keep the depths that divide the split's range; if none of this tile's
            // compiled depths does, keep only the shallowest (its ragged last stage is zero-filled)
            bool any_exact = false;
            int shallowest = 1 << 30;
            for (int j = 0; j < ns; ++j)
                if (shapes[j].kt == s.kt && shapes[j].mt == s.mt) {
                    if (padded_elems(dm, shapes[j], nbs) == logical_elems(dm, shapes[j], nbs)) any_exact = true;
                    shallowest = std::min(shallowest, shapes[j].ring);
                }
            const bool exact = padded_elems(dm, s, nbs) == logical_elems(dm, s, nbs);
            if (any_exact ? !exact : s.ring != shallowest) continue;
            if (sp > 1 && base_wg * sp > 8 * 256) continue;  // split only under-filled grids
            for (int raster = 0; raster < 2; ++raster) {
                if (raster == 1 && (n_mt == 1 || dm.K <= s.kt)) continue;
                Cand c;
                c.t.kt = s.kt; c.t.mt = s.mt; c.t.ring = s.ring; c.t.c_split = sp; c.t.raster = raster;
                c.sh = s;
                out.push_back(c);
            }
        }
    }
}

}  // namespace
}  // namespace ps

using namespace ps;

extern "C" int ps_tile_count(const ps_conv_desc *d)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    std::vector<Cand> c;
    enumerate(dm, c);
    return (int)c.size();
}

extern "C" int ps_tile_get(const ps_conv_desc *d, int idx, ps_tile *t)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!t) return PS_EINVAL;
    std::vector<Cand> c;
    enumerate(dm, c);
    if (idx < 0 || idx >= (int)c.size()) return PS_EINVAL;
    *t = c[idx].t;
    return PS_OK;
}

static double cost_of(const ps_conv_desc *d, const ps_tile *t, bool with_ws)
{
    Dims dm;
    if (make_dims(d, &dm) != PS_OK || !t || ps_tile_valid(d, t) != PS_OK) return -1.0;
    ShapeInfo shapes[128];
    const int ns = list_shapes(dm.dtype, shapes, 128);
    for (int i = 0; i < ns; ++i)
        if (shapes[i].kt == t->kt && shapes[i].mt == t->mt && shapes[i].ring == t->ring)
            return model_cost(dm, *t, shapes[i], with_ws);
    return -1.0;
}

extern "C" int ps_tile_level_times_ws(const ps_conv_desc *d, const ps_tile *t, double times_us[4])
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!t || !times_us) return PS_EINVAL;
    if ((rc = ps_tile_valid(d, t)) != PS_OK) return rc;
    ShapeInfo shapes[128];
    const int ns = list_shapes(dm.dtype, shapes, 128);
    for (int i = 0; i < ns; ++i)
        if (shapes[i].kt == t->kt && shapes[i].mt == t->mt && shapes[i].ring == t->ring) {
            model_cost(dm, *t, shapes[i], true, times_us);
            return PS_OK;
        }
    return PS_EUNSUPPORTED;
}

extern "C" double ps_tile_cost_us(const ps_conv_desc *d, const ps_tile *t) { return cost_of(d, t, false); }
extern "C" double ps_tile_cost_ws_us(const ps_conv_desc *d, const ps_tile *t) { return cost_of(d, t, true); }

static int select_best(const ps_conv_desc *d, bool with_ws, size_t ws_bytes, ps_tile *best, double *modelled_us)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!best) return PS_EINVAL;
    std::vector<Cand> c;
    enumerate(dm, c);
    double bu = 1e300;
    int bi = -1;
    for (size_t i = 0; i < c.size(); ++i) {
        bool ws = with_ws;
        if (with_ws && c[i].t.c_split > 1 &&
            (size_t)c[i].t.c_split * (size_t)dm.M * dm.K * 4 > ws_bytes)
            continue;  // its partial planes do not fit the caller's workspace
        const double u = model_cost(dm, c[i].t, c[i].sh, ws);
        if (u < bu) {
            bu = u;
            bi = (int)i;
        }
    }
    if (bi < 0) return PS_EUNSUPPORTED;
    *best = c[bi].t;
    if (modelled_us) *modelled_us = bu;
    return PS_OK;
}

extern "C" int ps_tile_rank_ws(const ps_conv_desc *d, size_t workspace_bytes, int k, ps_tile *tiles, double *modelled_us)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (k <= 0 || !tiles) return PS_EINVAL;
    std::vector<Cand> c;
    enumerate(dm, c);
    std::vector<std::pair<double, int>> order;
    for (size_t i = 0; i < c.size(); ++i) {
        if (c[i].t.c_split > 1 && (size_t)c[i].t.c_split * (size_t)dm.M * dm.K * 4 > workspace_bytes) continue;
        order.emplace_back(model_cost(dm, c[i].t, c[i].sh, true), (int)i);
    }
    if (order.empty()) return PS_EUNSUPPORTED;
    std::stable_sort(order.begin(), order.end());  // ties keep the enumeration order, as the k = 1 pick does
    const int n = std::min<int>(k, (int)order.size());
    for (int j = 0; j < n; ++j) {
        tiles[j] = c[order[j].second].t;
        if (modelled_us) modelled_us[j] = order[j].first;
    }
    return n;
}

extern "C" int ps_tile_select(const ps_conv_desc *d, ps_tile *best, double *modelled_us)
{
    return select_best(d, false, 0, best, modelled_us);
}

extern "C" int ps_tile_select_ws(const ps_conv_desc *d, size_t workspace_bytes, ps_tile *best, double *modelled_us)
{
    return select_best(d, true, workspace_bytes, best, modelled_us);
}
