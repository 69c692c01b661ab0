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
// All constants are per-chip figures, not fitted per layer.
#include <algorithm>
#include <cmath>
#include <vector>

#include "ps_internal.h"

namespace ps {

struct ShapeInfo {
    int kt, mt, bpp, threads, lds_bytes;
};
int list_shapes(int dtype, ShapeInfo *out, int cap);  // api.hip

namespace {

struct Chip {
    double cus = 256, xcds = 8;
    double clock_hz = 2.4e9;
    double lds_bytes = 160 * 1024;
    double l2_bytes = 4.0 * 1024 * 1024;      // per XCD
    double mall_bytes = 256.0 * 1024 * 1024;  // Infinity Cache
    double hbm_bw = 8.0e12 * 0.80;            // sustained fraction of 8 TB/s
    double mall_bw = 14.0e12;
    double l2_bw = 2048.0 * 8 * 2.4e9 * 0.5;  // 2 KB/clk/XCD peak, half sustained
    double lds_bw_cu = 128.0;                 // bytes/clk/CU
    double mfma_flop_clk_cu_f32 = 256.0;
    double mfma_flop_clk_cu_bf16 = 4096.0;
    double launch_us = 2.0;                   // grid launch + drain
    double stage_latency_clk = 2500.0;        // first global->LDS fill of a workgroup
    int max_waves_simd = 2;                   // register budget of these kernels
};

const Chip kChip;

struct Model {
    double us;
};

double model_cost(const Dims &dm, const ps_tile &t, const ShapeInfo &sh)
{
    const Chip &c = kChip;
    const double M = (double)dm.M;
    const double n_mt = std::ceil(M / t.mt), n_kt = std::ceil((double)dm.K / t.kt);
    const double nwg = n_mt * n_kt * t.c_split;
    const double nb_split = (double)dm.NB / t.c_split;
    const double nstage = std::ceil(nb_split / t.bpp);
    const double es = dm.es;

    // residency: workgroups per CU allowed by LDS and by the register budget
    const double waves_wg = sh.threads / 64.0;
    double occ = std::floor(c.lds_bytes / sh.lds_bytes);
    occ = std::min(occ, std::floor(c.max_waves_simd * 4.0 / waves_wg));
    occ = std::max(occ, 1.0);

    // matrix-core time of one workgroup (staged work includes the ragged last stage)
    const double flop_wg = 2.0 * t.mt * t.kt * 16.0 * nstage * t.bpp;
    const double rate = dm.dtype == PS_F32 ? c.mfma_flop_clk_cu_f32 : c.mfma_flop_clk_cu_bf16;
    // LDS bytes read per workgroup stage: every wave reads its pixel rows and its filter columns
    const int wk = sh.kt >= 128 ? 2 : (sh.kt == 64 ? (sh.mt >= 256 ? 1 : 2) : 1);
    const double wm = waves_wg / wk;
    const double lds_rd = t.bpp * 16.0 * es * (t.mt * wk + t.kt * wm);
    const double lds_wr = t.bpp * 16.0 * es * (t.mt + t.kt);
    const double clk_mfma_stage = 2.0 * t.mt * t.kt * 16.0 * t.bpp / rate;
    const double clk_lds_stage = (lds_rd + lds_wr) / c.lds_bw_cu;
    // with one resident workgroup nothing overlaps the barrier and LDS phases
    const double overlap = occ >= 2 ? 1.0 : 0.0;
    const double clk_stage = overlap > 0 ? std::max(clk_mfma_stage, clk_lds_stage) + 0.05 * clk_mfma_stage
                                         : clk_mfma_stage + clk_lds_stage + 200.0;
    const double clk_wg = nstage * clk_stage;
    const double clk_epi = t.mt * t.kt * 4.0 / 64.0 * (t.c_split > 1 ? 4.0 : 1.0) / waves_wg;  // store issue

    // wave quantisation: CUs that get the most workgroups finish last
    const double per_cu = std::ceil(nwg / c.cus);
    const double fill = c.stage_latency_clk * (occ >= 2 ? std::ceil(per_cu / occ) * 0.5 : per_cu);
    const double t_mfma = (per_cu * (clk_wg + clk_epi) + fill) / c.clock_hz;
    (void)flop_wg;

    // bytes that cross each level
    const double in_bytes = (double)dm.N * dm.Cb * dm.H * dm.W * 16.0 * es;
    const double wt_bytes = (double)dm.K * dm.Cb * 16.0 * dm.R * dm.S * es;
    const double out_bytes = M * dm.K * 4.0;
    // traffic into the CUs: every workgroup gathers its pixels once per batch element
    const double cu_in = nwg * t.mt * 16.0 * es * nb_split;
    const double cu_wt = nwg * t.kt * 16.0 * es * nb_split;
    // working sets that decide where the re-reads are served from
    //  - filter slice shared by the workgroups of one XCD
    const double wt_ws = (t.raster == 0 ? wt_bytes : wt_bytes / n_kt);
    //  - input slab one XCD's resident tiles touch
    const double in_ws = in_bytes / c.xcds;
    double l2_served = 0, mall_served = 0, hbm = in_bytes + wt_bytes + out_bytes * (t.c_split > 1 ? 2.0 : 1.0);
    const double ws = wt_ws + in_ws;
    if (ws <= c.l2_bytes) {
        l2_served = cu_in + cu_wt;
        hbm += wt_bytes * (c.xcds - 1);  // each XCD pulls the filters once
    } else if (in_bytes + wt_bytes + out_bytes <= c.mall_bytes) {
        l2_served = 0.5 * (cu_in + cu_wt);
        mall_served = 0.5 * (cu_in + cu_wt);
    } else {
        mall_served = 0.5 * (cu_in + cu_wt);
        hbm += 0.5 * (cu_in + cu_wt);
    }
    if (t.c_split > 1) mall_served += out_bytes * t.c_split;  // atomic traffic
    const double t_mem = std::max({(l2_served + mall_served) / c.l2_bw, mall_served / c.mall_bw, hbm / c.hbm_bw});

    return (std::max(t_mfma, t_mem) + 0.15 * std::min(t_mfma, t_mem)) * 1e6 + c.launch_us * (t.c_split > 1 ? 2 : 1);
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
        if ((dm.K + s.kt - 1) / s.kt * s.kt != (dm.K + 31) / 32 * 32) continue;
        if (s.mt > 64 && s.mt >= 2 * dm.M) continue;
        const long long n_mt = (dm.M + s.mt - 1) / s.mt;
        const long long base_wg = n_mt * ((dm.K + s.kt - 1) / s.kt);
        for (int sp : splits) {
            if (dm.NB % sp != 0) continue;
            const int nbs = dm.NB / sp;
            // stage depth: keep the depths that divide the split's range; if none of this tile's
            // compiled depths does, keep only the shallowest (its ragged last stage is zero-filled)
            bool any_exact = false;
            int shallowest = 1 << 30;
            for (int j = 0; j < ns; ++j)
                if (shapes[j].kt == s.kt && shapes[j].mt == s.mt) {
                    if (shapes[j].bpp <= nbs && nbs % shapes[j].bpp == 0) any_exact = true;
                    shallowest = std::min(shallowest, shapes[j].bpp);
                }
            const bool exact = s.bpp <= nbs && nbs % s.bpp == 0;
            if (any_exact ? !exact : s.bpp != shallowest) continue;
            if (sp > 1 && base_wg * (sp / 2 > 0 ? sp / 2 : 1) >= 4 * 256) continue;  // split only under-filled grids
            for (int raster = 0; raster < 2; ++raster) {
                if (raster == 1 && (n_mt == 1 || dm.K <= s.kt)) continue;
                Cand c;
                c.t.kt = s.kt; c.t.mt = s.mt; c.t.bpp = s.bpp; c.t.c_split = sp; c.t.raster = raster;
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

extern "C" double ps_tile_cost_us(const ps_conv_desc *d, const ps_tile *t)
{
    Dims dm;
    if (make_dims(d, &dm) != PS_OK || !t || ps_tile_valid(d, t) != PS_OK) return -1.0;
    ShapeInfo shapes[128];
    const int ns = list_shapes(dm.dtype, shapes, 128);
    for (int i = 0; i < ns; ++i)
        if (shapes[i].kt == t->kt && shapes[i].mt == t->mt && shapes[i].bpp == t->bpp)
            return model_cost(dm, *t, shapes[i]);
    return -1.0;
}

extern "C" int ps_tile_select(const ps_conv_desc *d, ps_tile *best, double *modelled_us)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!best) return PS_EINVAL;
    std::vector<Cand> c;
    enumerate(dm, c);
    if (c.empty()) return PS_EUNSUPPORTED;
    double bu = 1e300;
    int bi = 0;
    for (size_t i = 0; i < c.size(); ++i) {
        const double u = model_cost(dm, c[i].t, c[i].sh);
        if (u < bu) {
            bu = u;
            bi = (int)i;
        }
    }
    *best = c[bi].t;
    if (modelled_us) *modelled_us = bu;
    return PS_OK;
}
