// C ABI entry points: descriptor validation, size queries, convolution launch.
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <shared_mutex>
#include <unordered_map>

#include "conv_fwd_kernel.h"

namespace ps {

const ShapeEntry *f32_shapes(int *count);
const ShapeEntry *bf16_shapes(int *count);

int make_dims(const ps_conv_desc *d, Dims *o)
{
    if (!d || !o) return PS_EINVAL;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 ||
        d->stride <= 0 || d->pad < 0)
        return PS_EINVAL;
    if (d->dtype != PS_F32 && d->dtype != PS_BF16) return PS_EUNSUPPORTED;
    const long long hp = (long long)d->H + 2LL * d->pad - d->R, wp = (long long)d->W + 2LL * d->pad - d->S;
    if (hp < 0 || wp < 0) return PS_EINVAL;
    if (d->K % kBlock != 0) return PS_EUNSUPPORTED;
    // No field of a tensor that stays below 2 GiB can reach 2^27, and strides or pads beyond 2^20 have no use: refusing
    // them here keeps every later product inside 64 bits (and the sums above inside 32).
    const int32_t big = 1 << 27;
    if (d->N > big || d->C > big || d->H > big || d->W > big || d->K > big || d->R > big || d->S > big ||
        d->stride > (1 << 20) || d->pad > (1 << 20))
        return PS_EUNSUPPORTED;
    o->N = d->N; o->C = d->C; o->H = d->H; o->W = d->W; o->K = d->K; o->R = d->R; o->S = d->S;
    o->stride = d->stride; o->pad = d->pad; o->dtype = d->dtype;
    o->es = d->dtype == PS_F32 ? 4 : 2;
    o->P = (int)(hp / d->stride) + 1;
    o->Q = (int)(wp / d->stride) + 1;
    o->Cb = (d->C + kBlock - 1) / kBlock;
    o->Kb = d->K / kBlock;
    // 32-bit byte offsets inside the kernels: every blocked tensor must stay below 2 GiB (sizes compared as doubles:
    // four factors of up to 2^27 do not fit 64-bit integers, and the comparison needs no exactness at that size)
    const double lim = 2147483647.0;
    const double nb_d = (double)o->Cb * d->R * d->S;
    const double m_d = (double)d->N * o->P * o->Q;
    const double in_b = (double)d->N * o->Cb * d->H * d->W * kBlock * o->es;
    const double wt_b = (double)o->Kb * nb_d * kBlock * kBlock * o->es;
    const double out_b = m_d * d->K * 4;
    if (nb_d > (double)(1 << 24) || in_b > lim || wt_b > lim || out_b > lim) return PS_EUNSUPPORTED;
    const long long nb = (long long)o->Cb * d->R * d->S;
    o->M = (long long)d->N * o->P * o->Q;
    o->NB = (int)nb;
    return PS_OK;
}

// Square filter over few input channels (the first layer of an image network): the fp32 kernels pack 4 taps x 4
// channels into one 16-lane batch element (3x3, 5x5, 7x7, 11x11 over C <= 3; 7x7 also over C = 4), the 16-bit ones
// 2 taps x 8 channels (the same sides, C <= 8).
bool packs_taps(const Dims &dm)
{
    if (dm.R != dm.S) return false;
    if (dm.dtype == PS_F32) return packed_side_code(dm.R, dm.C) != 0;
    return dm.C <= 8 && (dm.R == 3 || dm.R == 5 || dm.R == 7 || dm.R == 11);
}

const ShapeEntry *find_shape(int dtype, int kt, int mt, int ring)
{
    int n = 0;
    const ShapeEntry *tab = dtype == PS_F32 ? f32_shapes(&n) : bf16_shapes(&n);
    for (int i = 0; i < n; ++i)
        if (tab[i].kt == kt && tab[i].mt == mt && tab[i].ring == ring) return &tab[i];
    return nullptr;
}

// Output channels are padded to whole 32-wide MFMA tiles anyway; a channel tile kt may add to that padding at most a
// quarter of what it then covers (K = 96 runs as two 64-channel tiles, K = 64 never as one 128-channel tile).
bool kt_admissible(int K, int kt)
{
    const int padded = (K + kt - 1) / kt * kt, base = (K + 31) / 32 * 32;
    return padded == base || (padded - base) * 4 <= padded;
}

struct ShapeInfo {
    int kt, mt, ring, threads, lds_bytes, group, halo_bytes, baked_only, stationary, lds_3x3, lds_halo, has_5x5, lds_5x5;
};

int list_shapes(int dtype, ShapeInfo *out, int cap)
{
    int n = 0;
    const ShapeEntry *tab = dtype == PS_F32 ? f32_shapes(&n) : bf16_shapes(&n);
    n = n < cap ? n : cap;
    for (int i = 0; i < n; ++i) out[i] = ShapeInfo{tab[i].kt, tab[i].mt, tab[i].ring, tab[i].threads, tab[i].lds_bytes, tab[i].group,
                                                   tab[i].launch_halo ? tab[i].halo_bytes : 0, tab[i].launch == nullptr, tab[i].stationary,
                                                   tab[i].lds_3x3, tab[i].lds_halo, tab[i].launch_5x5 != nullptr, tab[i].lds_5x5};
    return n;
}

int tile_valid(const Dims &dm, const ps_tile &t)
{
    if (t.kt <= 0 || t.mt <= 0 || t.ring <= 0 || t.c_split <= 0 || (t.raster != 0 && t.raster != 1))
        return PS_EUNSUPPORTED;
    const ShapeEntry *sh = find_shape(dm.dtype, t.kt, t.mt, t.ring);
    if (!sh) return PS_EUNSUPPORTED;
    // shapes without a loop for a runtime filter size and without an atomic epilogue: 1x1 and 3x3, unsplit
    if (!sh->launch && !(t.c_split == 1 && ((dm.R == dm.S && (dm.R == 1 || dm.R == 3 || dm.R == 5)) ||
                                            (packs_taps(dm) && dm.C <= 3 && sh->launch_packed))))
        return PS_EUNSUPPORTED;
    // pixel-stationary shapes: 1x1 filters over exactly 4 c-blocks, images of at least 16 pixels
    if (sh->stationary && !(dm.R == 1 && dm.S == 1 && t.c_split == 1 && dm.Cb == 4 && dm.P * dm.Q >= 16))
        return PS_EUNSUPPORTED;
    if (!kt_admissible(dm.K, t.kt)) return PS_EUNSUPPORTED;
    if (dm.NB % t.c_split != 0) return PS_EUNSUPPORTED;
    const long long n_mt = (dm.M + t.mt - 1) / t.mt;
    if (n_mt * ((dm.K + t.kt - 1) / t.kt) * t.c_split > (1LL << 30)) return PS_EUNSUPPORTED;
    return PS_OK;
}

// The patch kernels serve 3x3 / stride 1 / pad 1 on c-block-aligned ranges, if the extended rows of every pixel
// tile (its rows, one more above and below, two zero rows per image boundary inside it) fit the patch.
bool halo_applies(const Dims &dm, const ps_tile &t, int capacity_bytes)
{
    if (dm.dtype != PS_BF16 || dm.R != 3 || dm.S != 3 || dm.stride != 1 || dm.pad != 1) return false;
    if ((dm.NB / t.c_split) % 9 != 0) return false;
    const long long PQ = (long long)dm.P * dm.Q;
    int worst = 0;
    for (long long m0 = 0; m0 < dm.M; m0 += t.mt) {
        const long long ml = std::min<long long>(m0 + t.mt, dm.M) - 1;
        const long long e0 = (m0 / PQ) * (dm.H + 2) + (m0 % PQ) / dm.Q;
        const long long e1 = (ml / PQ) * (dm.H + 2) + (ml % PQ) / dm.Q + 2;
        worst = std::max(worst, (int)(e1 - e0 + 1));
    }
    return (long long)worst * (dm.W + 2) * 32 <= capacity_bytes;
}

// Which loop runs a tile: the filter size is baked into the loop when a specialised kernel exists and the
// (split) range falls on c-block boundaries.
int kernel_variant(const Dims &dm, const ps_tile &t, const ShapeEntry &sh)
{
    const int nb_split = dm.NB / t.c_split;
    if (sh.stationary) return PS_KERNEL_STATIONARY_1X1;  // (tile_valid admits these shapes for nothing else)
    if (sh.launch_halo && halo_applies(dm, t, sh.halo_bytes)) return PS_KERNEL_PATCH_3X3;
    if (packs_taps(dm) && t.c_split == 1 && sh.launch_packed) return PS_KERNEL_PACKED_TAPS;
    if (dm.R == dm.S && nb_split % (dm.R * dm.S) == 0) {
        if (dm.R == 1 && sh.launch_1x1) return PS_KERNEL_1X1;
        if (dm.R == 3 && sh.launch_3x3) return PS_KERNEL_3X3;
        if (dm.R == 5 && sh.launch_5x5) return PS_KERNEL_5X5;
    }
    return PS_KERNEL_GENERAL;
}

// Everything a launch of tile `t` on one descriptor needs, prepared once: which loop runs, its grid and its
// arguments except the caller's pointers.
struct Plan {
    Dims dm;
    ps_tile t;
    ConvArgs a;
    LaunchFn fn;
    unsigned grid;
    int variant;
    size_t ws_need;  // bytes of partial planes a split reduction stores when a workspace is lent
};

int build_plan(const Dims &dm, const ps_tile &t, Plan *pl)
{
    int rc = tile_valid(dm, t);
    if (rc != PS_OK) return rc;
    const ShapeEntry *sh = find_shape(dm.dtype, t.kt, t.mt, t.ring);
    pl->dm = dm;
    pl->t = t;
    ConvArgs &a = pl->a;
    a = ConvArgs{};
    a.cin = dm.C;
    a.H = dm.H; a.W = dm.W; a.Cb = dm.Cb; a.Kb = dm.Kb; a.R = dm.R; a.S = dm.S;
    a.stride = dm.stride; a.pad = dm.pad; a.Q = dm.Q;
    a.PQ = dm.P * dm.Q;
    a.M = (int)dm.M;
    a.NB = dm.NB;
    a.c_split = t.c_split;
    a.nb_split = dm.NB / t.c_split;
    a.n_mt = (int)((dm.M + t.mt - 1) / t.mt);
    a.n_kt = (dm.K + t.kt - 1) / t.kt;
    a.raster = t.raster;
    a.in_bytes = (unsigned)((size_t)dm.N * dm.Cb * dm.H * dm.W * kBlock * dm.es);
    a.wt_bytes = (unsigned)((size_t)dm.Kb * dm.NB * kBlock * kBlock * dm.es);
    a.out_elems = dm.M * dm.K;
    a.plane_bytes = dm.H * dm.W * kBlock * dm.es;
    const auto magic = [](int d) { return d == 1 ? 0xFFFFFFFFu : (unsigned)((1ULL << 32) / (unsigned)d); };
    a.magic_split = magic(a.c_split);
    a.magic_pitch = magic(dm.W + 2);
    a.magic_h2 = magic(dm.H + 2);
    a.magic_inner = magic(a.raster == 0 ? a.n_kt : a.n_mt);
    a.magic_pq = magic(a.PQ);
    a.magic_q = magic(a.Q);
    a.out_bytes = (unsigned)((size_t)dm.M * dm.K * 4);
    pl->variant = kernel_variant(dm, t, *sh);
    pl->fn = sh->launch;
    switch (pl->variant) {
    case PS_KERNEL_1X1:
    case PS_KERNEL_STATIONARY_1X1: pl->fn = sh->launch_1x1; break;
    case PS_KERNEL_3X3: pl->fn = sh->launch_3x3; break;
    case PS_KERNEL_5X5: pl->fn = sh->launch_5x5; break;
    case PS_KERNEL_PATCH_3X3: pl->fn = sh->launch_halo; break;
    case PS_KERNEL_PACKED_TAPS:
        pl->fn = sh->launch_packed;
        // four (two) taps per batch element; a.NB stays R * S for filter addressing
        a.nb_split = dm.dtype == PS_F32 ? (dm.R * dm.S + 3) / 4 : (dm.R * dm.S + 1) / 2;
        break;
    default: break;
    }
    pl->grid = (unsigned)(a.n_mt * a.n_kt * a.c_split);
    pl->ws_need = t.c_split > 1 ? (size_t)t.c_split * (size_t)dm.M * dm.K * 4 : 0;
    return PS_OK;
}

// ---- per-process caches -------------------------------------------------------------------------------------
// Tile selection enumerates and prices every candidate (tens of microseconds, as long as the kernels it
// selects for), and preparing a launch walks the shape table and, for the patch kernels, every pixel tile.  Both
// depend on the descriptor alone, so each result is computed on first use and kept for the life of the process:
// prepared launches are never changed or removed once published; a pick changes only when ps_tile_autotune replaces it
// with a measured winner (readers copy it out under a shared lock); a full table simply stops taking new entries (the
// call then computes its answer as before).
struct CacheKey {
    int32_t v[16];
    bool operator==(const CacheKey &o) const { return std::memcmp(v, o.v, sizeof(v)) == 0; }
};
struct CacheKeyHash {
    size_t operator()(const CacheKey &k) const
    {
        uint64_t h = 1469598103934665603ull;  // FNV-1a over the words
        for (int i = 0; i < 16; ++i) h = (h ^ (uint32_t)k.v[i]) * 1099511628211ull;
        return (size_t)h;
    }
};

template <class V>
class FrozenCache {
public:
    const V *find(const CacheKey &k)
    {
        std::shared_lock<std::shared_mutex> lk(mu_);
        auto it = map_.find(k);
        return it == map_.end() ? nullptr : &it->second;  // node addresses survive rehashing
    }
    // Publishes `v` unless another thread got there first; returns the published entry (nullptr if the table is full).
    const V *publish(const CacheKey &k, const V &v)
    {
        std::unique_lock<std::shared_mutex> lk(mu_);
        auto it = map_.find(k);
        if (it != map_.end()) return &it->second;
        if (map_.size() >= kMaxEntries) return nullptr;
        return &map_.emplace(k, v).first->second;
    }
    // Copy of the entry, taken under the lock (for entries that replace() may change).
    bool lookup(const CacheKey &k, V *out)
    {
        std::shared_lock<std::shared_mutex> lk(mu_);
        auto it = map_.find(k);
        if (it == map_.end()) return false;
        *out = it->second;
        return true;
    }
    // Sets the entry, new or not (false if the table is full and the key is new).
    bool replace(const CacheKey &k, const V &v)
    {
        std::unique_lock<std::shared_mutex> lk(mu_);
        auto it = map_.find(k);
        if (it != map_.end()) {
            it->second = v;
            return true;
        }
        if (map_.size() >= kMaxEntries) return false;
        map_.emplace(k, v);
        return true;
    }
    size_t size()
    {
        std::shared_lock<std::shared_mutex> lk(mu_);
        return map_.size();
    }

private:
    static constexpr size_t kMaxEntries = 1 << 14;
    std::shared_mutex mu_;
    std::unordered_map<CacheKey, V, CacheKeyHash> map_;
};

struct Pick {
    ps_tile t;
    double modelled_us;
};

FrozenCache<Pick> &pick_cache()
{
    static FrozenCache<Pick> c;
    return c;
}
FrozenCache<Plan> &plan_cache()
{
    static FrozenCache<Plan> c;
    return c;
}

CacheKey key_of(const ps_conv_desc &d)
{
    CacheKey k{};
    const int32_t f[10] = {d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.stride, d.pad, d.dtype};
    std::memcpy(k.v, f, sizeof(f));
    return k;
}

// Two environment variables, read when a descriptor is first ranked (the result is cached like any other pick):
//   PS_FORCE_TILE="kt,mt,ring,c_split,raster"  runs that tile on every descriptor it is valid for (and whose
//                                              workspace it fits) instead of the model's pick;
//   PS_DUMP_RANKING=k                          prints the k best candidates with their modelled times to stderr.
void apply_env_overrides(const ps_conv_desc *d, const Dims &dm, int mode, size_t ws_bytes, Pick *p)
{
    if (const char *dump = std::getenv("PS_DUMP_RANKING")) {
        const int k = std::max(1, std::min(64, std::atoi(dump)));
        ps_tile tiles[64];
        double us[64];
        const int n = ps_tile_rank_ws(d, mode ? ws_bytes : 0, k, tiles, us);
        std::fprintf(stderr, "ps ranking N=%d C=%d H=%d W=%d K=%d R=%d S=%d stride=%d pad=%d dtype=%d (%s)\n", d->N, d->C, d->H,
                     d->W, d->K, d->R, d->S, d->stride, d->pad, d->dtype, mode ? "workspace" : "no workspace: unsplit tiles shown");
        for (int i = 0; i < n; ++i)
            std::fprintf(stderr, "  %2d  kt=%d mt=%d ring=%d c_split=%d raster=%d  %.2f us\n", i + 1, tiles[i].kt, tiles[i].mt,
                         tiles[i].ring, tiles[i].c_split, tiles[i].raster, us[i]);
    }
    if (const char *force = std::getenv("PS_FORCE_TILE")) {
        ps_tile t;
        if (std::sscanf(force, "%d,%d,%d,%d,%d", &t.kt, &t.mt, &t.ring, &t.c_split, &t.raster) == 5 && tile_valid(dm, t) == PS_OK) {
            const size_t need = t.c_split > 1 ? (size_t)t.c_split * (size_t)dm.M * dm.K * 4 : 0;
            if (!mode || need <= ws_bytes) {
                p->t = t;
                p->modelled_us = mode ? ps_tile_cost_ws_us(d, &t) : ps_tile_cost_us(d, &t);
            }
        }
    }
}

// The pick for a descriptor: mode 0 = ps_tile_select (split reductions by atomics), mode 1 = ps_tile_select_ws.  What a
// workspace size decides is how many partial planes fit (splits go up to 16), so that count is the key, not the
// byte count.
CacheKey pick_key(const ps_conv_desc *d, const Dims &dm, int mode, size_t ws_bytes)
{
    CacheKey k = key_of(*d);
    k.v[10] = mode;
    k.v[11] = mode ? (int32_t)std::min<size_t>(16, ws_bytes / ((size_t)dm.M * dm.K * 4)) : 0;
    return k;
}

int cached_pick(const ps_conv_desc *d, const Dims &dm, int mode, size_t ws_bytes, ps_tile *t)
{
    const CacheKey k = pick_key(d, dm, mode, ws_bytes);
    Pick p;
    if (pick_cache().lookup(k, &p)) {
        *t = p.t;
        return PS_OK;
    }
    int rc = mode ? ps_tile_select_ws(d, ws_bytes, &p.t, &p.modelled_us) : ps_tile_select(d, &p.t, &p.modelled_us);
    if (rc != PS_OK) return rc;
    apply_env_overrides(d, dm, mode, ws_bytes, &p);
    pick_cache().publish(k, p);
    *t = p.t;
    return PS_OK;
}

// The prepared launch of tile `t` on `d`; *storage is used when the cache cannot take it.
int cached_plan(const ps_conv_desc *d, const Dims &dm, const ps_tile &t, Plan *storage, const Plan **out)
{
    CacheKey k = key_of(*d);
    k.v[10] = t.kt; k.v[11] = t.mt; k.v[12] = t.ring; k.v[13] = t.c_split; k.v[14] = t.raster;
    k.v[15] = 1;  // never equal to a pick's key
    if ((*out = plan_cache().find(k))) return PS_OK;
    const int rc = build_plan(dm, t, storage);
    if (rc != PS_OK) return rc;
    const Plan *pub = plan_cache().publish(k, *storage);
    *out = pub ? pub : storage;
    return PS_OK;
}

int run_plan(const Plan &pl, const void *in, const void *wt, float *out, float *ws, hipStream_t st,
             const float *bias = nullptr, int epi = 0)
{
    ConvArgs a = pl.a;
    a.in = in; a.wt = wt; a.out = out;
    a.bias = bias; a.epi = epi;
    const bool split = pl.t.c_split > 1;
    a.partial = split ? ws : nullptr;
    int rc;
    if (split && !ws) {
        rc = launch_fill_zero(out, (size_t)pl.dm.M * pl.dm.K, st);
        if (rc != PS_OK) return rc;
    }
    pl.fn(a, pl.grid, st);
    rc = hip_status(hipGetLastError());
    if (rc != PS_OK) return rc;
    if (split && ws)
        rc = launch_reduce_planes(ws, out, (size_t)pl.dm.M * pl.dm.K, pl.t.c_split, bias, epi, pl.dm.P * pl.dm.Q,
                                  pl.dm.Kb, st);
    return rc;
}

}  // namespace ps

using namespace ps;

extern "C" int ps_out_dims(const ps_conv_desc *d, int32_t *P, int32_t *Q)
{
    Dims dm;
    if (!P || !Q) return PS_EINVAL;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    *P = dm.P;
    *Q = dm.Q;
    return PS_OK;
}

extern "C" size_t ps_blocked_in_bytes(const ps_conv_desc *d)
{
    Dims dm;
    if (make_dims(d, &dm) != PS_OK) return 0;
    return (size_t)dm.N * dm.Cb * dm.H * dm.W * kBlock * dm.es;
}

extern "C" size_t ps_blocked_wt_bytes(const ps_conv_desc *d)
{
    Dims dm;
    if (make_dims(d, &dm) != PS_OK) return 0;
    return (size_t)dm.Kb * dm.Cb * dm.R * dm.S * kBlock * kBlock * dm.es;
}

extern "C" size_t ps_blocked_out_bytes(const ps_conv_desc *d)
{
    Dims dm;
    if (make_dims(d, &dm) != PS_OK) return 0;
    return (size_t)dm.M * dm.K * 4;
}

// Shared by the convolution entry points: validation, the cached pick when `t` is null (mode as in cached_pick), the
// cached launch plan, the workspace check, the launch.
static int conv_entry(const ps_conv_desc *d, const ps_tile *t, int mode, const void *in_blk, const void *wt_blk,
                      void *out_blk, void *workspace, size_t workspace_bytes, void *stream, const float *bias, int epi)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!in_blk || !wt_blk || !out_blk) return PS_EINVAL;
    if (!aligned16(in_blk) || !aligned16(wt_blk) || !aligned16(out_blk) || !aligned16(workspace)) return PS_EINVAL;
    ps_tile pick;
    if (!t) {
        rc = cached_pick(d, dm, mode, workspace ? workspace_bytes : 0, &pick);
        if (rc != PS_OK) return rc;
        t = &pick;
    }
    Plan storage;
    const Plan *pl = nullptr;
    rc = cached_plan(d, dm, *t, &storage, &pl);
    if (rc != PS_OK) return rc;
    const size_t need = mode ? pl->ws_need : 0;
    if (need > 0 && (!workspace || workspace_bytes < need)) return PS_EINVAL;
    return run_plan(*pl, in_blk, wt_blk, (float *)out_blk, need ? (float *)workspace : nullptr, (hipStream_t)stream, bias,
                    epi);
}

extern "C" int ps_conv2d_fwd_tile(const ps_conv_desc *d, const ps_tile *t, const void *in_blk, const void *wt_blk,
                                  void *out_blk, void *stream)
{
    if (!t) {
        Dims dm;
        const int rc = make_dims(d, &dm);
        return rc != PS_OK ? rc : PS_EINVAL;
    }
    return conv_entry(d, t, 0, in_blk, wt_blk, out_blk, nullptr, 0, stream, nullptr, 0);
}

extern "C" int ps_conv2d_fwd(const ps_conv_desc *d, const void *in_blk, const void *wt_blk, void *out_blk,
                             void *stream)
{
    return conv_entry(d, nullptr, 0, in_blk, wt_blk, out_blk, nullptr, 0, stream, nullptr, 0);
}

extern "C" size_t ps_workspace_bytes(const ps_conv_desc *d, const ps_tile *t)
{
    Dims dm;
    if (make_dims(d, &dm) != PS_OK || !t || tile_valid(dm, *t) != PS_OK) return 0;
    return t->c_split > 1 ? (size_t)t->c_split * (size_t)dm.M * dm.K * 4 : 0;
}

extern "C" int ps_conv2d_fwd_ws(const ps_conv_desc *d, const ps_tile *t, const void *in_blk, const void *wt_blk,
                                void *out_blk, void *workspace, size_t workspace_bytes, void *stream)
{
    return conv_entry(d, t, 1, in_blk, wt_blk, out_blk, workspace, workspace_bytes, stream, nullptr, 0);
}

// ---- library-owned scratch for callers that cannot allocate ---------------------------------------------------
// One array per GPU (every device that loads this code object holds its own copy at its own address, until the
// process ends).  In host code the array's name is only a handle for the symbol lookup: the address a kernel can use
// is what hipGetSymbolAddress returns with that device current, looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[PS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mu;

int scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_status(e);
    if (dev < 0 || dev >= kMaxDevices) return PS_EUNSUPPORTED;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lk(g_scratch_mu);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) return hip_status(e != hipSuccess ? e : hipErrorInvalidSymbol);
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return PS_OK;
}
}  // namespace

extern "C" int ps_conv2d_fwd_static(const ps_conv_desc *d, const ps_tile *t, const void *in_blk, const void *wt_blk,
                                    void *out_blk, void *stream)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!in_blk || !wt_blk || !out_blk) return PS_EINVAL;
    if (t) {  // an explicit tile whose partial planes exceed the array is refused before anything is looked up
        rc = tile_valid(dm, *t);
        if (rc != PS_OK) return rc;
        if (t->c_split > 1 && (size_t)t->c_split * (size_t)dm.M * dm.K * 4 > (size_t)PS_STATIC_SCRATCH_BYTES) return PS_ESCRATCH;
    }
    void *ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc != PS_OK) return rc;
    return conv_entry(d, t, 1, in_blk, wt_blk, out_blk, ws, (size_t)PS_STATIC_SCRATCH_BYTES, stream, nullptr, 0);
}

extern "C" int ps_conv2d_fwd_fused(const ps_conv_desc *d, const ps_tile *t, const ps_epilogue *e, const void *in_blk,
                                   const void *wt_blk, void *out_blk, void *workspace, size_t workspace_bytes,
                                   void *stream)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!e) return PS_EINVAL;
    if (e->out_dtype != PS_F32 && e->out_dtype != PS_BF16) return PS_EUNSUPPORTED;
    if (!aligned16(e->bias)) return PS_EINVAL;
    // a split reduction can only apply the epilogue where the sum is complete: in the plane-adding pass, so a split
    // tile needs its workspace here (conv_entry refuses it without)
    const int epi = (e->bias ? 1 : 0) | (e->relu ? 2 : 0) | (e->out_dtype == PS_BF16 ? 4 : 0);
    return conv_entry(d, t, 1, in_blk, wt_blk, out_blk, workspace, workspace_bytes, stream, (const float *)e->bias, epi);
}

extern "C" int ps_tile_pick(const ps_conv_desc *d, int with_workspace, size_t workspace_bytes, ps_tile *t)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!t) return PS_EINVAL;
    return cached_pick(d, dm, with_workspace ? 1 : 0, with_workspace ? workspace_bytes : 0, t);
}

extern "C" int ps_tile_autotune(const ps_conv_desc *d, int k, const void *in_blk, const void *wt_blk, void *out_blk,
                                void *workspace, size_t workspace_bytes, void *stream, ps_tile *best, double *best_us)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (k <= 0 || !in_blk || !wt_blk || !out_blk) return PS_EINVAL;
    if (!aligned16(in_blk) || !aligned16(wt_blk) || !aligned16(out_blk) || !aligned16(workspace)) return PS_EINVAL;
    k = std::min(k, 16);
    ps_tile tiles[16];
    const size_t ws_bytes = workspace ? workspace_bytes : 0;
    const int n = ps_tile_rank_ws(d, ws_bytes, k, tiles, nullptr);
    if (n < 0) return n;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if ((rc = hip_status(hipEventCreate(&e0))) != PS_OK) return rc;
    if ((rc = hip_status(hipEventCreate(&e1))) != PS_OK) {
        (void)hipEventDestroy(e0);
        return rc;
    }
    int win = -1;
    double win_us = 1e300;
    for (int i = 0; i < n && rc == PS_OK; ++i) {
        Plan storage;
        const Plan *pl = nullptr;
        if ((rc = cached_plan(d, dm, tiles[i], &storage, &pl)) != PS_OK) break;
        float *ws = pl->ws_need ? (float *)workspace : nullptr;
        // a few launches to settle, then two timed batches (the second as long as about two milliseconds); the faster counts
        for (int w = 0; w < 3 && rc == PS_OK; ++w) rc = run_plan(*pl, in_blk, wt_blk, (float *)out_blk, ws, st);
        int reps = 8;
        double us = 1e300;
        for (int batch = 0; batch < 2 && rc == PS_OK; ++batch) {
            if ((rc = hip_status(hipEventRecord(e0, st))) != PS_OK) break;
            for (int r = 0; r < reps && rc == PS_OK; ++r) rc = run_plan(*pl, in_blk, wt_blk, (float *)out_blk, ws, st);
            if (rc != PS_OK || (rc = hip_status(hipEventRecord(e1, st))) != PS_OK) break;
            if ((rc = hip_status(hipEventSynchronize(e1))) != PS_OK) break;
            float ms = 0.f;
            if ((rc = hip_status(hipEventElapsedTime(&ms, e0, e1))) != PS_OK) break;
            us = std::min(us, (double)ms * 1e3 / reps);
            reps = std::max(8, std::min(400, (int)(2000.0 / std::max(us, 1.0))));
        }
        if (rc == PS_OK && us < win_us) {
            win_us = us;
            win = i;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != PS_OK) return rc;
    if (win < 0) return PS_EUNSUPPORTED;
    const Pick p{tiles[win], win_us};
    pick_cache().replace(pick_key(d, dm, 1, ws_bytes), p);
    if (p.t.c_split == 1) pick_cache().replace(pick_key(d, dm, 0, 0), p);  // the call without a workspace can run it too
    if (best) *best = p.t;
    if (best_us) *best_us = win_us;
    return n;
}

extern "C" size_t ps_tile_cache_entries(void) { return pick_cache().size() + plan_cache().size(); }

extern "C" int ps_tile_kernel(const ps_conv_desc *d, const ps_tile *t)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!t) return PS_EINVAL;
    rc = tile_valid(dm, *t);
    if (rc != PS_OK) return rc;
    return kernel_variant(dm, *t, *find_shape(dm.dtype, t->kt, t->mt, t->ring));
}

extern "C" const char *ps_last_hip_error(void) { return last_hip_error_text(); }

extern "C" int ps_tile_valid(const ps_conv_desc *d, const ps_tile *t)
{
    Dims dm;
    int rc = make_dims(d, &dm);
    if (rc != PS_OK) return rc;
    if (!t) return PS_EINVAL;
    return tile_valid(dm, *t);
}

extern "C" const char *ps_strerror(int status)
{
    switch (status) {
    case PS_OK: return "ok";
    case PS_EINVAL: return "invalid argument (null or misaligned pointer, non-positive size, empty output)";
    case PS_EUNSUPPORTED: return "unsupported (K not a multiple of 16, unknown dtype, tensor over 2 GiB, or tile not valid)";
    case PS_EHIP: return "HIP runtime error at kernel launch";
    case PS_ESCRATCH: return "the tile's partial planes exceed the library's static scratch (PS_STATIC_SCRATCH_BYTES)";
    default: return "unknown status";
    }
}
