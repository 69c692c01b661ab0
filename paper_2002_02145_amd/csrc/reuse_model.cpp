// Host-side data-reuse analysis of Section 4 of the paper for rectangular single-statement loop nests:
// Algorithm 1 by enumeration of the iteration space with per-array bitmaps, Algorithm 2 and Eq. 1 as stated.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "polysci_conv.h"
#include "polysci_reuse.h"

namespace {

struct Space {
    int n_loops;
    int64_t extent[PS_REUSE_MAX_LOOPS];
    int64_t total;
};

// One reference with its array's bounding box folded into a linear element index: idx(it) = base + sum_l step[l]*it_l
struct LinRef {
    int array;
    int64_t base;
    int64_t step[PS_REUSE_MAX_LOOPS];
};

struct ArrayBox {
    bool used = false;
    int n_dims = 0;
    int elem_bytes = 1;
    int64_t lo[PS_REUSE_MAX_DIMS], hi[PS_REUSE_MAX_DIMS];
    int64_t size = 0;
};

// Walks iterations first .. last (linear positions in schedule order) and calls f(iterators).
template <class F>
void walk(const Space &sp, int64_t first, int64_t last, F f)
{
    int64_t it[PS_REUSE_MAX_LOOPS];
    int64_t rem = first;
    for (int l = sp.n_loops - 1; l >= 0; --l) {
        it[l] = rem % sp.extent[l];
        rem /= sp.extent[l];
    }
    for (int64_t pos = first; pos <= last; ++pos) {
        f(it, pos);
        for (int l = sp.n_loops - 1; l >= 0; --l) {  // odometer
            if (++it[l] < sp.extent[l]) break;
            it[l] = 0;
        }
    }
}

inline int64_t elem_of(const LinRef &r, const int64_t *it, int n_loops)
{
    int64_t e = r.base;
    for (int l = 0; l < n_loops; ++l) e += r.step[l] * it[l];
    return e;
}

}  // namespace

extern "C" int ps_reuse_working_sets(const ps_loop_nest *nest, const ps_array_ref *refs, int n_refs, ps_reuse_dep *out,
                                     int cap)
{
    if (!nest || !refs || n_refs < 1 || n_refs > 64 || cap < 0 || (cap > 0 && !out)) return PS_EINVAL;
    if (nest->n_loops < 1 || nest->n_loops > PS_REUSE_MAX_LOOPS) return PS_EINVAL;
    Space sp;
    sp.n_loops = nest->n_loops;
    sp.total = 1;
    for (int l = 0; l < sp.n_loops; ++l) {
        if (nest->extent[l] < 1) return PS_EINVAL;
        sp.extent[l] = nest->extent[l];
        sp.total *= sp.extent[l];
        if (sp.total > (int64_t(1) << 24)) return PS_EUNSUPPORTED;
    }

    // bounding box of every array over the whole iteration space
    ArrayBox box[32];
    for (int r = 0; r < n_refs; ++r) {
        const ps_array_ref &a = refs[r];
        if (a.array < 0 || a.array >= 32 || a.n_dims < 1 || a.n_dims > PS_REUSE_MAX_DIMS || a.elem_bytes < 1)
            return PS_EINVAL;
        ArrayBox &b = box[a.array];
        if (b.used && (b.n_dims != a.n_dims || b.elem_bytes != a.elem_bytes)) return PS_EINVAL;
        for (int d = 0; d < a.n_dims; ++d) {
            int64_t lo = a.offset[d], hi = a.offset[d];
            for (int l = 0; l < sp.n_loops; ++l) {
                const int64_t span = (int64_t)a.coef[d][l] * (sp.extent[l] - 1);
                (span < 0 ? lo : hi) += span;
            }
            if (!b.used) { b.lo[d] = lo; b.hi[d] = hi; }
            else { b.lo[d] = std::min(b.lo[d], lo); b.hi[d] = std::max(b.hi[d], hi); }
        }
        b.n_dims = a.n_dims;
        b.elem_bytes = a.elem_bytes;
        b.used = true;
    }
    for (ArrayBox &b : box) {
        if (!b.used) continue;
        b.size = 1;
        for (int d = 0; d < b.n_dims; ++d) {
            b.size *= b.hi[d] - b.lo[d] + 1;
            if (b.size > (int64_t(1) << 28)) return PS_EUNSUPPORTED;
        }
    }
    std::vector<LinRef> lin(n_refs);
    for (int r = 0; r < n_refs; ++r) {
        const ps_array_ref &a = refs[r];
        const ArrayBox &b = box[a.array];
        LinRef &q = lin[r];
        q.array = a.array;
        q.base = 0;
        for (int l = 0; l < PS_REUSE_MAX_LOOPS; ++l) q.step[l] = 0;
        int64_t pitch = 1;
        for (int d = a.n_dims - 1; d >= 0; --d) {
            q.base += (a.offset[d] - b.lo[d]) * pitch;
            for (int l = 0; l < sp.n_loops; ++l) q.step[l] += (int64_t)a.coef[d][l] * pitch;
            pitch *= b.hi[d] - b.lo[d] + 1;
        }
    }

    // distinct data touched by all references over iterations first .. last
    std::vector<std::vector<uint8_t>> mark(32);
    auto touched = [&](int64_t first, int64_t last) {
        for (int a = 0; a < 32; ++a)
            if (box[a].used) mark[a].assign((size_t)box[a].size, 0);
        int64_t bytes = 0;
        walk(sp, first, last, [&](const int64_t *it, int64_t) {
            for (int r = 0; r < n_refs; ++r) {
                uint8_t &m = mark[lin[r].array][(size_t)elem_of(lin[r], it, sp.n_loops)];
                if (!m) { m = 1; bytes += box[lin[r].array].elem_bytes; }
            }
        });
        return bytes;
    };

    int found = 0;
    std::vector<int64_t> last_touch;  // per element of the target reference's array: last iteration that touches it
    for (int ra = 0; ra < n_refs; ++ra)
        for (int rb = 0; rb < n_refs; ++rb) {
            if (lin[ra].array != lin[rb].array) continue;
            const ArrayBox &b = box[lin[ra].array];
            last_touch.assign((size_t)b.size, -1);
            walk(sp, 0, sp.total - 1, [&](const int64_t *it, int64_t pos) {
                last_touch[(size_t)elem_of(lin[rb], it, sp.n_loops)] = pos;
            });
            // first source: the earliest iteration whose element the target reference touches again later
            int64_t src = -1, src_elem = -1, t_max = -1;
            walk(sp, 0, sp.total - 1, [&](const int64_t *it, int64_t pos) {
                if (src >= 0) return;
                const int64_t e = elem_of(lin[ra], it, sp.n_loops);
                if (last_touch[(size_t)e] > pos) { src = pos; src_elem = e; t_max = last_touch[(size_t)e]; }
            });
            if (src < 0) continue;
            int64_t t_min = -1;
            walk(sp, src + 1, t_max, [&](const int64_t *it, int64_t pos) {
                if (t_min < 0 && elem_of(lin[rb], it, sp.n_loops) == src_elem) t_min = pos;
            });
            if (found < cap) {
                out[found].src_ref = ra;
                out[found].tgt_ref = rb;
                out[found].ws_min = touched(src, t_min);
                out[found].ws_max = t_max == t_min ? out[found].ws_min : touched(src, t_max);
            }
            ++found;
        }
    return found;
}

extern "C" int ps_reuse_assign(const int64_t *ws, int n_ws, const int64_t *cache_sizes, int n_levels, int64_t *level_ws,
                               int64_t *mem_ws)
{
    if (n_ws < 0 || (n_ws > 0 && !ws) || n_levels < 0 || (n_levels > 0 && (!cache_sizes || !level_ws)) || !mem_ws)
        return PS_EINVAL;
    for (int i = 0; i < n_levels; ++i)
        if (cache_sizes[i] < 0) return PS_EINVAL;
    std::vector<int64_t> s(ws, ws + n_ws);
    for (int64_t w : s)
        if (w < 0) return PS_EINVAL;
    std::sort(s.begin(), s.end());
    s.erase(std::unique(s.begin(), s.end()), s.end());
    for (int i = 0; i < n_levels; ++i) level_ws[i] = 0;
    *mem_ws = 0;
    for (int64_t w : s) {
        int i = 0;
        while (i < n_levels && w > cache_sizes[i] - level_ws[i]) ++i;  // (level_ws[i] <= cache_sizes[i]: no overflow)
        if (i < n_levels) level_ws[i] += w;
        else *mem_ws = w > INT64_MAX - *mem_ws ? INT64_MAX : *mem_ws + w;
    }
    return PS_OK;
}

extern "C" double ps_reuse_cost(const int64_t *level_ws, int n_levels, int64_t mem_ws, const double *lat, const double *bw)
{
    if (n_levels < 0 || (n_levels > 0 && !level_ws) || !lat || !bw) return -1.0;
    double c = 0.0;
    for (int i = 0; i <= n_levels; ++i) {
        if (!(bw[i] > 0.0)) return -1.0;
        c += (double)(i < n_levels ? level_ws[i] : mem_ws) * lat[i] / bw[i];
    }
    return c;
}
