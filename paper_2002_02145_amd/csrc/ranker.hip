// Pairwise neural ranking of candidate tiles (Section 4.2.2 of the paper): the statistics of a tile (host, through
// the working-set analysis of Section 4) and the tournament (GPU).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <numeric>
#include <vector>

#include "polysci_ranker.h"
#include "polysci_reuse.h"
#include "ps_internal.h"

namespace ps {
namespace {

constexpr int kIn = 2 * PS_RANKER_STATS;
constexpr int kW1 = 64, kW2 = 32, kW3 = 16, kW4 = 8, kOut = 2;
static_assert(kIn * kW1 + kW1 + kW1 * kW2 + kW2 + kW2 * kW3 + kW3 + kW3 * kW4 + kW4 + kW4 * kOut + kOut == PS_RANKER_PARAMS,
              "parameter layout");

// y[u] = b[u] + sum_k x[k] * W[k][u].  The parameters sit in LDS and every lane reads the same address (a
// broadcast), four values per read; activations stay in registers.  The weights are walked in chunks of 32 values;
// the reads of the next chunk are issued before the multiply-adds of the current one, and scheduling fences keep
// that order (without them the compiler hoists every read of a layer and runs out of registers).
template <int IN, int OUT>
__device__ __forceinline__ const float *dense(const float *p, const float (&x)[IN], float (&y)[OUT])
{
    constexpr int TOT = IN * OUT, CH = 32, NCH = (TOT + CH - 1) / CH;
    static_assert(TOT % 4 == 0, "rows are read four values at a time");
    const float4 *W = reinterpret_cast<const float4 *>(p);
    const float *b = p + TOT;
    float4 buf[2][CH / 4];
#pragma unroll
    for (int q = 0; q < CH / 4; ++q)
        if (q * 4 < TOT) buf[0][q] = W[q];
#pragma unroll
    for (int u = 0; u < OUT; ++u) y[u] = b[u];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        if (c + 1 < NCH) {
#pragma unroll
            for (int q = 0; q < CH / 4; ++q)
                if ((c + 1) * CH + q * 4 < TOT) buf[(c + 1) & 1][q] = W[(c + 1) * (CH / 4) + q];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            const int idx = c * CH + e;
            if (idx < TOT) {
                const float4 w4 = buf[c & 1][e / 4];
                const float w = e % 4 == 0 ? w4.x : e % 4 == 1 ? w4.y : e % 4 == 2 ? w4.z : w4.w;
                y[idx % OUT] = fmaf(x[idx / OUT], w, y[idx % OUT]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    return b + OUT;
}

// The two softmax outputs of the game "a first, b second".
__device__ __forceinline__ float2 play(const float *params, const float4 a, const float4 b)
{
    float x[kIn] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    float total = 0.f;
#pragma unroll
    for (int k = 0; k < kIn; ++k) total += x[k];
#pragma unroll
    for (int k = 0; k < kIn; ++k) x[k] = total != 0.f ? x[k] / total : 0.f;

    float h1[kW1], h2[kW2], h3[kW3], h4[kW4], z[kOut];
    const float *p = dense<kIn, kW1>(params, x, h1);
#pragma unroll
    for (int u = 0; u < kW1; ++u) h1[u] = fmaxf(h1[u], 0.f);
    p = dense<kW1, kW2>(p, h1, h2);
#pragma unroll
    for (int u = 0; u < kW2; ++u) h2[u] = fmaxf(h2[u], 0.f);
    p = dense<kW2, kW3>(p, h2, h3);
#pragma unroll
    for (int u = 0; u < kW3; ++u) h3[u] = h3[u] / (1.f + fabsf(h3[u]));  // softsign
    p = dense<kW3, kW4>(p, h3, h4);
#pragma unroll
    for (int u = 0; u < kW4; ++u) h4[u] = fmaxf(h4[u], 0.f);
    dense<kW4, kOut>(p, h4, z);
    const float m = fmaxf(z[0], z[1]);
    const float e0 = expf(z[0] - m), e1 = expf(z[1] - m);
    const float s = e0 + e1;
    return make_float2(e0 / s, e1 / s);
}

__global__ __launch_bounds__(256) void ranker_clear_kernel(int32_t *__restrict__ wins, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) wins[i] = 0;
}

// One lane per game: workgroup (x, y) plays variant i = y, presented first, against the 256 variants
// j = 256 x .. 256 x + 255, one per lane.  A first output that fires is a win for i: counted over the wave and added
// once; a second output that fires is a win for the lane's own j.  Integer additions commute, so the counts do not
// depend on the order in which workgroups finish.  wins must be zero on entry (ranker_clear_kernel).
__global__ __launch_bounds__(256) void ranker_tournament_kernel(const float4 *__restrict__ stats, int n,
                                                                const float *__restrict__ params, float theta,
                                                                int32_t *__restrict__ wins, float2 *__restrict__ probs)
{
    __shared__ __attribute__((aligned(16))) float net[PS_RANKER_PARAMS + 2];
    for (int k = threadIdx.x; k < PS_RANKER_PARAMS; k += 256) net[k] = params[k];
    __syncthreads();
    const int i = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j - (int)(threadIdx.x & 63) >= n) return;  // the whole wave lies beyond the last variant
    const bool live = j < n && j != i;
    const float4 mine = stats[i];
    const float4 other = live ? stats[j] : mine;
    const float2 out = play(net, mine, other);
    if (probs && j < n) probs[(size_t)i * n + j] = live ? out : make_float2(0.f, 0.f);
    // theta >= 0.5: at most one of the two outputs fires
    int first = live && out.x > theta ? 1 : 0;
    if (live && out.y > theta) atomicAdd(&wins[j], 1);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) first += __shfl_down(first, off, 64);
    if ((threadIdx.x & 63) == 0 && first > 0) atomicAdd(&wins[i], first);
}

}  // namespace
}  // namespace ps

extern "C" int ps_ranker_play(const float *stats, int n, const float *params, float theta, int32_t *wins, float *probs,
                              void *stream)
{
    if (n < 0 || !(theta >= 0.5f && theta < 1.f)) return PS_EINVAL;
    if (n == 0) return PS_OK;
    if (!stats || !params || !wins) return PS_EINVAL;
    if (n > PS_RANKER_MAX_VARIANTS) return PS_EUNSUPPORTED;
    if (!ps::aligned16(stats) || (probs && (reinterpret_cast<uintptr_t>(probs) & 7u))) return PS_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned chunks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(ps::ranker_clear_kernel, dim3(chunks), dim3(256), 0, st, wins, n);
    hipLaunchKernelGGL(ps::ranker_tournament_kernel, dim3(chunks, (unsigned)n), dim3(256), 0, st,
                       reinterpret_cast<const float4 *>(stats), n, params, theta, wins, reinterpret_cast<float2 *>(probs));
    return ps::hip_status(hipGetLastError());
}

extern "C" int ps_tile_reuse_levels(const ps_conv_desc *desc, const ps_tile *tile, int64_t level_ws[PS_RANKER_LEVELS],
                                    int64_t *mem_ws)
{
    if (!tile || !level_ws || !mem_ws) return PS_EINVAL;
    ps::Dims dm;
    if (int rc = ps::make_dims(desc, &dm)) return rc;
    if (tile->kt < 1 || tile->mt < 1 || tile->c_split < 1 || (tile->raster != 0 && tile->raster != 1)) return PS_EINVAL;
    if (dm.Cb % tile->c_split) return PS_EUNSUPPORTED;

    const long long n_mt = (dm.M + tile->mt - 1) / tile->mt;
    const int n_kt = (dm.K + tile->kt - 1) / tile->kt;
    const int cbs = dm.Cb / tile->c_split, taps = dm.R * dm.S;
    if (n_mt > (1ll << 24)) return PS_EUNSUPPORTED;

    // loops, outermost first: the two tile loops in launch order, the split, the channel blocks of a split, the taps
    const int lm = tile->raster == 0 ? 0 : 1, lk = 1 - lm, ls = 2, lc = 3, lt = 4;
    ps_loop_nest nest = {};
    nest.n_loops = 5;
    nest.extent[lm] = (int32_t)n_mt;
    nest.extent[lk] = n_kt;
    nest.extent[ls] = tile->c_split;
    nest.extent[lc] = cbs;
    nest.extent[lt] = taps;

    const long long m_eff = dm.M < tile->mt ? dm.M : tile->mt;
    const int k_eff = dm.K < tile->kt ? dm.K : tile->kt;
    const int out_bytes = (int)(m_eff * k_eff * 4);
    const int in_bytes = (int)(m_eff * 16 * dm.es);  // one channel block of the tile's pixels (the taps re-read it)
    const int wt_bytes = k_eff * 16 * dm.es;         // one tap of one channel block of the tile's filters

    ps_array_ref refs[4] = {};
    for (int w = 0; w < 2; ++w) {  // the partial output tile, read (accumulate) and written
        ps_array_ref &o = refs[w];
        o.array = 0, o.n_dims = 3, o.is_write = w, o.elem_bytes = out_bytes;
        o.coef[0][lm] = 1, o.coef[1][lk] = 1, o.coef[2][ls] = 1;
    }
    ps_array_ref &in = refs[2];
    in.array = 1, in.n_dims = 2, in.is_write = 0, in.elem_bytes = in_bytes;
    in.coef[0][lm] = 1, in.coef[1][ls] = cbs, in.coef[1][lc] = 1;
    ps_array_ref &wt = refs[3];
    wt.array = 2, wt.n_dims = 3, wt.is_write = 0, wt.elem_bytes = wt_bytes;
    wt.coef[0][lk] = 1, wt.coef[1][ls] = cbs, wt.coef[1][lc] = 1, wt.coef[2][lt] = 1;

    ps_reuse_dep deps[16];  // at most one dependence per ordered pair of the four references
    const int found = ps_reuse_working_sets(&nest, refs, 4, deps, 16);
    if (found < 0) return found;
    if (found > 16) return PS_EINVAL;
    std::vector<int64_t> ws;
    for (int d = 0; d < found; ++d) {
        ws.push_back(deps[d].ws_min);
        ws.push_back(deps[d].ws_max);
    }
    static const int64_t level_bytes[PS_RANKER_LEVELS] = {(160 + 512) * 1024, 8 * 4 * 1024 * 1024, 256 * 1024 * 1024};
    return ps_reuse_assign(ws.data(), (int)ws.size(), level_bytes, PS_RANKER_LEVELS, level_ws, mem_ws);
}

extern "C" size_t ps_tile_rank_dnn_scratch_bytes(const ps_conv_desc *desc)
{
    const int n = ps_tile_count(desc);
    return n > 0 ? (size_t)n * (PS_RANKER_STATS * sizeof(float) + sizeof(int32_t)) : 0;
}

extern "C" int ps_tile_rank_dnn(const ps_conv_desc *desc, size_t workspace_bytes, int stats_kind, const float *params,
                                float theta, void *scratch, size_t scratch_bytes, int k, ps_tile *tiles, int32_t *wins,
                                void *stream)
{
    ps::Dims dm;
    if (int rc = ps::make_dims(desc, &dm)) return rc;
    if (k <= 0 || !tiles || !params || !scratch) return PS_EINVAL;
    if (stats_kind != PS_RANKER_WORKING_SETS && stats_kind != PS_RANKER_LEVEL_TIMES) return PS_EINVAL;
    if (!(theta >= 0.5f && theta < 1.f) || !ps::aligned16(scratch)) return PS_EINVAL;
    const int total = ps_tile_count(desc);
    if (total < 0) return total;

    // the candidates that can run in the caller's workspace and have statistics of the requested kind
    std::vector<ps_tile> cand;
    std::vector<float> stats;
    for (int i = 0; i < total; ++i) {
        ps_tile t;
        if (int rc = ps_tile_get(desc, i, &t)) return rc;
        if (t.c_split > 1 && (size_t)t.c_split * (size_t)dm.M * dm.K * 4 > workspace_bytes) continue;
        float f[PS_RANKER_STATS];
        if (stats_kind == PS_RANKER_WORKING_SETS) {
            int64_t level[PS_RANKER_LEVELS], mem;
            const int rc = ps_tile_reuse_levels(desc, &t, level, &mem);
            if (rc == PS_EUNSUPPORTED) continue;
            if (rc != PS_OK) return rc;
            for (int l = 0; l < PS_RANKER_LEVELS; ++l) f[l] = (float)level[l];
            f[PS_RANKER_LEVELS] = (float)mem;
        } else {
            double us[PS_RANKER_STATS];
            if (int rc = ps_tile_level_times_ws(desc, &t, us)) return rc;
            for (int l = 0; l < PS_RANKER_STATS; ++l) f[l] = (float)us[l];
        }
        cand.push_back(t);
        stats.insert(stats.end(), f, f + PS_RANKER_STATS);
    }
    const int n = (int)cand.size();
    if (n == 0) return PS_EUNSUPPORTED;
    const size_t stats_bytes = (size_t)n * PS_RANKER_STATS * sizeof(float);
    if (scratch_bytes < stats_bytes + (size_t)n * sizeof(int32_t)) return PS_EINVAL;

    hipStream_t st = static_cast<hipStream_t>(stream);
    float *d_stats = static_cast<float *>(scratch);
    int32_t *d_wins = reinterpret_cast<int32_t *>(static_cast<char *>(scratch) + stats_bytes);
    // The copies use this function's own host buffers, so every path out of here waits for the stream first.
    std::vector<int32_t> won((size_t)n);
    int rc = ps::hip_status(hipMemcpyAsync(d_stats, stats.data(), stats_bytes, hipMemcpyHostToDevice, st));
    if (rc == PS_OK) rc = ps_ranker_play(d_stats, n, params, theta, d_wins, nullptr, stream);
    if (rc == PS_OK)
        rc = ps::hip_status(hipMemcpyAsync(won.data(), d_wins, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    const int rc_sync = ps::hip_status(hipStreamSynchronize(st));
    if (rc != PS_OK) return rc;
    if (rc_sync != PS_OK) return rc_sync;

    std::vector<int> order((size_t)n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return won[a] > won[b]; });  // ties: listing order
    const int m = std::min(k, n);
    for (int j = 0; j < m; ++j) {
        tiles[j] = cand[order[j]];
        if (wins) wins[j] = won[order[j]];
    }
    return m;
}
