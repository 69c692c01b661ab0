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
// broadcast), four values per read; activations stay in registers.
template <int IN, int OUT>
__device__ __forceinline__ const float *dense(const float *__restrict__ p, const float (&x)[IN], float (&y)[OUT])
{
    const float *__restrict__ W = p;
    const float *__restrict__ b = p + IN * OUT;
#pragma unroll
    for (int u = 0; u < OUT; ++u) y[u] = b[u];
#pragma unroll
    for (int k = 0; k < IN; ++k) {
#pragma unroll
        for (int u = 0; u < OUT; ++u) y[u] = fmaf(x[k], W[k * OUT + u], y[u]);
        if (k % 2 == 1) __builtin_amdgcn_sched_barrier(0);  // keeps the reads of later rows from piling up in registers
    }
    return b + OUT;
}

// The two softmax outputs of the game "a first, b second".
__device__ __forceinline__ float2 play(const float *__restrict__ params, const float4 a, const float4 b)
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

// Workgroup i tallies variant i: its lanes take the opponents j in turn and play both seatings, (i, j) and (j, i).
// Every game is therefore evaluated by both of its players' workgroups, which keeps the tally free of atomics and
// its result independent of scheduling.
__global__ __launch_bounds__(256) void ranker_tournament_kernel(const float4 *__restrict__ stats, int n,
                                                                const float *__restrict__ params, float theta,
                                                                int32_t *__restrict__ wins, float2 *__restrict__ probs)
{
    __shared__ __attribute__((aligned(16))) float net[PS_RANKER_PARAMS + 2];
    __shared__ int partial[4];
    for (int k = threadIdx.x; k < PS_RANKER_PARAMS; k += 256) net[k] = params[k];
    __syncthreads();
    const int i = blockIdx.x;
    const float4 mine = stats[i];
    int won = 0;
    for (int j = threadIdx.x; j < n; j += 256) {
        if (j == i) {
            if (probs) probs[(size_t)i * n + j] = make_float2(0.f, 0.f);
            continue;
        }
        const float4 other = stats[j];
#pragma unroll 1
        for (int seat = 0; seat < 2; ++seat) {  // one copy of the network's code serves both seatings
            const float2 out = play(net, seat == 0 ? mine : other, seat == 0 ? other : mine);
            if (seat == 0 && probs) probs[(size_t)i * n + j] = out;
            won += (seat == 0 ? out.x : out.y) > theta ? 1 : 0;  // theta >= 0.5: at most one output fires
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) won += __shfl_down(won, off, 64);
    if ((threadIdx.x & 63) == 0) partial[threadIdx.x >> 6] = won;
    __syncthreads();
    if (threadIdx.x == 0) wins[i] = partial[0] + partial[1] + partial[2] + partial[3];
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
    hipLaunchKernelGGL(ps::ranker_tournament_kernel, dim3((unsigned)n), dim3(256), 0, static_cast<hipStream_t>(stream),
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
    if (int rc = ps::hip_status(hipMemcpyAsync(d_stats, stats.data(), stats_bytes, hipMemcpyHostToDevice, st))) return rc;
    if (int rc = ps_ranker_play(d_stats, n, params, theta, d_wins, nullptr, stream)) return rc;
    std::vector<int32_t> won((size_t)n);
    if (int rc = ps::hip_status(hipMemcpyAsync(won.data(), d_wins, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost, st)))
        return rc;
    if (int rc = ps::hip_status(hipStreamSynchronize(st))) return rc;

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
