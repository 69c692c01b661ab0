// Drives the host-side code of the library (descriptor validation, tile enumeration and ranking, the per-process
// tile table, the working-set analysis of Section 4) and the C oracle under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Built and run by tests/test_host_sanitizers.py on the CPU; no GPU call is made.
// Exit status 0 and no sanitizer report = pass.  Every check that fails prints a line and counts as an error.
#include <climits>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "polysci_conv.h"
#include "polysci_ranker.h"
#include "polysci_reuse.h"

extern "C" {
typedef struct {
    int32_t N, C, H, W, K, R, S, stride, pad;
} oracle_shape;
int oracle_out_dims(const oracle_shape *sh, int32_t *P, int32_t *Q);
int oracle_conv2d_fwd(const oracle_shape *sh, const float *in, const float *wt, double *out, double *mag);
int oracle_conv2d_fwd_point(const oracle_shape *sh, const float *in, const float *wt, int32_t n, int32_t k, int32_t p,
                            int32_t q, double *out, double *mag);
}

// The host objects are built without device code, and this program must run where there is no GPU: the few HIP
// runtime entry points they refer to are answered here.  Registration of (absent) device code does nothing; every
// call that would need a device reports hipErrorNoDevice, which the library must turn into PS_EHIP.
extern "C" {
static void *g_no_fatbin = nullptr;
void **__hipRegisterFatBinary(const void *) { return &g_no_fatbin; }
void __hipUnregisterFatBinary(void **) {}
void __hipRegisterFunction(void **, const void *, char *, const char *, unsigned, void *, void *, void *, void *, int *) {}
void __hipRegisterVar(void **, void *, char *, const char *, int, size_t, int, int) {}
int __hipPushCallConfiguration(...) { return 100; }
int __hipPopCallConfiguration(...) { return 100; }
int hipLaunchKernel(...) { return 100; }
int hipGetLastError(void) { return 100; }
const char *hipGetErrorString(int) { return "no device (host sanitizer build)"; }
int hipGetDevice(int *) { return 100; }
int hipDeviceGetAttribute(...) { return 100; }
int hipGetSymbolAddress(...) { return 100; }
int hipMemcpyAsync(...) { return 100; }
int hipStreamSynchronize(...) { return 100; }
int hipEventCreate(...) { return 100; }
int hipEventDestroy(...) { return 100; }
int hipEventRecord(...) { return 100; }
int hipEventSynchronize(...) { return 100; }
int hipEventElapsedTime(...) { return 100; }
}

static int g_errors = 0;
#define CHECK(cond, ...)                    \
    do {                                    \
        if (!(cond)) {                      \
            ++g_errors;                     \
            std::fprintf(stderr, "CHECK failed (%s:%d): ", __FILE__, __LINE__); \
            std::fprintf(stderr, __VA_ARGS__);                                \
            std::fprintf(stderr, "\n");     \
        }                                   \
    } while (0)

// splitmix64: the driver's own draw of shapes and nests
struct Rng {
    uint64_t s;
    uint64_t next()
    {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    int range(int lo, int hi) { return lo + (int)(next() % (uint64_t)(hi - lo + 1)); }  // inclusive
};

static ps_conv_desc desc(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype)
{
    ps_conv_desc d = {N, C, H, W, K, R, S, stride, pad, dtype};
    return d;
}

// Every host-side call of the tile space on one descriptor; consistency between them is checked on the way.
static void drive_descriptor(const ps_conv_desc &d, bool expect_valid, bool with_working_sets)
{
    int32_t P = -7, Q = -7;
    const int rc = ps_out_dims(&d, &P, &Q);
    if (!expect_valid) {
        CHECK(rc != PS_OK, "malformed descriptor accepted (N=%d C=%d H=%d W=%d K=%d R=%d S=%d st=%d pad=%d dt=%d)", d.N, d.C,
              d.H, d.W, d.K, d.R, d.S, d.stride, d.pad, d.dtype);
        CHECK(ps_blocked_in_bytes(&d) == 0 && ps_blocked_wt_bytes(&d) == 0 && ps_blocked_out_bytes(&d) == 0, "sizes of a malformed descriptor");
        CHECK(ps_tile_count(&d) < 0, "tile count of a malformed descriptor");
        ps_tile t = {64, 64, 2, 1, 0};
        double us = 0;
        CHECK(ps_tile_get(&d, 0, &t) < 0 && ps_tile_valid(&d, &t) < 0 && ps_tile_select(&d, &t, &us) < 0 &&
                  ps_tile_select_ws(&d, 1 << 20, &t, &us) < 0 && ps_tile_pick(&d, 1, 1 << 20, &t) < 0 &&
                  ps_tile_rank_ws(&d, 1 << 20, 3, &t, &us) < 0 && ps_tile_kernel(&d, &t) < 0,
              "tile calls on a malformed descriptor");
        CHECK(ps_tile_cost_us(&d, &t) < 0 && ps_tile_cost_ws_us(&d, &t) < 0 && ps_workspace_bytes(&d, &t) == 0, "costs of a malformed descriptor");
        // the convolution calls refuse before touching a pointer or the device
        CHECK(ps_conv2d_fwd(&d, &t, &t, &t, nullptr) < 0, "ps_conv2d_fwd on a malformed descriptor");
        CHECK(ps_conv2d_fwd_ws(&d, nullptr, &t, &t, &t, nullptr, 0, nullptr) < 0, "ps_conv2d_fwd_ws on a malformed descriptor");
        CHECK(ps_conv2d_fwd_static(&d, nullptr, &t, &t, &t, nullptr) < 0, "ps_conv2d_fwd_static on a malformed descriptor");
        return;
    }
    CHECK(rc == PS_OK && P > 0 && Q > 0, "valid descriptor refused: rc %d", rc);
    if (rc != PS_OK) return;
    oracle_shape os = {d.N, d.C, d.H, d.W, d.K, d.R, d.S, d.stride, d.pad};
    int32_t oP = 0, oQ = 0;
    CHECK(oracle_out_dims(&os, &oP, &oQ) == 0 && oP == P && oQ == Q, "output size disagrees with the oracle's");
    const int n = ps_tile_count(&d);
    CHECK(n > 0, "no candidate tile");
    std::vector<ps_tile> tiles((size_t)(n > 0 ? n : 0));
    double best_ws = 1e300;
    for (int i = 0; i < n; ++i) {
        CHECK(ps_tile_get(&d, i, &tiles[i]) == PS_OK, "ps_tile_get(%d)", i);
        CHECK(ps_tile_valid(&d, &tiles[i]) == PS_OK, "enumerated tile %d not valid", i);
        const double c0 = ps_tile_cost_us(&d, &tiles[i]), c1 = ps_tile_cost_ws_us(&d, &tiles[i]);
        CHECK(c0 > 0 && c1 > 0 && std::isfinite(c0) && std::isfinite(c1), "cost of tile %d: %g %g", i, c0, c1);
        best_ws = c1 < best_ws ? c1 : best_ws;
        CHECK(ps_tile_kernel(&d, &tiles[i]) >= 0, "ps_tile_kernel of tile %d", i);
        double terms[PS_RANKER_STATS];
        CHECK(ps_tile_level_times_ws(&d, &tiles[i], terms) == PS_OK, "level times of tile %d", i);
        const size_t wsb = ps_workspace_bytes(&d, &tiles[i]);
        CHECK((wsb == 0) == (tiles[i].c_split == 1), "workspace bytes of tile %d", i);
    }
    ps_tile out_of_range;
    CHECK(ps_tile_get(&d, n, &out_of_range) < 0 && ps_tile_get(&d, -1, &out_of_range) < 0, "ps_tile_get out of range");
    CHECK(ps_tile_get(&d, 0, nullptr) < 0, "ps_tile_get null");
    ps_tile pick, cached;
    double us = 0;
    CHECK(ps_tile_select_ws(&d, (size_t)1 << 40, &pick, &us) == PS_OK && std::fabs(us - best_ws) <= 1e-9 * best_ws, "select_ws is not the arg min");
    for (int rep = 0; rep < 2; ++rep) {
        CHECK(ps_tile_pick(&d, 1, (size_t)1 << 40, &cached) == PS_OK && std::memcmp(&pick, &cached, sizeof pick) == 0, "cached pick differs (ws)");
    }
    CHECK(ps_tile_select(&d, &pick, &us) == PS_OK, "select");
    CHECK(ps_tile_pick(&d, 0, 0, &cached) == PS_OK && std::memcmp(&pick, &cached, sizeof pick) == 0, "cached pick differs");
    std::vector<ps_tile> ranked((size_t)n + 3);
    std::vector<double> rus((size_t)n + 3);
    const int got = ps_tile_rank_ws(&d, (size_t)1 << 40, n + 3, ranked.data(), rus.data());
    CHECK(got == n, "rank_ws returned %d of %d", got, n);
    for (int i = 1; i < got; ++i) CHECK(rus[i - 1] <= rus[i], "ranking not ascending at %d", i);
    CHECK(ps_tile_rank_ws(&d, 0, 0, ranked.data(), nullptr) < 0, "rank_ws with k = 0");
    // tiles that are not in the table of compiled shapes
    const ps_tile bad[] = {{0, 64, 2, 1, 0}, {64, 0, 2, 1, 0}, {64, 64, 3, 1, 0}, {64, 64, 2, 0, 0}, {64, 64, 2, 1, 2},
                           {INT_MAX, INT_MAX, INT_MAX, INT_MAX, 1}, {64, 64, 2, INT_MAX, 0}, {-64, 64, 2, 1, 0}};
    for (const ps_tile &b : bad) {
        CHECK(ps_tile_valid(&d, &b) < 0 && ps_tile_cost_us(&d, &b) < 0 && ps_workspace_bytes(&d, &b) == 0, "bad tile accepted");
        CHECK(ps_conv2d_fwd_static(&d, &b, &b, &b, const_cast<ps_tile *>(&b), nullptr) < 0, "bad tile launched");
    }
    if (with_working_sets) {  // Algorithms 1 and 2 on the tile's workgroup-level nest (enumeration: small shapes only)
        int64_t lvl[PS_RANKER_LEVELS], mem = -1;
        const int r = ps_tile_reuse_levels(&d, &tiles[0], lvl, &mem);
        CHECK(r == PS_OK || r == PS_EUNSUPPORTED, "ps_tile_reuse_levels: %d", r);
        if (r == PS_OK) CHECK(mem >= 0 && lvl[0] >= 0 && lvl[1] >= 0 && lvl[2] >= 0, "negative working set");
    }
}

static void drive_reuse(Rng &rng)
{
    // well-formed random nests: 1-4 loops, 1-3 arrays with small coefficients
    for (int it = 0; it < 200; ++it) {
        ps_loop_nest nest;
        std::memset(&nest, 0, sizeof nest);
        nest.n_loops = rng.range(1, 4);
        for (int l = 0; l < nest.n_loops; ++l) nest.extent[l] = rng.range(1, 6);
        const int n_refs = rng.range(1, 4);
        std::vector<ps_array_ref> refs((size_t)n_refs);
        for (auto &r : refs) {
            std::memset(&r, 0, sizeof r);
            r.array = rng.range(0, 2);
            r.n_dims = rng.range(1, 3);
            r.is_write = rng.range(0, 1);
            r.elem_bytes = 1;
            for (int dd = 0; dd < r.n_dims; ++dd) {
                for (int l = 0; l < nest.n_loops; ++l) r.coef[dd][l] = rng.range(-1, 2);
                r.offset[dd] = rng.range(-2, 2);
            }
        }
        for (size_t i = 0; i < refs.size(); ++i)   // references to one array agree in rank
            for (size_t j = 0; j < i; ++j)
                if (refs[i].array == refs[j].array) refs[i].n_dims = refs[j].n_dims;
        const int n = ps_reuse_working_sets(&nest, refs.data(), n_refs, nullptr, 0);
        CHECK(n >= 0 || n == PS_EINVAL || n == PS_EUNSUPPORTED, "working sets: %d", n);
        if (n > 0) {
            std::vector<ps_reuse_dep> deps((size_t)n);
            const int m = ps_reuse_working_sets(&nest, refs.data(), n_refs, deps.data(), n);
            CHECK(m == n, "second call found %d of %d", m, n);
            std::vector<int64_t> ws;
            for (const auto &dp : deps) {
                CHECK(dp.ws_min >= 1 && dp.ws_min <= dp.ws_max, "ws_min %lld ws_max %lld", (long long)dp.ws_min, (long long)dp.ws_max);
                ws.push_back(dp.ws_min);
                ws.push_back(dp.ws_max);
            }
            // a short output buffer is filled up to its capacity and no further (the guard word must survive)
            std::vector<ps_reuse_dep> few(2);
            few[1].ws_max = -12345;
            CHECK(ps_reuse_working_sets(&nest, refs.data(), n_refs, few.data(), 1) == n && few[1].ws_max == -12345, "capacity not respected");
            const int64_t caches[3] = {8, 64, 512};
            int64_t lvl[3], mem = -1;
            CHECK(ps_reuse_assign(ws.data(), (int)ws.size(), caches, 3, lvl, &mem) == PS_OK && mem >= 0, "assign");
            const double lat[4] = {1, 4, 20, 100}, bw[4] = {64, 32, 16, 4};
            CHECK(ps_reuse_cost(lvl, 3, mem, lat, bw) >= 0, "cost");
        }
    }
    // malformed arguments: every one must come back as an error code, not as an access
    ps_loop_nest nest;
    std::memset(&nest, 0, sizeof nest);
    ps_array_ref ref;
    std::memset(&ref, 0, sizeof ref);
    ref.n_dims = 1;
    ref.elem_bytes = 1;
    ref.coef[0][0] = 1;
    nest.n_loops = 1;
    nest.extent[0] = 4;
    CHECK(ps_reuse_working_sets(nullptr, &ref, 1, nullptr, 0) < 0, "null nest");
    CHECK(ps_reuse_working_sets(&nest, nullptr, 1, nullptr, 0) < 0, "null refs");
    CHECK(ps_reuse_working_sets(&nest, &ref, 1, nullptr, 5) < 0, "null out with capacity");
    const int bad_loops[] = {0, -1, PS_REUSE_MAX_LOOPS + 1, INT_MAX};
    for (int v : bad_loops) {
        ps_loop_nest b = nest;
        b.n_loops = v;
        CHECK(ps_reuse_working_sets(&b, &ref, 1, nullptr, 0) < 0, "n_loops = %d accepted", v);
    }
    const int bad_extent[] = {0, -3, INT_MAX};
    for (int v : bad_extent) {
        ps_loop_nest b = nest;
        b.extent[0] = v;
        CHECK(ps_reuse_working_sets(&b, &ref, 1, nullptr, 0) < 0, "extent = %d accepted", v);
    }
    const int bad_dims[] = {0, -1, PS_REUSE_MAX_DIMS + 1, INT_MAX};
    for (int v : bad_dims) {
        ps_array_ref b = ref;
        b.n_dims = v;
        CHECK(ps_reuse_working_sets(&nest, &b, 1, nullptr, 0) < 0, "n_dims = %d accepted", v);
    }
    const int bad_array[] = {-1, 32, INT_MAX, INT_MIN};
    for (int v : bad_array) {
        ps_array_ref b = ref;
        b.array = v;
        CHECK(ps_reuse_working_sets(&nest, &b, 1, nullptr, 0) < 0, "array id %d accepted", v);
    }
    {
        ps_array_ref b = ref;
        b.elem_bytes = 0;
        CHECK(ps_reuse_working_sets(&nest, &b, 1, nullptr, 0) < 0, "elem_bytes = 0 accepted");
        b = ref;  // coefficients and offsets at the ends of the integer range: bounding boxes that overflow 32 bits
        b.coef[0][0] = INT_MAX;
        b.offset[0] = INT_MAX;
        CHECK(ps_reuse_working_sets(&nest, &b, 1, nullptr, 0) < 0, "huge coefficient accepted");
        b.coef[0][0] = INT_MIN;
        b.offset[0] = INT_MIN;
        CHECK(ps_reuse_working_sets(&nest, &b, 1, nullptr, 0) < 0, "huge negative coefficient accepted");
        ps_loop_nest big = nest;
        big.n_loops = 8;
        for (int l = 0; l < 8; ++l) big.extent[l] = 64;  // 2^48 iterations
        CHECK(ps_reuse_working_sets(&big, &ref, 1, nullptr, 0) == PS_EUNSUPPORTED, "2^48 iterations accepted");
        CHECK(ps_reuse_working_sets(&nest, &ref, 0, nullptr, 0) <= 0, "no references");
        CHECK(ps_reuse_working_sets(&nest, &ref, -4, nullptr, 0) < 0, "negative reference count");
    }
    int64_t lvl[2], mem;
    const int64_t ws[3] = {4, 4, 9}, caches[2] = {8, 16}, neg_cache[2] = {8, -1}, neg_ws[2] = {4, -2};
    CHECK(ps_reuse_assign(ws, 3, caches, 2, lvl, &mem) == PS_OK && lvl[0] == 4 && lvl[1] == 9 && mem == 0, "assign example");
    CHECK(ps_reuse_assign(nullptr, 3, caches, 2, lvl, &mem) < 0 && ps_reuse_assign(ws, -1, caches, 2, lvl, &mem) < 0 &&
              ps_reuse_assign(ws, 3, nullptr, 2, lvl, &mem) < 0 && ps_reuse_assign(ws, 3, caches, 2, nullptr, &mem) < 0 &&
              ps_reuse_assign(ws, 3, caches, 2, lvl, nullptr) < 0 && ps_reuse_assign(ws, 3, neg_cache, 2, lvl, &mem) < 0 &&
              ps_reuse_assign(neg_ws, 2, caches, 2, lvl, &mem) < 0,
          "malformed assign accepted");
    const double lat[3] = {1, 2, 3}, bw[3] = {1, 1, 1}, zero_bw[3] = {1, 0, 1};
    CHECK(ps_reuse_cost(nullptr, 2, 0, lat, bw) < 0 && ps_reuse_cost(lvl, 2, 0, nullptr, bw) < 0 && ps_reuse_cost(lvl, 2, 0, lat, zero_bw) < 0 &&
              ps_reuse_cost(lvl, -1, 0, lat, bw) < 0,
          "malformed cost accepted");
}

static void drive_oracle(Rng &rng)
{
    // exactly-sized heap buffers: any index error in the oracle's loops is an out-of-bounds access here
    for (int it = 0; it < 60; ++it) {
        oracle_shape s = {rng.range(1, 2), rng.range(1, 5), rng.range(1, 9), rng.range(1, 9), rng.range(1, 4), rng.range(1, 5), rng.range(1, 5),
                          rng.range(1, 3), rng.range(0, 3)};
        int32_t P, Q;
        if (oracle_out_dims(&s, &P, &Q) != 0) continue;
        std::vector<float> in((size_t)s.N * s.C * s.H * s.W), wt((size_t)s.K * s.C * s.R * s.S);
        for (auto &v : in) v = (float)rng.range(-2, 2);
        for (auto &v : wt) v = (float)rng.range(-2, 2);
        std::vector<double> out((size_t)s.N * s.K * P * Q), mag(out.size());
        CHECK(oracle_conv2d_fwd(&s, in.data(), wt.data(), out.data(), mag.data()) == 0, "oracle refused a valid shape");
        const int n = rng.range(0, s.N - 1), k = rng.range(0, s.K - 1), p = rng.range(0, P - 1), q = rng.range(0, Q - 1);
        double o1, m1;
        CHECK(oracle_conv2d_fwd_point(&s, in.data(), wt.data(), n, k, p, q, &o1, &m1) == 0, "point call");
        const size_t o = (((size_t)n * s.K + k) * P + p) * Q + q;
        CHECK(o1 == out[o] && m1 == mag[o], "point and full result differ");
        CHECK(oracle_conv2d_fwd_point(&s, in.data(), wt.data(), s.N, k, p, q, &o1, &m1) != 0, "point outside the output accepted");
    }
    const oracle_shape bad[] = {{0, 1, 1, 1, 1, 1, 1, 1, 0}, {1, 1, 2, 2, 1, 5, 5, 1, 0}, {1, 1, 1, 1, 1, 1, 1, 0, 0}, {1, 1, 1, 1, 1, 1, 1, 1, -1},
                                {1, 1, INT_MAX, INT_MAX, 1, 1, 1, 1, INT_MAX}};
    for (const oracle_shape &s : bad) {
        int32_t P, Q;
        float x = 0;
        double o;
        if (s.pad == INT_MAX) continue;  // the oracle is a checker for sane shapes; its size arithmetic is plain int
        CHECK(oracle_out_dims(&s, &P, &Q) != 0 && oracle_conv2d_fwd(&s, &x, &x, &o, nullptr) != 0, "oracle accepted a malformed shape");
    }
}

int main()
{
    Rng rng{20260211};
    // shapes that exercise the edges of the tiling, both element types
    const int edge[][9] = {{1, 64, 14, 14, 64, 3, 3, 1, 1},  {3, 32, 7, 7, 64, 3, 3, 1, 1},   {2, 3, 23, 19, 32, 7, 7, 2, 3},
                           {2, 48, 9, 11, 32, 1, 1, 2, 0},   {1, 20, 6, 5, 16, 2, 3, 1, 1},   {5, 16, 5, 5, 128, 1, 1, 1, 0},
                           {1, 16, 1, 1, 16, 1, 1, 1, 0},    {2, 16, 4, 4, 32, 3, 3, 3, 2},   {1, 32, 12, 12, 256, 3, 3, 1, 0},
                           {2, 16, 6, 6, 48, 3, 3, 1, 1},    {1, 80, 3, 3, 96, 1, 1, 1, 0},   {2, 4, 9, 10, 16, 7, 7, 1, 3},
                           {3, 64, 9, 7, 256, 1, 1, 1, 0},   {28, 64, 56, 56, 64, 3, 3, 1, 1}, {28, 512, 7, 7, 512, 3, 3, 1, 1},
                           {28, 3, 224, 224, 64, 7, 7, 2, 3}, {28, 512, 28, 28, 1024, 1, 1, 2, 0}, {28, 2048, 7, 7, 512, 1, 1, 1, 0},
                           {28, 48, 27, 27, 128, 5, 5, 1, 2}, {28, 3, 227, 227, 64, 11, 11, 4, 0}};
    int idx = 0;
    for (const auto &e : edge) {
        for (int dt = 0; dt < 2; ++dt)
            drive_descriptor(desc(e[0], e[1], e[2], e[3], e[4], e[5], e[6], e[7], e[8], dt), true, idx < 13 && dt == 0);
        ++idx;
    }
    // seeded random shapes over the accepted parameter space
    for (int it = 0; it < 150; ++it) {
        const int R = rng.range(1, 7), S = rng.range(0, 1) ? R : rng.range(1, 7);
        const int stride = rng.range(1, 3), pad = rng.range(0, 3), H = rng.range(1, 40), W = rng.range(1, 40);
        if (H + 2 * pad < R || W + 2 * pad < S) continue;
        drive_descriptor(desc(rng.range(1, 30), rng.range(1, 300), H, W, 16 * rng.range(1, 40), R, S, stride, pad, rng.range(0, 1)), true, false);
    }
    // malformed descriptors: zero, negative and extreme fields, K off the block size, unknown element types, tensors
    // beyond 32-bit offsets
    const ps_conv_desc ok = desc(2, 16, 8, 8, 16, 3, 3, 1, 1, 0);
    for (int field = 0; field < 10; ++field)
        for (int v : {0, -1, INT_MIN, INT_MAX, INT_MAX - 1, 1 << 30}) {
            ps_conv_desc d = ok;
            reinterpret_cast<int32_t *>(&d)[field] = v;
            int32_t P, Q;
            if ((field == 8 && v == 0) || (field == 9 && v == 0)) continue;  // pad 0, dtype 0 are fine
            // whatever the answer, no call may misbehave; an answer of "valid" must come with positive sizes
            const bool valid = ps_out_dims(&d, &P, &Q) == PS_OK;
            drive_descriptor(d, valid, false);
        }
    drive_descriptor(desc(1, 16, 8, 8, 24, 3, 3, 1, 1, 0), false, false);          // K not a multiple of 16
    drive_descriptor(desc(1, 16, 2, 2, 16, 5, 5, 1, 0, 0), false, false);          // filter larger than the padded image
    drive_descriptor(desc(512, 1024, 224, 224, 16, 1, 1, 1, 0, 0), false, false);  // input beyond 2 GiB
    drive_descriptor(desc(1, 16, 8, 8, 16, 3, 3, 1, 1, 7), false, false);          // unknown element type
    CHECK(ps_out_dims(nullptr, nullptr, nullptr) < 0 && ps_tile_count(nullptr) < 0 && ps_blocked_in_bytes(nullptr) == 0, "null descriptor");

    // the per-process tile table under concurrent first use
    std::vector<std::thread> threads;
    for (int th = 0; th < 8; ++th)
        threads.emplace_back([th, &edge] {
            for (int rep = 0; rep < 3; ++rep)
                for (int i = 0; i < 20; ++i) {
                    const auto &e = edge[(i + th) % 20];
                    const ps_conv_desc d = desc(e[0] + 1, e[1], e[2], e[3], e[4], e[5], e[6], e[7], e[8], th & 1);  // N + 1: not seen above
                    ps_tile a, b;
                    double us;
                    if (ps_tile_pick(&d, 1, (size_t)64 << 20, &a) != PS_OK || ps_tile_select_ws(&d, (size_t)64 << 20, &b, &us) != PS_OK ||
                        std::memcmp(&a, &b, sizeof a) != 0)
                        std::fprintf(stderr, "thread %d: cached pick differs\n", th), std::abort();
                }
        });
    for (auto &t : threads) t.join();
    CHECK(ps_tile_cache_entries() > 0, "table empty after use");

    drive_reuse(rng);
    drive_oracle(rng);
    CHECK(std::strlen(ps_strerror(PS_ESCRATCH)) > 0 && std::strlen(ps_strerror(-99)) > 0 && std::strlen(ps_last_hip_error()) == 0, "strings");
    {   // a valid call where no device answers: an error code and the runtime's text, nothing else
        const ps_conv_desc d = desc(1, 16, 8, 8, 16, 3, 3, 1, 1, 0);
        alignas(16) static float buf[16 * 64 * 9];
        CHECK(ps_conv2d_fwd_static(&d, nullptr, buf, buf, buf, nullptr) == PS_EHIP && std::strlen(ps_last_hip_error()) > 0, "no-device call");
        ps_tile t;
        double us;
        CHECK(ps_tile_autotune(&d, 3, buf, buf, buf, nullptr, 0, nullptr, &t, &us) == PS_EHIP, "autotune without a device");
        CHECK(ps_tile_autotune(&d, 0, buf, buf, buf, nullptr, 0, nullptr, &t, &us) == PS_EINVAL, "autotune with k = 0");
        CHECK(ps_tile_autotune(&d, 3, nullptr, buf, buf, nullptr, 0, nullptr, &t, &us) == PS_EINVAL, "autotune with a null tensor");
    }
    std::printf("host sanitizer driver: %d errors\n", g_errors);
    return g_errors == 0 ? 0 : 1;
}
