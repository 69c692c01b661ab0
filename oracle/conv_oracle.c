/*
 * CPU oracle for forward 2-D convolution.  TEST INFRASTRUCTURE ONLY: a slow, plain,
 * obviously-correct statement of what the GPU path must compute.  Nothing in the product
 * path may call it, and it shares no code, header or table with the GPU library.
 *
 * What is computed: the convolution of the paper's Fig. 4 ("The 2-D Convolution code",
 * Section 5) with its channel blocking undone, i.e. with c = ifm_tile*16 + ifm,
 * k = ofm_tile*16 + ofm, input row = oj*STRIDE_H + kj, input column = oi*STRIDE_W + ki:
 *
 *   out[n][k][p][q] = sum_{c<C} sum_{r<R} sum_{s<S}
 *                         x(n, c, p*stride + r - pad, q*stride + s - pad) * w[k][c][r][s]
 *   x(n,c,h,w)      = in[n][c][h][w] if 0 <= h < H and 0 <= w < W, else 0
 *   mag[n][k][p][q] = the same sum over |x * w|        (denominator of the relative error)
 *
 * It is a cross-correlation (no filter flip: the index is ij + kj in Fig. 4).  Tensors are
 * plain dense NCHW / KCRS / NKPQ.  Every product and every sum is taken in double
 * precision; inputs are fp32 (bf16 test values arrive already widened, exactly, to fp32).
 * The output starts from zero (the figure's "+=" presumes a cleared output).
 *
 * Readings where the paper is silent: the figure reads a physically pre-padded input and
 * lists "padding" only as a layer parameter (Section 2); here padding is logical zero
 * padding, symmetric, one value for both dimensions, and stride is one value for both
 * dimensions.  Output size is floor((H + 2*pad - R)/stride) + 1.
 *
 * Parallelism: OpenMP over (n, k), the same axis family the paper parallelises
 * ("omp parallel for" over img).  The order of additions inside one output is fixed
 * (c, then r, then s), so results are reproducible for any thread count.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t N, C, H, W, K, R, S, stride, pad;
} oracle_shape;

int oracle_out_dims(const oracle_shape *sh, int32_t *P, int32_t *Q)
{
    if (!sh || sh->N <= 0 || sh->C <= 0 || sh->H <= 0 || sh->W <= 0 || sh->K <= 0 ||
        sh->R <= 0 || sh->S <= 0 || sh->stride <= 0 || sh->pad < 0)
        return -1;
    int hp = sh->H + 2 * sh->pad - sh->R;
    int wp = sh->W + 2 * sh->pad - sh->S;
    if (hp < 0 || wp < 0)
        return -1;
    *P = hp / sh->stride + 1;
    *Q = wp / sh->stride + 1;
    return 0;
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* in: [N][C][H][W] fp32; wt: [K][C][R][S] fp32; out, mag: [N][K][P][Q] fp64 (mag may be NULL).
 * Images n0 <= n < n1 only are computed (others left untouched), so a caller can time or
 * check a bounded sample of a large layer. */
int oracle_conv2d_fwd_range(const oracle_shape *sh, const float *in, const float *wt,
                            double *out, double *mag, int32_t n0, int32_t n1)
{
    int32_t P, Q;
    if (oracle_out_dims(sh, &P, &Q) != 0 || !in || !wt || !out)
        return -1;
    if (n0 < 0 || n1 > sh->N || n0 > n1)
        return -1;
    const int C = sh->C, H = sh->H, W = sh->W, K = sh->K, R = sh->R, S = sh->S;
    const int st = sh->stride, pad = sh->pad;

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = n0; n < n1; ++n) {
        for (int k = 0; k < K; ++k) {
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0, amag = 0.0;
                    for (int c = 0; c < C; ++c) {
                        for (int r = 0; r < R; ++r) {
                            const int h = p * st + r - pad;
                            if (h < 0 || h >= H)
                                continue; /* zero-padding row: contributes 0 */
                            for (int s = 0; s < S; ++s) {
                                const int w = q * st + s - pad;
                                if (w < 0 || w >= W)
                                    continue; /* zero-padding column */
                                const double xv = (double)in[(((size_t)n * C + c) * H + h) * W + w];
                                const double wv = (double)wt[(((size_t)k * C + c) * R + r) * S + s];
                                const double t = xv * wv;
                                acc += t;
                                amag += fabs(t);
                            }
                        }
                    }
                    const size_t o = (((size_t)n * K + k) * P + p) * Q + q;
                    out[o] = acc;
                    if (mag)
                        mag[o] = amag;
                }
            }
        }
    }
    return 0;
}

int oracle_conv2d_fwd(const oracle_shape *sh, const float *in, const float *wt, double *out,
                      double *mag)
{
    if (!sh)
        return -1;
    return oracle_conv2d_fwd_range(sh, in, wt, out, mag, 0, sh->N);
}

/* One output element, for spot checks of layers too large to compute whole. */
int oracle_conv2d_fwd_point(const oracle_shape *sh, const float *in, const float *wt, int32_t n,
                            int32_t k, int32_t p, int32_t q, double *out, double *mag)
{
    int32_t P, Q;
    if (oracle_out_dims(sh, &P, &Q) != 0 || !in || !wt || !out)
        return -1;
    if (n < 0 || n >= sh->N || k < 0 || k >= sh->K || p < 0 || p >= P || q < 0 || q >= Q)
        return -1;
    double acc = 0.0, amag = 0.0;
    for (int c = 0; c < sh->C; ++c)
        for (int r = 0; r < sh->R; ++r) {
            const int h = p * sh->stride + r - sh->pad;
            if (h < 0 || h >= sh->H)
                continue;
            for (int s = 0; s < sh->S; ++s) {
                const int w = q * sh->stride + s - sh->pad;
                if (w < 0 || w >= sh->W)
                    continue;
                const double t =
                    (double)in[(((size_t)n * sh->C + c) * sh->H + h) * sh->W + w] *
                    (double)wt[(((size_t)k * sh->C + c) * sh->R + r) * sh->S + s];
                acc += t;
                amag += fabs(t);
            }
        }
    *out = acc;
    if (mag)
        *mag = amag;
    return 0;
}
