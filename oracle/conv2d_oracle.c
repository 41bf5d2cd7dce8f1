/*
 * CPU oracle for the 2-D spatial convolution layer of convnet training.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP library is
 * checked against; it shares no code, header, table or helper with that
 * library and is never on the product path.
 *
 * What it computes.  The paper (Sec. 4.2, "im2col") states that the
 * convolution of one 3-D image with the 4-D weight tensor equals one product
 * of two 2-D matrices: the K x (C*R*S) weight matrix times the lowered image.
 * Written element by element that product is a sum over (c, r, t) of
 * x * w with no reversal of the filter, i.e. a cross-correlation, with
 * zero contribution from taps that fall outside the image (zero padding).
 * The paper prints no formula, worked example or error bound, so against the
 * paper itself parity is unpinned; the functions below are pinned by
 * mathematics instead (hand-worked cases, identity/shift filters, 1x1 ==
 * matmul, explicit lowering + matmul, the adjoint identity, exact finite
 * differences, exhaustive rational-arithmetic loops on tiny shapes).
 *
 * Definitions (inputs fp32 read exactly, every product and sum in fp64):
 *   P = floor((H + 2*pad_h - R) / stride_h) + 1, Q likewise.
 *   fwd : y[n,k,p,q]  = b[k] + sum_{c,r,t} x[n,c,p*sh-ph+r,q*sw-pw+t] * w[k,c,r,t]
 *   bwdD: dx[n,c,h,u] = sum over all (k,p,q,r,t) whose tap lands on (h,u) of
 *                       dy[n,k,p,q] * w[k,c,r,t]            (the transpose of fwd)
 *   bwdW: dw[k,c,r,t] = scale * sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*sh-ph+r,q*sw-pw+t]
 *         db[k]       = scale * sum_{n,p,q} dy[n,k,p,q]
 * Layouts: x NCHW, w KCRS, y/dy NKPQ, dense and contiguous.
 *
 * No lowering, no blocking, no BLAS, no Winograd: plain loops in the order of
 * the definitions, parallelised with OpenMP over independent output slices only.
 * Return value: 0 ok, -1 bad geometry / null pointer.
 */
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct {
    int N, C, H, W, K, R, S, sh, sw, ph, pw, P, Q;
} geom_t;

static int make_geom(geom_t *g, int N, int C, int H, int W, int K, int R, int S,
                     int sh, int sw, int ph, int pw)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1) return -1;
    if (sh < 1 || sw < 1 || ph < 0 || pw < 0) return -1;
    if (H + 2 * ph < R || W + 2 * pw < S) return -1;
    g->N = N; g->C = C; g->H = H; g->W = W; g->K = K; g->R = R; g->S = S;
    g->sh = sh; g->sw = sw; g->ph = ph; g->pw = pw;
    g->P = (H + 2 * ph - R) / sh + 1;
    g->Q = (W + 2 * pw - S) / sw + 1;
    return 0;
}

int oracle_conv2d_output_dims(int N, int C, int H, int W, int K, int R, int S,
                              int sh, int sw, int ph, int pw, int *P, int *Q)
{
    geom_t g;
    if (!P || !Q || make_geom(&g, N, C, H, W, K, R, S, sh, sw, ph, pw)) return -1;
    *P = g.P; *Q = g.Q;
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}

/* ---------------------------------------------------------------- forward */
int oracle_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S,
                      int sh, int sw, int ph, int pw,
                      const float *x, const float *w, const float *b, double *y)
{
    geom_t g;
    if (!x || !w || !y || make_geom(&g, N, C, H, W, K, R, S, sh, sw, ph, pw)) return -1;
    const int P = g.P, Q = g.Q;
    long nk;
#pragma omp parallel for schedule(dynamic, 1)
    for (nk = 0; nk < (long)N * K; ++nk) {
        const int n = (int)(nk / K), k = (int)(nk % K);
        double *yo = y + (size_t)nk * P * Q;
        for (int i = 0; i < P * Q; ++i) yo[i] = b ? (double)b[k] : 0.0;
        for (int c = 0; c < C; ++c) {
            const float *xc = x + ((size_t)n * C + c) * H * W;
            for (int r = 0; r < R; ++r)
                for (int t = 0; t < S; ++t) {
                    const double wv = (double)w[(((size_t)k * C + c) * R + r) * S + t];
                    for (int p = 0; p < P; ++p) {
                        const int ih = p * sh - ph + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int q = 0; q < Q; ++q) {
                            const int iw = q * sw - pw + t;
                            if (iw < 0 || iw >= W) continue;
                            yo[p * Q + q] += (double)xc[(size_t)ih * W + iw] * wv;
                        }
                    }
                }
        }
    }
    return 0;
}

/* ---------------------------------------------------- backward w.r.t. input */
int oracle_conv2d_bwd_data(int N, int C, int H, int W, int K, int R, int S,
                           int sh, int sw, int ph, int pw,
                           const float *dy, const float *w, double *dx)
{
    geom_t g;
    if (!dy || !w || !dx || make_geom(&g, N, C, H, W, K, R, S, sh, sw, ph, pw)) return -1;
    const int P = g.P, Q = g.Q;
    long nc;
    /* Transpose of the forward map: every forward tap x[ih,iw] -> y[p,q] with
     * weight w[k,c,r,t] sends dy[p,q] back to dx[ih,iw] with the same weight. */
#pragma omp parallel for schedule(dynamic, 1)
    for (nc = 0; nc < (long)N * C; ++nc) {
        const int n = (int)(nc / C), c = (int)(nc % C);
        double *dxo = dx + (size_t)nc * H * W;
        for (int i = 0; i < H * W; ++i) dxo[i] = 0.0;
        for (int k = 0; k < K; ++k) {
            const float *dyk = dy + ((size_t)n * K + k) * P * Q;
            for (int r = 0; r < R; ++r)
                for (int t = 0; t < S; ++t) {
                    const double wv = (double)w[(((size_t)k * C + c) * R + r) * S + t];
                    for (int p = 0; p < P; ++p) {
                        const int ih = p * sh - ph + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int q = 0; q < Q; ++q) {
                            const int iw = q * sw - pw + t;
                            if (iw < 0 || iw >= W) continue;
                            dxo[(size_t)ih * W + iw] += (double)dyk[p * Q + q] * wv;
                        }
                    }
                }
        }
    }
    return 0;
}

/* -------------------------------------------------- backward w.r.t. weights */
int oracle_conv2d_bwd_weight(int N, int C, int H, int W, int K, int R, int S,
                             int sh, int sw, int ph, int pw,
                             const float *x, const float *dy, double scale,
                             double *dw, double *db)
{
    geom_t g;
    if (!x || !dy || !dw || make_geom(&g, N, C, H, W, K, R, S, sh, sw, ph, pw)) return -1;
    const int P = g.P, Q = g.Q;
    long kc;
#pragma omp parallel for schedule(dynamic, 1)
    for (kc = 0; kc < (long)K * C; ++kc) {
        const int k = (int)(kc / C), c = (int)(kc % C);
        for (int r = 0; r < R; ++r)
            for (int t = 0; t < S; ++t) {
                double acc = 0.0;
                for (int n = 0; n < N; ++n) {
                    const float *xc = x + ((size_t)n * C + c) * H * W;
                    const float *dyk = dy + ((size_t)n * K + k) * P * Q;
                    for (int p = 0; p < P; ++p) {
                        const int ih = p * sh - ph + r;
                        if (ih < 0 || ih >= H) continue;
                        for (int q = 0; q < Q; ++q) {
                            const int iw = q * sw - pw + t;
                            if (iw < 0 || iw >= W) continue;
                            acc += (double)dyk[p * Q + q] * (double)xc[(size_t)ih * W + iw];
                        }
                    }
                }
                dw[((size_t)kc * R + r) * S + t] = scale * acc;
            }
    }
    if (db) {
        int k;
#pragma omp parallel for schedule(static)
        for (k = 0; k < K; ++k) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                const float *dyk = dy + ((size_t)n * K + k) * P * Q;
                for (int i = 0; i < P * Q; ++i) acc += (double)dyk[i];
            }
            db[k] = scale * acc;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Single-element evaluators: the same definitions, one output element at a
 * time, for spot checks at sizes where the full tensors would take minutes.
 * idx[] holds flat (row-major) indices into y / dx / dw.  bwd_data is written
 * here in its gather form (which outputs (p,q) does tap (r,t) reach from
 * (h,u)?), a second formulation that the tests compare with the scatter above.
 * ---------------------------------------------------------------------- */
int oracle_conv2d_fwd_at(int N, int C, int H, int W, int K, int R, int S,
                         int sh, int sw, int ph, int pw,
                         const float *x, const float *w, const float *b,
                         const int64_t *idx, int64_t n_idx, double *out)
{
    geom_t g;
    if (!x || !w || !idx || !out || make_geom(&g, N, C, H, W, K, R, S, sh, sw, ph, pw)) return -1;
    const int P = g.P, Q = g.Q;
    int64_t i;
#pragma omp parallel for schedule(dynamic, 64)
    for (i = 0; i < n_idx; ++i) {
        int64_t f = idx[i];
        const int q = (int)(f % Q); f /= Q;
        const int p = (int)(f % P); f /= P;
        const int k = (int)(f % K); f /= K;
        const int n = (int)f;
        double acc = b ? (double)b[k] : 0.0;
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int t = 0; t < S; ++t) {
                    const int ih = p * sh - ph + r, iw = q * sw - pw + t;
                    if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                    acc += (double)x[(((size_t)n * C + c) * H + ih) * W + iw] *
                           (double)w[(((size_t)k * C + c) * R + r) * S + t];
                }
        out[i] = acc;
    }
    return 0;
}

int oracle_conv2d_bwd_data_at(int N, int C, int H, int W, int K, int R, int S,
                              int sh, int sw, int ph, int pw,
                              const float *dy, const float *w,
                              const int64_t *idx, int64_t n_idx, double *out)
{
    geom_t g;
    if (!dy || !w || !idx || !out || make_geom(&g, N, C, H, W, K, R, S, sh, sw, ph, pw)) return -1;
    const int P = g.P, Q = g.Q;
    int64_t i;
#pragma omp parallel for schedule(dynamic, 64)
    for (i = 0; i < n_idx; ++i) {
        int64_t f = idx[i];
        const int u = (int)(f % W); f /= W;
        const int h = (int)(f % H); f /= H;
        const int c = (int)(f % C); f /= C;
        const int n = (int)f;
        double acc = 0.0;
        for (int k = 0; k < K; ++k)
            for (int r = 0; r < R; ++r) {
                const int hp = h + ph - r;
                if (hp < 0 || hp % sh) continue;
                const int p = hp / sh;
                if (p >= P) continue;
                for (int t = 0; t < S; ++t) {
                    const int up = u + pw - t;
                    if (up < 0 || up % sw) continue;
                    const int q = up / sw;
                    if (q >= Q) continue;
                    acc += (double)dy[(((size_t)n * K + k) * P + p) * Q + q] *
                           (double)w[(((size_t)k * C + c) * R + r) * S + t];
                }
            }
        out[i] = acc;
    }
    return 0;
}

int oracle_conv2d_bwd_weight_at(int N, int C, int H, int W, int K, int R, int S,
                                int sh, int sw, int ph, int pw,
                                const float *x, const float *dy, double scale,
                                const int64_t *idx, int64_t n_idx, double *out)
{
    geom_t g;
    if (!x || !dy || !idx || !out || make_geom(&g, N, C, H, W, K, R, S, sh, sw, ph, pw)) return -1;
    const int P = g.P, Q = g.Q;
    int64_t i;
#pragma omp parallel for schedule(dynamic, 1)
    for (i = 0; i < n_idx; ++i) {
        int64_t f = idx[i];
        const int t = (int)(f % S); f /= S;
        const int r = (int)(f % R); f /= R;
        const int c = (int)(f % C); f /= C;
        const int k = (int)f;
        double acc = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < P; ++p) {
                const int ih = p * sh - ph + r;
                if (ih < 0 || ih >= H) continue;
                for (int q = 0; q < Q; ++q) {
                    const int iw = q * sw - pw + t;
                    if (iw < 0 || iw >= W) continue;
                    acc += (double)dy[(((size_t)n * K + k) * P + p) * Q + q] *
                           (double)x[(((size_t)n * C + c) * H + ih) * W + iw];
                }
            }
        out[i] = scale * acc;
    }
    return 0;
}
