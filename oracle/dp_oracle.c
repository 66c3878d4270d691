/*
 * CPU oracle for the per-layer training compute of a data-parallel CNN job.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition against
 * which the GPU library is checked.  It shares no code with the GPU path and
 * nothing in the product may call it.
 *
 * What it computes: the layer operations whose forward+backward time is the
 * planner's comp(i,g) input (paper, section 4.1 "Computation cost"), for the
 * "Conv, Dense" layer kinds of the evaluated models (paper, Table 1).  The
 * paper treats the layers as black boxes, so the arithmetic is the textbook
 * definition of a deep-learning conv2d / linear layer (cross-correlation, zero
 * padding, floor output size), evaluated by direct nested loops in fp64:
 *
 *   fwd    y[n,p,q,k]  = b[k] + sum_{r,s,c} x[n, p*sh-ph+r, q*sw-pw+s, c] * w[k,r,s,c]
 *                        (terms whose input coordinate is outside the image are 0),
 *                        optionally followed by ReLU
 *   dgrad  dx[n,h,w,c] = sum_{k,r,s} g[n,p,q,k] * w[k,r,s,c]
 *                        over the (p,q) with p*sh-ph+r == h and q*sw-pw+s == w
 *   wgrad  dw[k,r,s,c] = sum_{n,p,q} g[n,p,q,k] * x[n, p*sh-ph+r, q*sw-pw+s, c]
 *   db[k]              = sum_{n,p,q} g[n,p,q,k]
 *   where g = dy * [y_saved > 0] if a saved post-ReLU output is given, else dy.
 *
 * Layouts: activations NHWC, weights KRSC (K = output channels), dense.
 * No im2col, no GEMM call, no blocking: one loop nest per definition.
 * OpenMP is used only across independent output elements.
 */
#include <stddef.h>
#include <stdint.h>

typedef struct {
    int n, h, w, c, k, r, s, sh, sw, ph, pw;
} orc_conv;

static int out_h(const orc_conv *d) { return (d->h + 2 * d->ph - d->r) / d->sh + 1; }
static int out_w(const orc_conv *d) { return (d->w + 2 * d->pw - d->s) / d->sw + 1; }

/* ---- forward -------------------------------------------------------- */
static double fwd_elem(const orc_conv *d, const double *x, const double *w,
                       const double *bias, int relu, int n, int p, int q, int k)
{
    double acc = bias ? bias[k] : 0.0;
    for (int r = 0; r < d->r; ++r) {
        int ih = p * d->sh - d->ph + r;
        if (ih < 0 || ih >= d->h) continue;
        for (int s = 0; s < d->s; ++s) {
            int iw = q * d->sw - d->pw + s;
            if (iw < 0 || iw >= d->w) continue;
            const double *xp = x + (((size_t)n * d->h + ih) * d->w + iw) * d->c;
            const double *wp = w + (((size_t)k * d->r + r) * d->s + s) * d->c;
            for (int c = 0; c < d->c; ++c) acc += xp[c] * wp[c];
        }
    }
    if (relu && !(acc > 0.0)) acc = 0.0;
    return acc;
}

void orc_conv2d_fwd(const orc_conv *d, const double *x, const double *w,
                    const double *bias, int relu, double *y)
{
    const int ho = out_h(d), wo = out_w(d);
    const long long rows = (long long)d->n * ho * wo;
#pragma omp parallel for schedule(static)
    for (long long m = 0; m < rows; ++m) {
        int q = (int)(m % wo);
        int p = (int)((m / wo) % ho);
        int n = (int)(m / ((long long)wo * ho));
        for (int k = 0; k < d->k; ++k)
            y[(size_t)m * d->k + k] = fwd_elem(d, x, w, bias, relu, n, p, q, k);
    }
}

/* ---- masked upstream gradient --------------------------------------- */
static inline double gmask(const double *dy, const double *ysaved, size_t i)
{
    if (ysaved && !(ysaved[i] > 0.0)) return 0.0;
    return dy[i];
}

/* ---- backward data -------------------------------------------------- */
static double dgrad_elem(const orc_conv *d, const double *dy, const double *ysaved,
                         const double *w, int n, int h, int wi, int c)
{
    const int ho = out_h(d), wo = out_w(d);
    double acc = 0.0;
    for (int r = 0; r < d->r; ++r) {
        int hp = h + d->ph - r;
        if (hp < 0 || hp % d->sh != 0) continue;
        int p = hp / d->sh;
        if (p >= ho) continue;
        for (int s = 0; s < d->s; ++s) {
            int wq = wi + d->pw - s;
            if (wq < 0 || wq % d->sw != 0) continue;
            int q = wq / d->sw;
            if (q >= wo) continue;
            size_t gbase = (((size_t)n * ho + p) * wo + q) * d->k;
            for (int k = 0; k < d->k; ++k)
                acc += gmask(dy, ysaved, gbase + k) *
                       w[(((size_t)k * d->r + r) * d->s + s) * d->c + c];
        }
    }
    return acc;
}

void orc_conv2d_bwd_data(const orc_conv *d, const double *dy, const double *ysaved,
                         const double *w, double *dx)
{
    const long long rows = (long long)d->n * d->h * d->w;
#pragma omp parallel for schedule(static)
    for (long long m = 0; m < rows; ++m) {
        int wi = (int)(m % d->w);
        int h = (int)((m / d->w) % d->h);
        int n = (int)(m / ((long long)d->w * d->h));
        for (int c = 0; c < d->c; ++c)
            dx[(size_t)m * d->c + c] = dgrad_elem(d, dy, ysaved, w, n, h, wi, c);
    }
}

/* ---- backward filter ------------------------------------------------ */
static double wgrad_elem(const orc_conv *d, const double *x, const double *dy,
                         const double *ysaved, int k, int r, int s, int c)
{
    const int ho = out_h(d), wo = out_w(d);
    double acc = 0.0;
    for (int n = 0; n < d->n; ++n)
        for (int p = 0; p < ho; ++p) {
            int ih = p * d->sh - d->ph + r;
            if (ih < 0 || ih >= d->h) continue;
            for (int q = 0; q < wo; ++q) {
                int iw = q * d->sw - d->pw + s;
                if (iw < 0 || iw >= d->w) continue;
                size_t gi = (((size_t)n * ho + p) * wo + q) * d->k + k;
                acc += gmask(dy, ysaved, gi) *
                       x[(((size_t)n * d->h + ih) * d->w + iw) * d->c + c];
            }
        }
    return acc;
}

void orc_conv2d_bwd_filter(const orc_conv *d, const double *x, const double *dy,
                           const double *ysaved, double *dw, double *db)
{
    const long long total = (long long)d->k * d->r * d->s * d->c;
#pragma omp parallel for schedule(dynamic, 16)
    for (long long e = 0; e < total; ++e) {
        int c = (int)(e % d->c);
        int s = (int)((e / d->c) % d->s);
        int r = (int)((e / ((long long)d->c * d->s)) % d->r);
        int k = (int)(e / ((long long)d->c * d->s * d->r));
        dw[e] = wgrad_elem(d, x, dy, ysaved, k, r, s, c);
    }
    if (db) {
        const long long rows = (long long)d->n * out_h(d) * out_w(d);
#pragma omp parallel for schedule(static)
        for (int k = 0; k < d->k; ++k) {
            double acc = 0.0;
            for (long long m = 0; m < rows; ++m) acc += gmask(dy, ysaved, (size_t)m * d->k + k);
            db[k] = acc;
        }
    }
}

/* ---- ReLU gradient + bias gradient on a [rows, k] matrix ------------- */
void orc_relu_bias_grad(long long rows, int k, const double *dy, const double *ysaved,
                        double *g_out, double *db)
{
    if (g_out) {
#pragma omp parallel for schedule(static)
        for (long long i = 0; i < rows * k; ++i) g_out[i] = gmask(dy, ysaved, (size_t)i);
    }
    if (db) {
#pragma omp parallel for schedule(static)
        for (int j = 0; j < k; ++j) {
            double acc = 0.0;
            for (long long m = 0; m < rows; ++m) acc += gmask(dy, ysaved, (size_t)m * k + j);
            db[j] = acc;
        }
    }
}

/* ---- dense layer: y = x W^T + b ; dx = g W ; dW = g^T x ; db = sum_n g -- */
void orc_linear_fwd(int n, int in_f, int out_f, const double *x, const double *W,
                    const double *bias, int relu, double *y)
{
#pragma omp parallel for schedule(static)
    for (long long e = 0; e < (long long)n * out_f; ++e) {
        int o = (int)(e % out_f), i = (int)(e / out_f);
        double acc = bias ? bias[o] : 0.0;
        for (int j = 0; j < in_f; ++j) acc += x[(size_t)i * in_f + j] * W[(size_t)o * in_f + j];
        if (relu && !(acc > 0.0)) acc = 0.0;
        y[e] = acc;
    }
}

void orc_linear_bwd(int n, int in_f, int out_f, const double *x, const double *W,
                    const double *dy, const double *ysaved,
                    double *dx, double *dW, double *db)
{
    if (dx) {
#pragma omp parallel for schedule(static)
        for (long long e = 0; e < (long long)n * in_f; ++e) {
            int j = (int)(e % in_f), i = (int)(e / in_f);
            double acc = 0.0;
            for (int o = 0; o < out_f; ++o)
                acc += gmask(dy, ysaved, (size_t)i * out_f + o) * W[(size_t)o * in_f + j];
            dx[e] = acc;
        }
    }
    if (dW) {
#pragma omp parallel for schedule(static)
        for (long long e = 0; e < (long long)out_f * in_f; ++e) {
            int j = (int)(e % in_f), o = (int)(e / in_f);
            double acc = 0.0;
            for (int i = 0; i < n; ++i)
                acc += gmask(dy, ysaved, (size_t)i * out_f + o) * x[(size_t)i * in_f + j];
            dW[e] = acc;
        }
    }
    if (db) {
        for (int o = 0; o < out_f; ++o) {
            double acc = 0.0;
            for (int i = 0; i < n; ++i) acc += gmask(dy, ysaved, (size_t)i * out_f + o);
            db[o] = acc;
        }
    }
}

/* ---- single-element evaluation at listed flat output indices --------
 * Same definitions, for spot checks at sizes where the full tensor is too
 * slow.  Inputs are fp32 arrays (every bf16 / fp32 test value is exactly
 * representable) and are widened to fp64 before any arithmetic.
 */
static inline double gmaskf(const float *dy, const float *ysaved, size_t i)
{
    if (ysaved && !(ysaved[i] > 0.0f)) return 0.0;
    return (double)dy[i];
}

void orc_conv2d_fwd_at(const orc_conv *d, const float *x, const float *w, const float *bias,
                       int relu, const long long *idx, long long n_idx, double *out)
{
    const int ho = out_h(d), wo = out_w(d);
#pragma omp parallel for schedule(dynamic, 64)
    for (long long t = 0; t < n_idx; ++t) {
        long long e = idx[t];
        int k = (int)(e % d->k);
        long long m = e / d->k;
        int q = (int)(m % wo), p = (int)((m / wo) % ho), n = (int)(m / ((long long)wo * ho));
        double acc = bias ? (double)bias[k] : 0.0;
        for (int r = 0; r < d->r; ++r) {
            int ih = p * d->sh - d->ph + r;
            if (ih < 0 || ih >= d->h) continue;
            for (int s = 0; s < d->s; ++s) {
                int iw = q * d->sw - d->pw + s;
                if (iw < 0 || iw >= d->w) continue;
                const float *xp = x + (((size_t)n * d->h + ih) * d->w + iw) * d->c;
                const float *wp = w + (((size_t)k * d->r + r) * d->s + s) * d->c;
                for (int c = 0; c < d->c; ++c) acc += (double)xp[c] * (double)wp[c];
            }
        }
        if (relu && !(acc > 0.0)) acc = 0.0;
        out[t] = acc;
    }
}

void orc_conv2d_bwd_data_at(const orc_conv *d, const float *dy, const float *ysaved,
                            const float *w, const long long *idx, long long n_idx, double *out)
{
    const int ho = out_h(d), wo = out_w(d);
#pragma omp parallel for schedule(dynamic, 64)
    for (long long t = 0; t < n_idx; ++t) {
        long long e = idx[t];
        int c = (int)(e % d->c);
        long long m = e / d->c;
        int wi = (int)(m % d->w), h = (int)((m / d->w) % d->h), n = (int)(m / ((long long)d->w * d->h));
        double acc = 0.0;
        for (int r = 0; r < d->r; ++r) {
            int hp = h + d->ph - r;
            if (hp < 0 || hp % d->sh != 0) continue;
            int p = hp / d->sh;
            if (p >= ho) continue;
            for (int s = 0; s < d->s; ++s) {
                int wq = wi + d->pw - s;
                if (wq < 0 || wq % d->sw != 0) continue;
                int q = wq / d->sw;
                if (q >= wo) continue;
                size_t gbase = (((size_t)n * ho + p) * wo + q) * d->k;
                for (int k = 0; k < d->k; ++k)
                    acc += gmaskf(dy, ysaved, gbase + k) *
                           (double)w[(((size_t)k * d->r + r) * d->s + s) * d->c + c];
            }
        }
        out[t] = acc;
    }
}

void orc_conv2d_bwd_filter_at(const orc_conv *d, const float *x, const float *dy,
                              const float *ysaved, const long long *idx, long long n_idx,
                              double *out)
{
    const int ho = out_h(d), wo = out_w(d);
#pragma omp parallel for schedule(dynamic, 4)
    for (long long t = 0; t < n_idx; ++t) {
        long long e = idx[t];
        int c = (int)(e % d->c);
        int s = (int)((e / d->c) % d->s);
        int r = (int)((e / ((long long)d->c * d->s)) % d->r);
        int k = (int)(e / ((long long)d->c * d->s * d->r));
        double acc = 0.0;
        for (int n = 0; n < d->n; ++n)
            for (int p = 0; p < ho; ++p) {
                int ih = p * d->sh - d->ph + r;
                if (ih < 0 || ih >= d->h) continue;
                for (int q = 0; q < wo; ++q) {
                    int iw = q * d->sw - d->pw + s;
                    if (iw < 0 || iw >= d->w) continue;
                    size_t gi = (((size_t)n * ho + p) * wo + q) * d->k + k;
                    acc += gmaskf(dy, ysaved, gi) *
                           (double)x[(((size_t)n * d->h + ih) * d->w + iw) * d->c + c];
                }
            }
        out[t] = acc;
    }
}

void orc_linear_fwd_at(int n, int in_f, int out_f, const float *x, const float *W,
                       const float *bias, int relu, const long long *idx, long long n_idx,
                       double *out)
{
    (void)n;
#pragma omp parallel for schedule(dynamic, 64)
    for (long long t = 0; t < n_idx; ++t) {
        int o = (int)(idx[t] % out_f), i = (int)(idx[t] / out_f);
        double acc = bias ? (double)bias[o] : 0.0;
        for (int j = 0; j < in_f; ++j)
            acc += (double)x[(size_t)i * in_f + j] * (double)W[(size_t)o * in_f + j];
        if (relu && !(acc > 0.0)) acc = 0.0;
        out[t] = acc;
    }
}

void orc_linear_dx_at(int n, int in_f, int out_f, const float *W, const float *dy,
                      const float *ysaved, const long long *idx, long long n_idx, double *out)
{
    (void)n;
#pragma omp parallel for schedule(dynamic, 64)
    for (long long t = 0; t < n_idx; ++t) {
        int j = (int)(idx[t] % in_f), i = (int)(idx[t] / in_f);
        double acc = 0.0;
        for (int o = 0; o < out_f; ++o)
            acc += gmaskf(dy, ysaved, (size_t)i * out_f + o) * (double)W[(size_t)o * in_f + j];
        out[t] = acc;
    }
}

void orc_linear_dw_at(int n, int in_f, int out_f, const float *x, const float *dy,
                      const float *ysaved, const long long *idx, long long n_idx, double *out)
{
#pragma omp parallel for schedule(dynamic, 256)
    for (long long t = 0; t < n_idx; ++t) {
        int j = (int)(idx[t] % in_f), o = (int)(idx[t] / in_f);
        double acc = 0.0;
        for (int i = 0; i < n; ++i)
            acc += gmaskf(dy, ysaved, (size_t)i * out_f + o) * (double)x[(size_t)i * in_f + j];
        out[t] = acc;
    }
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
