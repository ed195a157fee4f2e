/*
 * dp_oracle.c -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT (see dp_oracle.h).
 *
 * fp64, one example at a time, direct loops.  Written from the definitions:
 *   DPSGD step ............ NanoBatch Privacy, Section 2, first equation
 *   per-group bound ....... Section 3.5 (each of M groups clipped to C / sqrt(M))
 *   Philox4x32-10 ......... Salmon et al., "Parallel random numbers: as easy as 1, 2, 3", SC'11
 */
#include "dp_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ shapes */

int orc_out_h(const orc_layer *l)
{
    if (l->kind == ORC_CONV2D) return (l->h + 2 * l->pad - l->kh) / l->stride + 1;
    return l->h;
}

int orc_out_w(const orc_layer *l)
{
    if (l->kind == ORC_CONV2D) return (l->w + 2 * l->pad - l->kw) / l->stride + 1;
    return l->w;
}

size_t orc_x_elems(const orc_layer *l)
{
    return (size_t)l->cin * (size_t)l->h * (size_t)l->w;   /* dense: tokens * in */
}

size_t orc_dy_elems(const orc_layer *l)
{
    if (l->kind == ORC_GN_AFFINE) return orc_x_elems(l);
    return (size_t)l->cout * (size_t)orc_out_h(l) * (size_t)orc_out_w(l);
}

size_t orc_w_elems(const orc_layer *l)
{
    if (l->kind == ORC_GN_AFFINE) return (size_t)l->cin;
    if (l->kind == ORC_DENSE) return (size_t)l->cout * (size_t)l->cin;
    return (size_t)l->cout * (size_t)l->cin * (size_t)l->kh * (size_t)l->kw;
}

size_t orc_b_elems(const orc_layer *l)
{
    if (l->kind == ORC_GN_AFFINE) return (size_t)l->cin;
    return l->has_bias ? (size_t)l->cout : 0;
}

/* ------------------------------------------- per-example gradient elements */

/* conv: dW[co,ci,kh,kw] = sum_{oh,ow} dY[co,oh,ow] * Xpad[ci, oh*s+kh-p, ow*s+kw-p];
 * positions that fall in the zero padding contribute nothing.                      */
static double conv_dw(const orc_layer *l, const float *x, const float *dy,
                      int co, int ci, int kh, int kw)
{
    const int oh_n = orc_out_h(l), ow_n = orc_out_w(l);
    double s = 0.0;
    for (int oh = 0; oh < oh_n; ++oh) {
        const int ih = oh * l->stride + kh - l->pad;
        if (ih < 0 || ih >= l->h) continue;
        for (int ow = 0; ow < ow_n; ++ow) {
            const int iw = ow * l->stride + kw - l->pad;
            if (iw < 0 || iw >= l->w) continue;
            s += (double)dy[((size_t)co * oh_n + oh) * ow_n + ow] *
                 (double)x[((size_t)ci * l->h + ih) * l->w + iw];
        }
    }
    return s;
}

/* conv: db[co] = sum_{oh,ow} dY[co,oh,ow] */
static double conv_db(const orc_layer *l, const float *dy, int co)
{
    const size_t s_n = (size_t)orc_out_h(l) * (size_t)orc_out_w(l);
    double s = 0.0;
    for (size_t p = 0; p < s_n; ++p) s += (double)dy[(size_t)co * s_n + p];
    return s;
}

/* dense over T tokens: dW[o,k] = sum_t dY[t,o] * X[t,k];  db[o] = sum_t dY[t,o] */
static double dense_dw(const orc_layer *l, const float *x, const float *dy, int o, int k)
{
    double s = 0.0;
    for (int t = 0; t < l->h; ++t)
        s += (double)dy[(size_t)t * l->cout + o] * (double)x[(size_t)t * l->cin + k];
    return s;
}

static double dense_db(const orc_layer *l, const float *dy, int o)
{
    double s = 0.0;
    for (int t = 0; t < l->h; ++t) s += (double)dy[(size_t)t * l->cout + o];
    return s;
}

/* GroupNorm statistics of the group that holds channel c: mean and biased variance
 * over the (C/G)*H*W elements of that group.                                        */
static void gn_stats(const orc_layer *l, const float *x, int c, double *mean, double *var)
{
    const int cg = l->cin / l->gn_groups;
    const int g = c / cg;
    const size_t hw = (size_t)l->h * (size_t)l->w;
    const size_t first = (size_t)g * cg * hw, cnt = (size_t)cg * hw;
    double m = 0.0;
    for (size_t p = 0; p < cnt; ++p) m += (double)x[first + p];
    m /= (double)cnt;
    double v = 0.0;
    for (size_t p = 0; p < cnt; ++p) {
        const double d = (double)x[first + p] - m;
        v += d * d;
    }
    *mean = m;
    *var = v / (double)cnt;
}

/* GroupNorm scale: dgamma[c] = sum_{h,w} dY[c,h,w] * xhat[c,h,w], xhat = (x-mean)/sqrt(var+eps) */
static double gn_dgamma(const orc_layer *l, const float *x, const float *dy, int c)
{
    double mean, var;
    gn_stats(l, x, c, &mean, &var);
    const double rstd = 1.0 / sqrt(var + l->gn_eps);
    const size_t hw = (size_t)l->h * (size_t)l->w;
    double s = 0.0;
    for (size_t p = 0; p < hw; ++p)
        s += (double)dy[(size_t)c * hw + p] * (((double)x[(size_t)c * hw + p] - mean) * rstd);
    return s;
}

/* GroupNorm shift: dbeta[c] = sum_{h,w} dY[c,h,w] */
static double gn_dbeta(const orc_layer *l, const float *dy, int c)
{
    const size_t hw = (size_t)l->h * (size_t)l->w;
    double s = 0.0;
    for (size_t p = 0; p < hw; ++p) s += (double)dy[(size_t)c * hw + p];
    return s;
}

double orc_weight_grad_elem(const orc_layer *l, const float *x, const float *dy, size_t e)
{
    switch (l->kind) {
    case ORC_DENSE:
        return dense_dw(l, x, dy, (int)(e / (size_t)l->cin), (int)(e % (size_t)l->cin));
    case ORC_CONV2D: {
        const int kw = (int)(e % (size_t)l->kw);  e /= (size_t)l->kw;
        const int kh = (int)(e % (size_t)l->kh);  e /= (size_t)l->kh;
        const int ci = (int)(e % (size_t)l->cin); e /= (size_t)l->cin;
        return conv_dw(l, x, dy, (int)e, ci, kh, kw);
    }
    default:
        return gn_dgamma(l, x, dy, (int)e);
    }
}

double orc_bias_grad_elem(const orc_layer *l, const float *x, const float *dy, size_t e)
{
    (void)x;
    switch (l->kind) {
    case ORC_DENSE:  return dense_db(l, dy, (int)e);
    case ORC_CONV2D: return conv_db(l, dy, (int)e);
    default:         return gn_dbeta(l, dy, (int)e);
    }
}

void orc_example_grad(const orc_layer *l, const float *x, const float *dy, double *gw, double *gb)
{
    const size_t pw = orc_w_elems(l), pb = orc_b_elems(l);
    for (size_t e = 0; e < pw; ++e) gw[e] = orc_weight_grad_elem(l, x, dy, e);
    if (gb)
        for (size_t e = 0; e < pb; ++e) gb[e] = orc_bias_grad_elem(l, x, dy, e);
}

/* ------------------------------------------------------------ norm and clip */

double orc_sqnorm(const double *g, size_t n)
{
    double s = 0.0;
    for (size_t i = 0; i < n; ++i) s += g[i] * g[i];
    return s;
}

double orc_clip_factor(double n2, double clip_c)
{
    if (n2 == 0.0) return 1.0;
    const double r = clip_c / sqrt(n2);
    return r < 1.0 ? r : 1.0;
}

/* Per-group bounds (Section 3.5): with M clipping groups every group is clipped to C / sqrt(M), so that
 * the squared group norms add up to at most C^2; the noise is scaled by the bound on the whole clipped
 * gradient, sqrt(sum_g C_g^2).  With M = 1 this is the single global bound of Section 2.            */
void orc_group_bounds(double clip_c, int n_groups, double *group_clip, double *clip_total)
{
    double sum = 0.0;
    for (int g = 0; g < n_groups; ++g) {
        group_clip[g] = clip_c / sqrt((double)n_groups);
        sum += group_clip[g] * group_clip[g];
    }
    *clip_total = sqrt(sum);
}

static double uniform_open(uint32_t r);     /* defined with the noise stream below */

/* Per-example form of the noise (second equation of the Algorithm section): every clipped example
 * carries its own N(0, sigma^2 C^2 / |B|) draw, so the sum over the |B| examples of a step has the
 * variance sigma^2 C^2 of the once-per-step form.  The draws of example j (its index within the
 * optimiser step) come from the same Philox4x32-10 / Box-Muller construction with the example index
 * in the second counter word and a flipped key word, so the two forms never share a draw:
 *   counter (q, j, tensor_id, step lo), key (seed lo, seed hi ^ 0x50455245), elements 4q..4q+3.
 * acc[e] += sigma * clip_total / sqrt(total_batch) * sum_{j = first .. first+count-1} z(j, e).     */
void orc_add_example_noise(double *acc, size_t p, double sigma, double clip_total, uint64_t total_batch,
                           uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_example, int count)
{
    const double two_pi = 6.283185307179586476925286766559;
    const double scale = sigma * clip_total / sqrt((double)total_batch);
    if (sigma == 0.0) return;
    for (size_t e = 0; e < p; ++e) {
        double sum = 0.0;
        for (int jj = 0; jj < count; ++jj) {
            const uint64_t j = first_example + (uint64_t)jj;
            const uint32_t ctr[4] = { (uint32_t)(e / 4), (uint32_t)j, tensor_id, (uint32_t)step };
            const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) ^ 0x50455245u };
            uint32_t r[4];
            orc_philox4x32_10(ctr, key, r);
            const int pair = (int)((e % 4) / 2);
            const double ua = uniform_open(r[2 * pair]), ub = uniform_open(r[2 * pair + 1]);
            const double radius = sqrt(-2.0 * log(ua));
            sum += (e % 2 == 0) ? radius * cos(two_pi * ub) : radius * sin(two_pi * ub);
        }
        acc[e] += scale * sum;
    }
}

/* SGD step on the privatised gradient (Section 2 names SGD with a stepped learning-rate decay as the
 * optimiser; Sections 3.2 and 3.3 run it with momentum 0.9).  g is the finalized
 * gradient of one tensor; the buffer v is the plain heavy-ball momentum: v <- mu v + g,
 * theta <- theta - lr v.  mu == 0 (or v == NULL) is SGD without momentum.                    */
void orc_sgd_update(const double *g, double *theta, double *v, size_t p, double lr, double momentum)
{
    for (size_t e = 0; e < p; ++e) {
        double step = g[e];
        if (v) {
            v[e] = momentum * v[e] + g[e];
            step = v[e];
        }
        theta[e] -= lr * step;
    }
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int orc_clip_accumulate(const orc_layer *layers, int n_layers,
                        const float *const *x, const float *const *dy, int n,
                        int n_groups, const double *group_clip,
                        double *const *acc_w, double *const *acc_b,
                        double *n2_out, double *f_out, int threads)
{
    if (!layers || n_layers <= 0 || n <= 0 || n_groups <= 0 || !group_clip) return -1;
    for (int l = 0; l < n_layers; ++l)
        if (layers[l].group < 0 || layers[l].group >= n_groups) return -1;
    if (threads <= 0) threads = orc_max_threads();
    if (threads > n) threads = n;

    /* offsets of each layer's tensors in one flat parameter vector */
    size_t *off_w = (size_t *)malloc(sizeof(size_t) * (size_t)n_layers);
    size_t *off_b = (size_t *)malloc(sizeof(size_t) * (size_t)n_layers);
    if (!off_w || !off_b) { free(off_w); free(off_b); return -1; }
    size_t total = 0;
    for (int l = 0; l < n_layers; ++l) {
        off_w[l] = total; total += orc_w_elems(&layers[l]);
        off_b[l] = total; total += orc_b_elems(&layers[l]);
    }
    int failed = 0;

#pragma omp parallel num_threads(threads)
    {
        double *g = (double *)malloc(sizeof(double) * total);      /* this example's gradient */
        double *mine = (double *)calloc(total, sizeof(double));    /* this thread's clipped sum */
        double *n2 = (double *)malloc(sizeof(double) * (size_t)n_groups);
        double *f = (double *)malloc(sizeof(double) * (size_t)n_groups);
        if (!g || !mine || !n2 || !f) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 1)
            for (int i = 0; i < n; ++i) {
                /* (a) per-example gradients of every layer */
                for (int l = 0; l < n_layers; ++l) {
                    const orc_layer *L = &layers[l];
                    orc_example_grad(L, x[l] + (size_t)i * orc_x_elems(L),
                                     dy[l] + (size_t)i * orc_dy_elems(L),
                                     g + off_w[l], orc_b_elems(L) ? g + off_b[l] : NULL);
                }
                /* (b) squared L2 norm per clipping group */
                for (int q = 0; q < n_groups; ++q) n2[q] = 0.0;
                for (int l = 0; l < n_layers; ++l) {
                    const orc_layer *L = &layers[l];
                    n2[L->group] += orc_sqnorm(g + off_w[l], orc_w_elems(L));
                    n2[L->group] += orc_sqnorm(g + off_b[l], orc_b_elems(L));
                }
                /* (c) clip factor per group */
                for (int q = 0; q < n_groups; ++q) f[q] = orc_clip_factor(n2[q], group_clip[q]);
                /* (d) clipped sum */
                for (int l = 0; l < n_layers; ++l) {
                    const orc_layer *L = &layers[l];
                    const double fl = f[L->group];
                    const size_t cnt = orc_w_elems(L) + orc_b_elems(L);   /* w then b, adjacent */
                    for (size_t e = 0; e < cnt; ++e) mine[off_w[l] + e] += fl * g[off_w[l] + e];
                }
                for (int q = 0; q < n_groups; ++q) {
                    if (n2_out) n2_out[(size_t)i * n_groups + q] = n2[q];
                    if (f_out) f_out[(size_t)i * n_groups + q] = f[q];
                }
            }
#pragma omp critical
            {
                for (int l = 0; l < n_layers; ++l) {
                    const orc_layer *L = &layers[l];
                    const size_t pw = orc_w_elems(L), pb = orc_b_elems(L);
                    for (size_t e = 0; e < pw; ++e) acc_w[l][e] += mine[off_w[l] + e];
                    if (pb && acc_b && acc_b[l])
                        for (size_t e = 0; e < pb; ++e) acc_b[l][e] += mine[off_b[l] + e];
                }
            }
        }
        free(g); free(mine); free(n2); free(f);
    }
    free(off_w); free(off_b);
    return failed ? -1 : 0;
}

int orc_clip_accumulate_units(const orc_layer *layers, int n_layers,
                              const float *const *x, const float *const *dy, int n, int unit,
                              int n_groups, const double *group_clip,
                              double *const *acc_w, double *const *acc_b,
                              double *n2_out, double *f_out, int threads)
{
    if (!layers || n_layers <= 0 || n <= 0 || unit <= 0 || n % unit || n_groups <= 0 || !group_clip) return -1;
    for (int l = 0; l < n_layers; ++l)
        if (layers[l].group < 0 || layers[l].group >= n_groups) return -1;
    const int units = n / unit;
    if (threads <= 0) threads = orc_max_threads();
    if (threads > units) threads = units;

    size_t *off_w = (size_t *)malloc(sizeof(size_t) * (size_t)n_layers);
    size_t *off_b = (size_t *)malloc(sizeof(size_t) * (size_t)n_layers);
    if (!off_w || !off_b) { free(off_w); free(off_b); return -1; }
    size_t total = 0;
    for (int l = 0; l < n_layers; ++l) {
        off_w[l] = total; total += orc_w_elems(&layers[l]);
        off_b[l] = total; total += orc_b_elems(&layers[l]);
    }
    int failed = 0;

#pragma omp parallel num_threads(threads)
    {
        double *g = (double *)malloc(sizeof(double) * total);      /* one example's gradient */
        double *gbar = (double *)malloc(sizeof(double) * total);   /* the unit's mean gradient */
        double *mine = (double *)calloc(total, sizeof(double));    /* this thread's clipped sum */
        double *n2 = (double *)malloc(sizeof(double) * (size_t)n_groups);
        double *f = (double *)malloc(sizeof(double) * (size_t)n_groups);
        if (!g || !gbar || !mine || !n2 || !f) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 1)
            for (int u = 0; u < units; ++u) {
                /* (a) mean of the unit's per-example gradients */
                for (size_t e = 0; e < total; ++e) gbar[e] = 0.0;
                for (int k = 0; k < unit; ++k) {
                    const int i = u * unit + k;
                    for (int l = 0; l < n_layers; ++l) {
                        const orc_layer *L = &layers[l];
                        orc_example_grad(L, x[l] + (size_t)i * orc_x_elems(L),
                                         dy[l] + (size_t)i * orc_dy_elems(L),
                                         g + off_w[l], orc_b_elems(L) ? g + off_b[l] : NULL);
                    }
                    for (size_t e = 0; e < total; ++e) gbar[e] += g[e];
                }
                for (size_t e = 0; e < total; ++e) gbar[e] /= (double)unit;
                /* (b) squared norm per clipping group, (c) factor, (d) clipped sum */
                for (int q = 0; q < n_groups; ++q) n2[q] = 0.0;
                for (int l = 0; l < n_layers; ++l) {
                    const orc_layer *L = &layers[l];
                    n2[L->group] += orc_sqnorm(gbar + off_w[l], orc_w_elems(L));
                    n2[L->group] += orc_sqnorm(gbar + off_b[l], orc_b_elems(L));
                }
                for (int q = 0; q < n_groups; ++q) f[q] = orc_clip_factor(n2[q], group_clip[q]);
                for (int l = 0; l < n_layers; ++l) {
                    const orc_layer *L = &layers[l];
                    const double fl = f[L->group];
                    const size_t cnt = orc_w_elems(L) + orc_b_elems(L);
                    for (size_t e = 0; e < cnt; ++e) mine[off_w[l] + e] += fl * gbar[off_w[l] + e];
                }
                for (int q = 0; q < n_groups; ++q) {
                    if (n2_out) n2_out[(size_t)u * n_groups + q] = n2[q];
                    if (f_out) f_out[(size_t)u * n_groups + q] = f[q];
                }
            }
#pragma omp critical
            {
                for (int l = 0; l < n_layers; ++l) {
                    const orc_layer *L = &layers[l];
                    const size_t pw = orc_w_elems(L), pb = orc_b_elems(L);
                    for (size_t e = 0; e < pw; ++e) acc_w[l][e] += mine[off_w[l] + e];
                    if (pb && acc_b && acc_b[l])
                        for (size_t e = 0; e < pb; ++e) acc_b[l][e] += mine[off_b[l] + e];
                }
            }
        }
        free(g); free(gbar); free(mine); free(n2); free(f);
    }
    free(off_w); free(off_b);
    return failed ? -1 : 0;
}

void orc_weighted_sum_elems(const orc_layer *l, const float *x, const float *dy, int n,
                            const double *f, const size_t *idx, size_t n_idx, int is_bias,
                            double *out)
{
    const size_t xs = orc_x_elems(l), ys = orc_dy_elems(l);
#pragma omp parallel for schedule(dynamic, 1)
    for (long j = 0; j < (long)n_idx; ++j) {
        double s = 0.0;
        for (int i = 0; i < n; ++i) {
            const float *xi = x + (size_t)i * xs, *dyi = dy + (size_t)i * ys;
            const double g = is_bias ? orc_bias_grad_elem(l, xi, dyi, idx[j])
                                     : orc_weight_grad_elem(l, xi, dyi, idx[j]);
            s += f[i] * g;
        }
        out[j] = s;
    }
}

/* ------------------------------------------------------------------ Philox */

void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {            /* key schedule: Weyl increments between rounds */
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void noise_call(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t q, uint32_t r[4])
{
    const uint32_t ctr[4] = { (uint32_t)q, (uint32_t)(q >> 32), tensor_id, (uint32_t)step };
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    orc_philox4x32_10(ctr, key, r);
}

void orc_noise_raw(uint64_t seed, uint64_t step, uint32_t tensor_id, size_t first, size_t count,
                   uint32_t *raw)
{
    for (size_t j = 0; j < count; ++j) {
        const size_t e = first + j;
        uint32_t r[4];
        noise_call(seed, step, tensor_id, (uint64_t)(e / 4), r);
        raw[j] = r[e % 4];
    }
}

static double uniform_open(uint32_t r)
{
    return ((double)(r >> 9) + 0.5) * (1.0 / 8388608.0);   /* 2^-23; in (0,1), never 0 or 1 */
}

void orc_noise_normal(uint64_t seed, uint64_t step, uint32_t tensor_id, size_t first, size_t count,
                      double *z)
{
    const double two_pi = 6.283185307179586476925286766559;
    for (size_t j = 0; j < count; ++j) {
        const size_t e = first + j;
        uint32_t r[4];
        noise_call(seed, step, tensor_id, (uint64_t)(e / 4), r);
        const int pair = (int)((e % 4) / 2);               /* (u0,u1) or (u2,u3) */
        const double ua = uniform_open(r[2 * pair]), ub = uniform_open(r[2 * pair + 1]);
        const double radius = sqrt(-2.0 * log(ua));
        z[j] = (e % 2 == 0) ? radius * cos(two_pi * ub) : radius * sin(two_pi * ub);
    }
}

void orc_noise_finalize(const double *acc, double *out, size_t p, double sigma, double clip_total,
                        uint64_t total_batch, uint64_t seed, uint64_t step, uint32_t tensor_id)
{
    for (size_t e = 0; e < p; ++e) {
        double noise = 0.0;
        if (sigma != 0.0) {
            double z;
            orc_noise_normal(seed, step, tensor_id, e, 1, &z);
            noise = sigma * clip_total * z;
        }
        out[e] = (acc[e] + noise) / (double)total_batch;
    }
}
