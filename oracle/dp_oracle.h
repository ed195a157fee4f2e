/*
 * dp_oracle.h -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what the DPSGD gradient-privatisation step
 * computes (NanoBatch Privacy, Section 2, first equation):
 *
 *     g_t = 1/|B| * ( N(0, sigma^2 C^2 I) + sum_{x_j in B} clip(grad L(theta, x_j), C) )
 *
 * with clip(g, C) = g * min(1, C / ||g||_2) and, for per-layer / per-stage clipping
 * (Section 3.5), one bound C_g = C / sqrt(M) per group of parameter tensors.
 *
 * It loops over examples, one at a time, with direct nested loops and shares no code,
 * header or table with the HIP library.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may use it.
 *
 * All tensors are host pointers owned by the caller.  Activations / output gradients
 * come as float (fp32 values, or bf16 values widened exactly) and are converted to
 * double element by element; every sum is carried in double.
 *
 * Pins (see tests/): Philox known-answer vectors of the published algorithm, finite
 * differences, library GEMM / autograd special cases, closed-form norms, the clip
 * invariant, noise moments; for the per-example noise form its moments, the independence of
 * the examples' draws and the documented counter / key words; for the SGD step the closed-form
 * momentum series and a library optimiser; for clipping units the unit-of-one case, a worked
 * scalar example, a library autograd mean-loss gradient and the sum-form identity.  No function
 * here is "parity unpinned".
 */
#ifndef DP_ORACLE_H
#define DP_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_DENSE = 0, ORC_CONV2D = 1, ORC_GN_AFFINE = 2 };

typedef struct {
    int kind;
    int cin, cout;      /* dense: in/out features; GroupNorm: cin == cout == channels      */
    int h, w;           /* conv / GroupNorm: input height, width; dense: h = tokens, w = 1 */
    int kh, kw, stride, pad;   /* conv only (cross-correlation, zero padding, dilation 1)  */
    int has_bias;       /* conv / dense: bias present; GroupNorm always has scale + shift  */
    int gn_groups;
    double gn_eps;
    int group;          /* clipping group of this layer's tensors, 0 <= group < n_groups   */
} orc_layer;

/* Shapes. */
int    orc_out_h(const orc_layer *l);
int    orc_out_w(const orc_layer *l);
size_t orc_x_elems(const orc_layer *l);      /* elements of one example's input activation */
size_t orc_dy_elems(const orc_layer *l);     /* elements of one example's output gradient  */
size_t orc_w_elems(const orc_layer *l);      /* weight (or GroupNorm scale) parameters     */
size_t orc_b_elems(const orc_layer *l);      /* bias (or GroupNorm shift) parameters       */

/* One element of one example's weight / bias gradient, straight from the definition.
 * x, dy point at THAT example's tensors.  `e` is the flat index into the parameter
 * tensor ([cout,cin,kh,kw], [out,in], or [c]).                                           */
double orc_weight_grad_elem(const orc_layer *l, const float *x, const float *dy, size_t e);
double orc_bias_grad_elem(const orc_layer *l, const float *x, const float *dy, size_t e);

/* Whole per-example gradient of one layer: gw[orc_w_elems], gb[orc_b_elems] (gb may be
 * NULL when the layer has no bias).                                                      */
void orc_example_grad(const orc_layer *l, const float *x, const float *dy, double *gw, double *gb);

/* sum of squares */
double orc_sqnorm(const double *g, size_t n);

/* min(1, C / sqrt(n2)); 1 when n2 == 0 or C is +inf.                                      */
double orc_clip_factor(double n2, double clip_c);

/* Bounds for M = n_groups clipping groups (Section 3.5): group_clip[g] = clip_c / sqrt(M) for every g,
 * *clip_total = sqrt(sum_g group_clip[g]^2), the bound on the whole clipped gradient (scales the noise). */
void orc_group_bounds(double clip_c, int n_groups, double *group_clip, double *clip_total);

/* One micro-step of clip-and-accumulate over n examples:
 *   for each example i: per-layer gradients, per-group squared norms n2[i*n_groups + g],
 *   factors f[i*n_groups + g], then acc_w[l] += f * gw, acc_b[l] += f * gb.
 * x[l], dy[l]: [n, ...] per layer.  acc_w[l] / acc_b[l]: double accumulators (acc_b[l]
 * may be NULL when the layer has no bias); they are added to, never cleared.  n2 and f may
 * be NULL.  threads <= 0 uses every online core (examples are spread over threads, each
 * with a private accumulator that is added once at the end).  Returns 0, or -1 on a bad
 * argument / allocation failure.                                                           */
int orc_clip_accumulate(const orc_layer *layers, int n_layers,
                        const float *const *x, const float *const *dy, int n,
                        int n_groups, const double *group_clip,
                        double *const *acc_w, double *const *acc_b,
                        double *n2, double *f, int threads);

/* The same micro-step with CLIPPING UNITS of `unit` consecutive examples (the micro-batching of the
 * GPU baseline, Abstract and Table 1: the gradient of a micro-batch is clipped instead of the gradient
 * of each example).  For each unit u = examples [u*unit, (u+1)*unit):
 *   gbar_u = 1/unit * sum of the unit's per-example gradients (the gradient of the unit's mean loss),
 *   per-group squared norms of gbar_u, factors, then acc += f * gbar_u.
 * n must be a multiple of unit; n2 and f (may be NULL) have n/unit rows.  unit == 1 is
 * orc_clip_accumulate.  Returns 0, or -1 on a bad argument / allocation failure.               */
int orc_clip_accumulate_units(const orc_layer *layers, int n_layers,
                              const float *const *x, const float *const *dy, int n, int unit,
                              int n_groups, const double *group_clip,
                              double *const *acc_w, double *const *acc_b,
                              double *n2, double *f, int threads);

/* Selected elements of sum_i f[i] * g_i for one layer (weights if is_bias == 0). */
void orc_weighted_sum_elems(const orc_layer *l, const float *x, const float *dy, int n,
                            const double *f, const size_t *idx, size_t n_idx, int is_bias,
                            double *out);

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11). */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* Noise stream contract: flat elements 4q..4q+3 of tensor `tensor_id` come from the call
 * with counter (q lo, q hi, tensor_id, step lo) and key (seed lo, seed hi).
 * raw[e]: the 32-bit draw behind element e.  u = ((raw >> 9) + 0.5) * 2^-23.
 * Box-Muller on (u0,u1) -> z0 = r cos(2 pi u1), z1 = r sin(2 pi u1), r = sqrt(-2 ln u0);
 * (u2,u3) -> z2, z3 likewise.                                                             */
void orc_noise_raw(uint64_t seed, uint64_t step, uint32_t tensor_id, size_t first, size_t count,
                   uint32_t *raw);
void orc_noise_normal(uint64_t seed, uint64_t step, uint32_t tensor_id, size_t first, size_t count,
                      double *z);

/* out[e] = (acc[e] + sigma * clip_total * z_e) / total_batch.  sigma == 0 draws nothing. */
void orc_noise_finalize(const double *acc, double *out, size_t p, double sigma, double clip_total,
                        uint64_t total_batch, uint64_t seed, uint64_t step, uint32_t tensor_id);

/* acc[e] += sigma * clip_total / sqrt(total_batch) * (sum of the per-example draws of `count` examples
 * starting at example index first_example); see the .c file for the stream. */
void orc_add_example_noise(double *acc, size_t p, double sigma, double clip_total, uint64_t total_batch,
                           uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_example, int count);

/* theta <- theta - lr * v with v <- momentum * v + g (v may be NULL: theta <- theta - lr * g). */
void orc_sgd_update(const double *g, double *theta, double *v, size_t p, double lr, double momentum);

int orc_max_threads(void);

#ifdef __cplusplus
}
#endif
#endif
