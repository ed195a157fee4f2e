/*
 * dp_privatise.h -- C ABI of the MI355X (gfx950) DPSGD gradient-privatisation library.
 *
 * What it computes (NanoBatch Privacy, arxiv 2109.12191, Section 2, first equation):
 *
 *     g_t = 1/|B| * ( N(0, sigma^2 C^2 I) + sum_{x_j in B} clip(grad L(theta, x_j), C) )
 *
 * with clip(g, C) = g * min(1, C / ||g||_2), the sum accumulated over micro-steps
 * (Section 2, gradient accumulation), and optionally one bound C_g = C / sqrt(M) per group
 * of parameter tensors instead of one global bound (Section 3.5).
 *
 * The path is split into the calls below; a caller runs, per micro-step,
 *   dp_per_example_grad  (per layer)      -> per-example, per-layer squared norms
 *   dp_norms                              -> per-example, per-group squared norms
 *   dp_clip_accumulate[_recompute] (per layer) -> acc += sum_i f_i * g_i
 * and once per optimiser step, per parameter tensor,
 *   dp_add_noise_finalize                 -> (acc + sigma*C*z) / |B|
 *
 * Conventions shared by every entry point
 *   - Pointers marked [device] are device memory owned by the caller, valid until the
 *     stream has executed the enqueued work.  Activations, gradients, accumulators, outputs
 *     and workspaces must be 16-byte aligned; the small per-example vectors (squared norms,
 *     factors, group ids, raw random words) need 4-byte alignment only.  Pointers marked [host] are
 *     read before the call returns.  The library allocates, frees and synchronises nothing
 *     and never changes the current device.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously; calls return at once.
 *   - Every argument is validated on the host before anything is launched.  On error no
 *     work is enqueued, the code says why, and dp_last_error() gives a sentence
 *     (thread-local).  Nothing aborts or throws.
 *   - Parameter-gradient tensors use the framework layout: conv [cout, cin, kh, kw],
 *     dense [out, in], GroupNorm scale/shift [c]; fp32.
 *   - Activations x and output gradients dy: NCHW ([n, c, h, w]) for conv / GroupNorm,
 *     [n, tokens, features] for dense; fp32 or bf16 (dp_dtype).  All arithmetic
 *     accumulates in fp32.
 */
#ifndef DP_PRIVATISE_H
#define DP_PRIVATISE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DP_OK = 0,
    DP_ERR_INVALID_ARG = 1,   /* null / misaligned pointer, non-positive size, NaN, C <= 0, sigma < 0 ... */
    DP_ERR_UNSUPPORTED = 2,   /* a layout, dtype or layer geometry this build has no kernel for          */
    DP_ERR_WORKSPACE = 3,     /* workspace missing or smaller than dp_workspace_bytes()                   */
    DP_ERR_DEVICE = 4         /* the HIP runtime refused a launch                                         */
} dp_status;

typedef enum { DP_DENSE = 0, DP_CONV2D = 1, DP_GN_AFFINE = 2 } dp_kind;
typedef enum { DP_F32 = 0, DP_BF16 = 1 } dp_dtype;
typedef enum { DP_NCHW = 0, DP_NHWC = 1 } dp_layout;   /* activations channels-first or channels-last */

/* One parameterised layer and the micro-batch it is evaluated on.
 * Layout DP_NCHW as written below; DP_NHWC: conv2d / gn_affine activations and output gradients are
 * x [n, h, w, cin], dy [n, oh, ow, cout] (parameter gradients keep their [cout, cin, kh, kw] order; a dense
 * layer is the same in both).  Channels-last inputs are transposed into the end of the workspace by a
 * pre-pass and the kernels read the copy: dp_workspace_bytes grows by the size of both tensors, the
 * results are bit for bit those of the channels-first call.
 *   dense     : x [n, h, cin], dy [n, h, cout]; h = tokens per example, w = 1
 *   conv2d    : x [n, cin, h, w], dy [n, cout, oh, ow], oh = (h + 2 pad - kh)/stride + 1;
 *               cross-correlation, zero padding, dilation 1, groups 1
 *   gn_affine : x [n, cin, h, w] is the input of the GroupNorm (before normalisation),
 *               dy [n, cin, h, w]; cout == cin; statistics per (example, group) over
 *               (cin/gn_groups)*h*w elements, biased variance, xhat = (x-mean)/sqrt(var+eps);
 *               the "weight" is the scale gamma, the "bias" the shift beta (always present). */
typedef struct dp_layer_desc {
    int kind;        /* dp_kind   */
    int in_dtype;    /* dp_dtype of x and dy */
    int layout;      /* dp_layout */
    int n;           /* examples in this micro-step, >= 1 */
    int cin, cout, h, w;
    int kh, kw, stride, pad;     /* conv2d only; ignored otherwise */
    int has_bias;                /* conv2d / dense */
    int gn_groups;               /* gn_affine only */
    float gn_eps;                /* gn_affine only */
} dp_layer_desc;

typedef void *dp_stream;   /* a hipStream_t */

/* Bounds for M = n_groups clipping groups (Section 3.5: every group is clipped to C / sqrt(M), so the
 * squared group norms add up to at most C^2; M = 1 is the single global bound of Section 2):
 *   group_clip[g] = clip_c / sqrt(n_groups),   *clip_total = sqrt(sum_g group_clip[g]^2)
 * clip_total, the bound on the whole clipped gradient, is what the noise of H5 is scaled by.
 * group_clip [host] n_groups floats, clip_total [host] one float, both written.  Pure host.
 * clip_c <= 0 or NaN, n_groups < 1, NULL outputs -> DP_ERR_INVALID_ARG.                        */
dp_status dp_group_clip_bounds(float clip_c, int n_groups, float *group_clip, float *clip_total);

/* Which call a workspace is sized for. */
typedef enum { DP_WS_PER_EXAMPLE_GRAD = 0, DP_WS_RECOMPUTE = 1 } dp_ws_use;

/* Number of weight / bias parameters of a layer (0 on a bad descriptor).  Pure host. */
size_t dp_weight_count(const dp_layer_desc *desc /*[host]*/);
size_t dp_bias_count(const dp_layer_desc *desc /*[host]*/);

/* Bytes of device workspace the given call needs for this descriptor (pure host; 0 on a
 * bad descriptor).  What it holds, depending on the layer: partial squared norms (one float
 * per example and output tile, or per slice-sum workgroup), the partial tiles of contractions
 * whose K (or example range) is cut into slices, and rewritten copies of the operands where a
 * kernel reads them in another layout (sampled positions of a strided 1x1 conv, parity-split
 * rows of a strided 3x3 conv, K-contiguous pre-scaled operands of the clip-weighted form);
 * DP_WS_RECOMPUTE of a GroupNorm layer: n*2*cin floats.  From a few KB to a few tens of MB.
 * Partial sums go through the workspace so that reductions run in a fixed order: the same
 * inputs give the same bits on every call.  The contents are scratch: nothing has to be
 * preserved between calls (except as dp_per_example_grad_partials documents).               */
size_t dp_workspace_bytes(const dp_layer_desc *desc /*[host]*/, int use /*dp_ws_use*/);

/* Name of the kernel variant that dp_per_example_grad (use = DP_WS_PER_EXAMPLE_GRAD) or
 * dp_clip_accumulate_recompute (use = DP_WS_RECOMPUTE) launches for this descriptor, e.g.
 * "conv_contract<bf16,128x128,per_example>"; "" on a bad descriptor.  With DP_VARIANT_SHARED or-ed
 * into `use`: the variant the layer runs as inside a batch call of several layers (tiling is chosen
 * differently when a launch is shared); layers with equal names then share one launch, at most 16
 * per launch, and so do all layers whose names begin with "conv3x3_rows<" (every row width, stride
 * and K slicing of that kernel runs in one launch inside a batch call).  Pure host; lets a profiler's
 * per-kernel rows be tied to layers.  The string is static.                                     */
#define DP_VARIANT_SHARED 2
#define DP_VARIANT_MATERIALISE 4   /* or-ed into DP_WS_PER_EXAMPLE_GRAD: the variant of a call that stores the gradients
                                      (g_w given); without it the norm-only call, which may take another route */
const char *dp_kernel_variant(const dp_layer_desc *desc /*[host]*/, int use /*dp_ws_use*/);

/* H1 (+ the layer's share of H2): per-example weight gradients of one layer
 * (Section 2: the gradient of each example's loss is formed on its own), from each example's input activation
 * and output gradient:
 *   conv   dW_i[co,ci,kh,kw] = sum_{oh,ow} dY_i[co,oh,ow] * Xpad_i[ci, oh*s+kh-p, ow*s+kw-p]
 *          db_i[co] = sum_{oh,ow} dY_i[co,oh,ow]
 *   dense  dW_i[o,k] = sum_t dY_i[t,o] * X_i[t,k];   db_i[o] = sum_t dY_i[t,o]
 *   gn     dgamma_i[c] = sum_{h,w} dY_i[c,h,w] * xhat_i[c,h,w];  dbeta_i[c] = sum dY_i[c,h,w]
 * x, dy      [device] inputs as described by desc.
 * g_w        [device] fp32, example i's weight gradient at g_w + i*stride_w, overwritten;
 *            NULL = do not materialise (norms only).
 * g_b        [device] fp32, example i's bias gradient at g_b + i*stride_b, overwritten; must be
 *            given exactly when g_w is given and the layer has a bias.
 * g_stride   elements between consecutive examples' rows in g_w and in g_b; 0 means packed
 *            (stride_w = dp_weight_count, stride_b = dp_bias_count).  A non-zero value lets
 *            all tensors of a model share one [n, P_total] matrix; it must be a multiple of 4
 *            and at least the tensor's size.
 * sqnorm     [device] [n] fp32, overwritten with ||dW_i||^2 + ||db_i||^2, reduced inside the
 *            contraction's epilogue (the gradients are not read back); may be NULL only if
 *            g_w is given.
 * ws         [device] workspace of at least dp_workspace_bytes(desc, DP_WS_PER_EXAMPLE_GRAD).  */
dp_status dp_per_example_grad(const dp_layer_desc *desc /*[host]*/, const void *x, const void *dy,
                              float *g_w, float *g_b, size_t g_stride, float *sqnorm,
                              void *ws, size_t ws_bytes, dp_stream stream);

/* dp_per_example_grad without a workspace argument and without any allocation: for callers that
 * cannot call hipMalloc or carry a workspace around (code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation).  The workspace is a device array built into the library,
 * dp_static_scratch_bytes() = 32 MiB per GPU, held from the first call on a GPU until the process ends.
 * Same kernels, same results (bit for bit) as dp_per_example_grad.  The stream's device must be the
 * current device.  A layer whose dp_workspace_bytes(desc, DP_WS_PER_EXAMPLE_GRAD) exceeds the built-in
 * size -> DP_ERR_WORKSPACE (nothing is launched).  Every call on one GPU shares that GPU's array:
 * calls that overlap in time on one GPU (different streams, different host threads) race; issue them
 * on one stream, or order them with events.  Nothing in the array has to start at zero or survive
 * between calls.  Calls no hipMalloc / hipFree or other allocating routine.                        */
size_t dp_static_scratch_bytes(void);
dp_status dp_per_example_grad_static(const dp_layer_desc *desc /*[host]*/, const void *x, const void *dy,
                                     float *g_w, float *g_b, size_t g_stride, float *sqnorm, dp_stream stream);

/* The same per-example call without the per-layer reduction: the partial squared norms of the layer
 * stay in the workspace, ws[0 .. n * count) as a row-major [n, count] float matrix with
 * count = dp_norm_partial_count(desc, g_w != NULL), until the workspace is used again.
 * dp_norms_from_partials then reduces the partials of all layers in one launch, so a model of L
 * layers needs L fewer small launches per micro-step than with dp_per_example_grad + dp_norms (H2,
 * same sums in a fixed order).  Arguments as dp_per_example_grad.                                 */
size_t dp_norm_partial_count(const dp_layer_desc *desc, int materialise);
dp_status dp_per_example_grad_partials(const dp_layer_desc *desc, const void *x, const void *dy, float *g_w, float *g_b,
                                       size_t g_stride, void *ws, size_t ws_bytes, dp_stream stream);

/* H1 and the per-layer part of H2 for SEVERAL layers in one call: for every layer l the result of
 * dp_per_example_grad(&descs[l], x[l], dy[l], g_w[l], g_b[l], g_stride, sqnorm[l], ws[l], ws_bytes[l])
 * (same definition, Section 2; the numbers may differ from the single-layer call in the last bits, since
 * sums may be split differently).  Layers that run the same kernel share ONE launch, so a launch has
 * enough workgroups to fill the chip even when a micro-step holds one example (the batch-size-one
 * regime of Section 2), and the per-layer reductions of all layers are one launch.  Fixed summation
 * order: the same inputs give the same bits on every call.
 * descs [host] n_layers descriptors, all with the same n.  x, dy, sqnorm, ws [host] arrays of n_layers
 * device pointers; g_w, g_b [host] arrays of device pointers or NULL (= no layer materialises), entry NULL
 * = that layer does not; sqnorm[l] [device] [n], overwritten; ws[l] at least dp_workspace_bytes(&descs[l],
 * DP_WS_PER_EXAMPLE_GRAD), one workspace per layer (they are in use at the same time).  Every argument of
 * every layer is validated before anything is launched.
 * sqnorm may be NULL: then the per-layer reduction is left to the caller, who collects the partial sums of
 * several batch calls (one per stream, say) and reduces them all in one dp_layer_norms_from_partials launch.
 * Layer l's partial squared norms stay at the start of its workspace, ws[l][0 .. n * partial_counts[l]) as a
 * row-major [n, partial_counts[l]] float matrix, until that workspace is used again.
 * partial_counts [host] n_layers ints, written by the call (the count depends on how the batch was planned),
 * or NULL when not wanted; required when sqnorm is NULL.                                               */
dp_status dp_per_example_grad_batch(const dp_layer_desc *descs, const void *const *x, const void *const *dy,
                                    float *const *g_w, float *const *g_b, size_t g_stride, float *const *sqnorm,
                                    void *const *ws, const size_t *ws_bytes, int32_t *partial_counts, int n_layers,
                                    dp_stream stream);

/* Per-layer part of H2 from partial sums: sqnorm[l][i] = sum_c partials[l][i * counts[l] + c], c in order, for
 * n_layers layers in one launch (64 layers per launch beyond that).  partials, sqnorm [host] arrays of n_layers
 * device pointers (4-byte aligned), counts [host] n_layers ints >= 1; sqnorm[l] [device] [n], overwritten.   */
dp_status dp_layer_norms_from_partials(const float *const *partials, const int32_t *counts, float *const *sqnorm,
                                       int n_layers, int n, dp_stream stream);

/* H4, recomputing form, for several layers in one call: for every layer l what
 * dp_clip_accumulate_recompute(&descs[l], x[l], dy[l], sqnorm[l], clip_c[l], acc_w[l], acc_b[l], ws[l], ws_bytes[l])
 * computes, with the layers that run the same kernel sharing one launch.  sqnorm[l] [device] [n]: squared norms
 * of layer l's clipping group; clip_c [host] n_layers bounds; acc_b may be NULL when no layer has a bias.  */
dp_status dp_clip_accumulate_recompute_batch(const dp_layer_desc *descs, const void *const *x, const void *const *dy,
                                             const float *const *sqnorm, const float *clip_c, float *const *acc_w,
                                             float *const *acc_b, void *const *ws, const size_t *ws_bytes, int n_layers,
                                             dp_stream stream);

/* H1 + H2 for CLIPPING UNITS of several examples (the micro-batching of the GPU baseline in the Abstract and
 * Table 1: the gradient of a micro-batch of clip_unit examples is clipped instead of each example's).  Unit u
 * holds the consecutive examples [u * clip_unit, (u + 1) * clip_unit); the call gives, per unit, the SUM of its
 * per-example gradients (definitions as in dp_per_example_grad; the contraction runs over the unit's examples as
 * well as its positions) and the squared norm of that sum:
 *   g_w / g_b  [device] unit u's sums at g_w + u * stride_w, g_b + u * stride_b (n / clip_unit rows), or NULL
 *   sqnorm     [device] [n / clip_unit], ||S_u||^2; may be NULL only if g_w is given
 * The rest of the path then treats a unit like an example.  With gbar_u = S_u / clip_unit the unit's mean,
 *   sum_u clip(gbar_u, C) = 1/clip_unit * sum_u clip(S_u, clip_unit * C),
 * so H3/H4 run on the sums with the bound clip_unit * C, H5 with clip_total = clip_unit * C and
 * total_batch = clip_unit * (number of units) = the number of examples: the result is
 * (N(0, sigma^2 C^2) + sum_u clip(gbar_u, C)) / (number of units).
 * desc->n must be a multiple of clip_unit (else DP_ERR_INVALID_ARG); clip_unit == 1 is dp_per_example_grad.
 * ws: at least dp_unit_workspace_bytes(desc, clip_unit) (0 on a bad descriptor / unit).  Other arguments and
 * errors as dp_per_example_grad.                                                                       */
size_t dp_unit_workspace_bytes(const dp_layer_desc *desc /*[host]*/, int clip_unit);
dp_status dp_unit_grad(const dp_layer_desc *desc /*[host]*/, int clip_unit, const void *x, const void *dy, float *g_w,
                       float *g_b, size_t g_stride, float *sqnorm, void *ws, size_t ws_bytes, dp_stream stream);

/* dp_unit_grad for several layers in one call (clip_unit >= 2): layers that run the same kernel share one launch,
 * and the per-layer reductions of all layers are one launch.  Arrays as in dp_per_example_grad_batch; g_w / g_b
 * rows and sqnorm[l] entries are units (n / clip_unit of them); ws[l] at least dp_unit_workspace_bytes.       */
dp_status dp_unit_grad_batch(const dp_layer_desc *descs, int clip_unit, const void *const *x, const void *const *dy,
                             float *const *g_w, float *const *g_b, size_t g_stride, float *const *sqnorm,
                             void *const *ws, const size_t *ws_bytes, int n_layers, dp_stream stream);

/* group_sqnorm[g, i] = sum over the layers l of group g, in order, of sum_c partials[l][i * counts[l] + c].
 * partials [host] array of n_layers device pointers (4-byte aligned); counts, group_of_layer [host]
 * arrays of n_layers ints; group_sqnorm [device] [n_groups, n], overwritten.                       */
dp_status dp_norms_from_partials(const float *const *partials, const int32_t *counts, const int32_t *group_of_layer,
                                 int n_layers, int n, int n_groups, float *group_sqnorm, dp_stream stream);

/* H2: per-example squared norms per clipping group (Section 2: one global norm;
 * Section 3.5: one norm per group):
 *   group_sqnorm[g, i] = sum over layers l with group_of_layer[l] == g of layer_sqnorm[l, i],
 * summed in a fixed order (the same bits on every call).
 * layer_sqnorm   [device] [n_layers, n] fp32
 * group_of_layer [device] [n_layers] int32, each in [0, n_groups) (not checked on the host;
 *                out-of-range entries are ignored by the kernel)
 * group_sqnorm   [device] [n_groups, n] fp32, overwritten                                    */
dp_status dp_norms(const float *layer_sqnorm, const int32_t *group_of_layer, int n_layers, int n,
                   int n_groups, float *group_sqnorm, dp_stream stream);

/* H3, for observability (H4 evaluates the same expression itself):
 *   f[i] = min(1, clip_c / sqrt(sqnorm[i])), and 1 where sqnorm[i] == 0 or clip_c = +inf.
 * sqnorm, f  [device] [n] fp32.  clip_c > 0 (may be +inf).                                   */
dp_status dp_clip_factors(const float *sqnorm, float clip_c, int n, float *f, dp_stream stream);

/* H4, materialised form: acc[e] += sum_{i<n} f_i * g[i, e]   (Section 2: the clipped
 * per-example gradients are summed over the whole batch; called once per micro-step it is
 * the gradient accumulation over micro-steps).
 * g        [device] fp32 per-example gradients, example i's p values at g + i*g_stride
 *          (g_stride = 0 means p; several tensors of one clipping group that sit side by
 *          side in a [n, P_total] matrix can be accumulated by one call)
 * sqnorm   [device] [n] fp32 squared norms of the clipping group this tensor belongs to
 * acc      [device] [p] fp32, read and written; the caller zeroes it when a step starts      */
dp_status dp_clip_accumulate(const float *g, size_t g_stride, const float *sqnorm, float clip_c, int n,
                             size_t p, float *acc, dp_stream stream);

/* H4, materialised form, for several clipping groups in one launch (Section 3.5: one bound per group
 * of tensors): the columns [0, p) of g are cut into n_seg segments; segment k covers columns
 * seg_begin[k] .. seg_begin[k+1] (the last one ends at p), belongs to clipping group seg_group[k] and is
 * clipped to seg_clip[k]:
 *     acc[e] += sum_{i<n} min(1, seg_clip[k] / sqrt(group_sqnorm[seg_group[k], i])) * g[i, e],  e in segment k.
 * Same sums, same order as one dp_clip_accumulate call per segment.
 * g, acc as above; group_sqnorm [device] [n_groups, n]; seg_begin, seg_group, seg_clip [host] arrays of
 * n_seg entries, boundaries increasing multiples of 4 starting at 0; p a multiple of 4.               */
dp_status dp_clip_accumulate_segments(const float *g, size_t g_stride, const float *group_sqnorm, int n_groups,
                                      const size_t *seg_begin, const int32_t *seg_group, const float *seg_clip, int n_seg,
                                      int n, size_t p, float *acc, dp_stream stream);

/* H4, recomputing form: the same sum without per-example gradients in memory,
 *   acc_w += sum_i f_i * dW_i,  acc_b += sum_i f_i * db_i,
 * evaluated as one contraction over (example, position) with dY_i scaled by f_i as it is
 * staged (for bf16 inputs the scaled value is rounded to bf16 once more).
 * acc_b may be NULL only when the layer has no bias.  ws as for DP_WS_RECOMPUTE.             */
dp_status dp_clip_accumulate_recompute(const dp_layer_desc *desc /*[host]*/, const void *x, const void *dy,
                                       const float *sqnorm, float clip_c, float *acc_w, float *acc_b,
                                       void *ws, size_t ws_bytes, dp_stream stream);

/* H5: out[e] = (acc[e] + sigma * clip_total * z_e) / total_batch  (Section 2, first equation),
 * z_e iid N(0,1) from Philox4x32-10: elements 4q..4q+3 come from the call with counter
 * (q mod 2^32, q div 2^32, tensor_id, step mod 2^32) and key (seed mod 2^32, seed div 2^32);
 * each 32-bit word r gives u = ((r >> 9) + 0.5) * 2^-23; (u0,u1) -> z0 = R cos(2 pi u1),
 * z1 = R sin(2 pi u1), R = sqrt(-2 ln u0); (u2,u3) -> z2, z3.  The result does not depend on
 * the launch geometry.  sigma == 0 evaluates no random numbers.  out may alias acc.
 * clip_total = sqrt(sum_g C_g^2), the bound on the whole clipped gradient.
 * acc, out  [device] [p] fp32.  sigma >= 0, clip_total > 0 (finite unless sigma == 0: an infinite
 * bound draws no noise), total_batch >= 1.                                                    */
dp_status dp_add_noise_finalize(const float *acc, float *out, size_t p, float sigma, float clip_total,
                                uint64_t total_batch, uint64_t seed, uint64_t step, uint32_t tensor_id,
                                dp_stream stream);

/* The per-example form of the noise (second equation of the Algorithm section, the form the paper's
 * implementation uses): every clipped example carries its own N(0, sigma^2 clip_total^2 / total_batch)
 * draw, so that after all total_batch examples the accumulated noise has the variance of the
 * once-per-step form.  Called once per micro-step and tensor, after the clipped sum:
 *     acc[e] += sigma * clip_total / sqrt(total_batch) * sum_{j = first_example}^{first_example + n_examples - 1} z(j, e)
 * with z(j, .) from Philox4x32-10 as above but counter (q, j, tensor_id, step mod 2^32) and key
 * (seed mod 2^32, (seed div 2^32) xor 0x50455245): j is the example's index within the optimiser step.
 * The step is then finished with dp_add_noise_finalize(sigma = 0).  Same distribution as the
 * once-per-step form, different bits, n_examples Philox calls per four parameters.
 * acc [device] [p] fp32, 16-byte aligned.  step_dev [device]: NULL, or one uint64 the kernel reads the
 * step from instead of `step` (see dp_add_noise_finalize_flat).  first_example + n_examples >
 * total_batch, n_examples < 1, bad sigma / clip_total -> DP_ERR_INVALID_ARG.                       */
dp_status dp_add_example_noise(float *acc, size_t p, float sigma, float clip_total, uint64_t total_batch, uint64_t seed,
                               uint64_t step, uint32_t tensor_id, uint64_t first_example, int n_examples,
                               const uint64_t *step_dev, dp_stream stream);

/* H5 fused with the SGD step that consumes it (the step right after the path: Section 2 names SGD
 * with a stepped learning-rate decay as the optimiser, Sections 3.2 and 3.3 run it with momentum
 * 0.9): with g[e] = (acc[e] + sigma * clip_total * z_e) / total_batch as above,
 *     velocity[e] = momentum * velocity[e] + g[e];   theta[e] -= lr * velocity[e]
 * or, with velocity == NULL (momentum must be 0),  theta[e] -= lr * g[e].
 * g is written to `out` only if out != NULL.  lr is this step's learning rate (decay and scaling
 * policies are the caller's).  acc, theta, velocity, out [device] [p] fp32, 16-byte aligned;
 * theta and velocity are updated in place.  Same stream contract and errors as
 * dp_add_noise_finalize; lr or momentum not finite, momentum < 0, momentum != 0 without a
 * velocity buffer -> DP_ERR_INVALID_ARG.                                                         */
dp_status dp_add_noise_finalize_update(const float *acc, float *theta, float *velocity, float *out, size_t p, float sigma,
                                       float clip_total, uint64_t total_batch, uint64_t seed, uint64_t step,
                                       uint32_t tensor_id, float lr, float momentum, dp_stream stream);

/* H5 (optionally with the fused SGD step) for every tensor of a flat parameter vector in ONE launch.
 * The vector acc (and out, theta, velocity, laid out alike) holds n_seg tensors; tensor k occupies the
 * elements seg_begin[k] .. seg_begin[k] + seg_size[k] and draws its noise exactly as
 * dp_add_noise_finalize(acc + seg_begin[k], ..., p = seg_size[k], tensor_id = seg_tensor_id[k]) would:
 * same counters, same bits.  Elements between tensors (padding) are neither read nor written.
 * seg_begin, seg_size, seg_tensor_id  [host] n_seg entries; every seg_begin a multiple of 4, tensors in
 *            increasing order without overlap, every seg_size in [1, 2^32).
 * step_dev   [device] NULL, or one uint64: then the kernel takes the step from this word instead of
 *            `step` -- a caller that replays a captured graph advances the word between replays, so
 *            that no two optimiser steps ever share a noise draw.
 * theta      [device] NULL = finalize only (out required).  Otherwise the SGD step of
 *            dp_add_noise_finalize_update is applied to theta / velocity with lr and momentum, and out
 *            may be NULL.
 * Errors as dp_add_noise_finalize / dp_add_noise_finalize_update.                                   */
dp_status dp_add_noise_finalize_flat(const float *acc, float *out, float *theta, float *velocity,
                                     const uint64_t *seg_begin, const uint64_t *seg_size, const uint32_t *seg_tensor_id,
                                     int n_seg, float sigma, float clip_total, uint64_t total_batch, uint64_t seed,
                                     uint64_t step, const uint64_t *step_dev, float lr, float momentum, dp_stream stream);

/* The raw 32-bit Philox word behind each element of the stream above (diagnostic; lets a
 * test compare the integer stream bit for bit).  raw [device] [p] uint32.                      */
dp_status dp_philox_raw(uint32_t *raw, size_t p, uint64_t seed, uint64_t step, uint32_t tensor_id,
                        dp_stream stream);

/* Timing aid for benchmarks (not part of the method): the NEXT contraction kernel this thread
 * launches through dp_per_example_grad or dp_clip_accumulate_recompute -- the kernel whose name
 * dp_kernel_variant reports, not the small packing / slice-sum / partial-sum kernels around it --
 * is bracketed by hipEventRecord(start, stream) and hipEventRecord(stop, stream) on the stream it
 * is launched on.  start / stop are hipEvent_t handles passed as void*; the request is consumed
 * by that launch; (NULL, NULL) cancels it.  Layers without a contraction (dense, GroupNorm)
 * leave it pending.  Always DP_OK.                                                              */
dp_status dp_profile_next_contraction(void *start, void *stop);

/* Sentence describing the last error on this thread ("" if none).  Never NULL. */
const char *dp_last_error(void);

/* "major.minor gfx950" */
const char *dp_version(void);

#ifdef __cplusplus
}
#endif
#endif
