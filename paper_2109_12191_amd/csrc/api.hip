// C ABI of libdp_privatise: argument validation (all on the host, before any launch) and
// dispatch to the kernels.  See include/dp_privatise.h for the contract of every call.
#include "internal.h"
#include "group.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#define DP_TRY_ST(expr) do { dp_status st__ = (expr); if (st__ != DP_OK) return st__; } while (0)

namespace dp {

static thread_local char g_err[512] = "";
static thread_local hipEvent_t g_prof_start = nullptr, g_prof_stop = nullptr;

void profile_begin(hipStream_t s)
{
    if (g_prof_start) (void)hipEventRecord(g_prof_start, s);
    g_prof_start = nullptr;
}

void profile_end(hipStream_t s)
{
    if (g_prof_stop) (void)hipEventRecord(g_prof_stop, s);
    g_prof_stop = nullptr;
}

dp_status fail(dp_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

dp_status check_launch(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DP_ERR_DEVICE, "%s: launch failed: %s", what, hipGetErrorString(e));
    return DP_OK;
}

// ---- grouped launches (group.h)
static thread_local LaunchQueue *g_queue = nullptr;
LaunchQueue *open_queue() { return g_queue; }
void set_open_queue(LaunchQueue *q) { g_queue = q; }
int crowd_hint() { return g_queue ? g_queue->crowd : 0; }
int fuse_hint() { return g_queue ? g_queue->fuse : 0; }

dp_status flush_queue(LaunchQueue &q)
{
    set_open_queue(nullptr);                         // from here on everything is launched at once
    std::vector<char> args;
    std::vector<unsigned> blocks;
    for (int tier = 0; tier < TIER_COUNT; ++tier) {
        std::vector<LaunchQueue::Item> &held = q.tier[tier];
        std::vector<char> done(held.size(), 0);
        for (size_t i = 0; i < held.size(); ++i) {
            if (done[i]) continue;
            const LaunchQueue::Item &first = held[i];
            // every held launch of the same kernel, in the order they were submitted, GROUP_MAX per launch
            args.clear(); blocks.clear();
            auto fire = [&]() -> dp_status {
                if (blocks.empty()) return DP_OK;
                if (tier == TIER_MAIN) profile_begin(q.stream);
                const dp_status st = first.go(first.fn, args.data(), blocks.data(), (int)blocks.size(), first.threads, first.lds, q.stream);
                if (tier == TIER_MAIN) profile_end(q.stream);
                args.clear(); blocks.clear();
                return st != DP_OK ? st : check_launch(first.what);
            };
            for (size_t j = i; j < held.size(); ++j) {
                const LaunchQueue::Item &it = held[j];
                if (done[j] || it.fn != first.fn || it.lds != first.lds || it.threads != first.threads) continue;
                done[j] = 1;
                args.insert(args.end(), it.args.begin(), it.args.end());
                blocks.push_back(it.blocks);
                if ((int)blocks.size() == GROUP_MAX) DP_TRY_ST(fire());
            }
            DP_TRY_ST(fire());
        }
        held.clear();
    }
    for (auto &fn : q.post) DP_TRY_ST(fn());
    q.post.clear();
    return DP_OK;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Validate a descriptor and derive its geometry.  Limits keep every index in 32 bits inside
// the kernels: per-example tensors below 2^31 elements.
static dp_status make_geo(const dp_layer_desc *d, Geo &g)
{
    if (!d) return fail(DP_ERR_INVALID_ARG, "descriptor is NULL");
    if (d->kind != DP_DENSE && d->kind != DP_CONV2D && d->kind != DP_GN_AFFINE)
        return fail(DP_ERR_INVALID_ARG, "unknown layer kind %d", d->kind);
    if (d->in_dtype != DP_F32 && d->in_dtype != DP_BF16)
        return fail(DP_ERR_INVALID_ARG, "unknown input dtype %d", d->in_dtype);
    if (d->layout != DP_NCHW && d->layout != DP_NHWC) return fail(DP_ERR_INVALID_ARG, "unknown layout %d", d->layout);
    if (d->n < 1) return fail(DP_ERR_INVALID_ARG, "n = %d examples (need >= 1)", d->n);
    if (d->cin < 1 || d->cout < 1 || d->h < 1 || d->w < 1)
        return fail(DP_ERR_INVALID_ARG, "non-positive dimension (cin %d cout %d h %d w %d)", d->cin, d->cout, d->h, d->w);
    memset(&g, 0, sizeof(g));
    g.kind = d->kind; g.bf16 = d->in_dtype == DP_BF16; g.n = d->n;
    g.nhwc = (d->layout == DP_NHWC && d->kind != DP_DENSE) ? 1 : 0;       // a dense layer's [n, tokens, features] is the same in both
    g.cin = d->cin; g.cout = d->cout; g.h = d->h; g.w = d->w;
    g.kh = g.kw = 1; g.stride = 1; g.pad = 0; g.oh = d->h; g.ow = d->w;
    g.has_bias = d->has_bias ? 1 : 0;
    if (d->kind == DP_CONV2D) {
        if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0)
            return fail(DP_ERR_INVALID_ARG, "bad conv geometry (kh %d kw %d stride %d pad %d)", d->kh, d->kw, d->stride, d->pad);
        if (d->h + 2 * d->pad < d->kh || d->w + 2 * d->pad < d->kw)
            return fail(DP_ERR_INVALID_ARG, "kernel %dx%d larger than padded input %dx%d", d->kh, d->kw, d->h + 2 * d->pad, d->w + 2 * d->pad);
        if (d->kh > 255 || d->kw > 255 || d->pad > 255 || d->h > 16384 || d->w > 16384)
            return fail(DP_ERR_UNSUPPORTED, "conv geometry beyond kernel limits (k, pad <= 255; h, w <= 16384)");
        g.kh = d->kh; g.kw = d->kw; g.stride = d->stride; g.pad = d->pad;
        g.oh = (d->h + 2 * d->pad - d->kh) / d->stride + 1;
        g.ow = (d->w + 2 * d->pad - d->kw) / d->stride + 1;
        g.pw = (size_t)d->cout * d->cin * d->kh * d->kw;
        g.pb = g.has_bias ? (size_t)d->cout : 0;
        g.x_elems = (size_t)d->cin * d->h * d->w;
        g.dy_elems = (size_t)d->cout * g.oh * g.ow;
    } else if (d->kind == DP_DENSE) {
        if (d->w != 1) return fail(DP_ERR_INVALID_ARG, "dense layer: w must be 1 (h = tokens), got %d", d->w);
        g.pw = (size_t)d->cout * d->cin;
        g.pb = g.has_bias ? (size_t)d->cout : 0;
        g.x_elems = (size_t)d->h * d->cin;
        g.dy_elems = (size_t)d->h * d->cout;
    } else {
        if (d->cout != d->cin) return fail(DP_ERR_INVALID_ARG, "GroupNorm: cout (%d) must equal cin (%d)", d->cout, d->cin);
        if (d->gn_groups < 1 || d->cin % d->gn_groups != 0)
            return fail(DP_ERR_INVALID_ARG, "GroupNorm: %d groups do not divide %d channels", d->gn_groups, d->cin);
        if (!(d->gn_eps >= 0.0f) || !std::isfinite(d->gn_eps))
            return fail(DP_ERR_INVALID_ARG, "GroupNorm: eps must be finite and >= 0");
        g.gn_groups = d->gn_groups; g.gn_eps = d->gn_eps; g.has_bias = 1;
        g.pw = (size_t)d->cin; g.pb = (size_t)d->cin;
        g.x_elems = g.dy_elems = (size_t)d->cin * d->h * d->w;
    }
    const size_t lim = (size_t)1 << 31;
    if (g.x_elems >= lim || g.dy_elems >= lim || g.pw >= lim)
        return fail(DP_ERR_UNSUPPORTED, "per-example tensor of 2^31 elements or more");
    if ((size_t)d->n > 65535 && d->kind != DP_CONV2D)
        return fail(DP_ERR_UNSUPPORTED, "more than 65535 examples per call for dense / GroupNorm layers");
    return DP_OK;
}

// Channels-last inputs are transposed into the end of the workspace before anything else reads them.
static size_t align16_api(size_t b) { return (b + 15) & ~(size_t)15; }
static size_t layout_copy_bytes(const Geo &g)
{
    if (!g.nhwc) return 0;
    const size_t es = g.bf16 ? 2 : 4;
    return align16_api((size_t)g.n * g.x_elems * es) + align16_api((size_t)g.n * g.dy_elems * es);
}

static size_t ws_kernels_for(const Geo &g, int mode)
{
    size_t b;
    if (g.kind == DP_CONV2D) b = conv_ws_bytes(g, mode);
    else if (g.kind == DP_DENSE) b = dense_ws_bytes(g, mode);
    else b = gn_ws_bytes(g, mode);
    return align16_api(b);
}

static size_t ws_bytes_for(const Geo &g, int mode) { return ws_kernels_for(g, mode) + layout_copy_bytes(g); }

// x, dy as the kernels read them: the caller's tensors, or their channels-first copies behind the first
// `kernels_bytes` bytes of the workspace
static dp_status channels_first_inputs(const Geo &g, size_t kernels_bytes, const void *&x, const void *&dy, void *ws, hipStream_t s)
{
    if (!g.nhwc) return DP_OK;
    const int es = g.bf16 ? 2 : 4;
    char *xt = static_cast<char *>(ws) + kernels_bytes;
    char *dyt = xt + align16_api((size_t)g.n * g.x_elems * es);
    dp_status st = launch_to_channels_first(x, xt, g.n, g.h * g.w, g.cin, es, s);
    if (st != DP_OK) return st;
    st = launch_to_channels_first(dy, dyt, g.n, g.oh * g.ow, g.cout, es, s);
    x = xt;
    dy = dyt;
    return st;
}

// One layer's kernels for a per-example call (mode NORM / MATERIALISE) or the recomputing clipped sum (WEIGHTED)
static dp_status launch_layer(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                              size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c, void *ws,
                              hipStream_t s)
{
    DP_TRY_ST(channels_first_inputs(g, ws_kernels_for(g, mode == MODE_WEIGHTED ? MODE_WEIGHTED : MODE_NORM), x, dy, ws, s));
    if (g.kind == DP_CONV2D) return launch_conv(g, mode, x, dy, out_w, out_b, out_stride, sqnorm, group_sqnorm, clip_c, ws, s);
    if (g.kind == DP_DENSE) return launch_dense(g, mode, x, dy, out_w, out_b, out_stride, sqnorm, group_sqnorm, clip_c, ws, s);
    return launch_gn(g, mode, x, dy, out_w, out_b, out_stride, sqnorm, group_sqnorm, clip_c, ws, s);
}

// Tensors that are read or written with 16-byte accesses need 16-byte alignment; the small
// per-example vectors (norms, factors, group ids, raw words) are accessed word by word.
static dp_status check_ptr(const void *p, const char *name, bool required, unsigned align = 16)
{
    if (!p) return required ? fail(DP_ERR_INVALID_ARG, "%s is NULL", name) : DP_OK;
    if (reinterpret_cast<uintptr_t>(p) & (align - 1))
        return fail(DP_ERR_INVALID_ARG, "%s is not %u-byte aligned", name, align);
    return DP_OK;
}

static dp_status check_clip(float clip_c)
{
    if (std::isnan(clip_c) || !(clip_c > 0.0f)) return fail(DP_ERR_INVALID_ARG, "clip_c must be > 0 (may be +inf)");
    return DP_OK;
}

static dp_status check_ws(const Geo &g, int mode, const void *ws, size_t ws_bytes)
{
    const size_t need = ws_bytes_for(g, mode);
    if (need == 0) return DP_OK;
    if (!ws) return fail(DP_ERR_WORKSPACE, "workspace is NULL; %zu bytes needed", need);
    if (!aligned16(ws)) return fail(DP_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
    if (ws_bytes < need) return fail(DP_ERR_WORKSPACE, "workspace of %zu bytes is smaller than the %zu needed", ws_bytes, need);
    return DP_OK;
}

}  // namespace dp

using namespace dp;

#define DP_TRY(expr) do { dp_status st__ = (expr); if (st__ != DP_OK) return st__; } while (0)

extern "C" {

const char *dp_last_error(void) { return g_err; }

dp_status dp_profile_next_contraction(void *start, void *stop)
{
    dp::g_prof_start = static_cast<hipEvent_t>(start);
    dp::g_prof_stop = static_cast<hipEvent_t>(stop);
    return DP_OK;
}
const char *dp_version(void) { return "0.2 gfx950"; }

dp_status dp_group_clip_bounds(float clip_c, int n_groups, float *group_clip, float *clip_total)
{
    DP_TRY(check_clip(clip_c));
    if (n_groups < 1) return fail(DP_ERR_INVALID_ARG, "n_groups = %d (need >= 1)", n_groups);
    if (!group_clip || !clip_total) return fail(DP_ERR_INVALID_ARG, "group_clip and clip_total must be non-NULL");
    const double each = (double)clip_c / std::sqrt((double)n_groups);
    double sum = 0.0;
    for (int g = 0; g < n_groups; ++g) {
        group_clip[g] = (float)each;
        sum += (double)group_clip[g] * (double)group_clip[g];
    }
    *clip_total = (float)std::sqrt(sum);
    g_err[0] = 0;
    return DP_OK;
}

size_t dp_weight_count(const dp_layer_desc *desc)
{
    Geo g;
    return make_geo(desc, g) == DP_OK ? g.pw : 0;
}

size_t dp_bias_count(const dp_layer_desc *desc)
{
    Geo g;
    return make_geo(desc, g) == DP_OK ? g.pb : 0;
}

size_t dp_workspace_bytes(const dp_layer_desc *desc, int use)
{
    Geo g;
    if (make_geo(desc, g) != DP_OK) return 0;
    if (use != DP_WS_PER_EXAMPLE_GRAD && use != DP_WS_RECOMPUTE) {
        fail(DP_ERR_INVALID_ARG, "unknown workspace use %d", use);
        return 0;
    }
    return ws_bytes_for(g, use == DP_WS_RECOMPUTE ? MODE_WEIGHTED : MODE_NORM);
}

const char *dp_kernel_variant(const dp_layer_desc *desc, int use)
{
    Geo g;
    if (make_geo(desc, g) != DP_OK) return "";
    const bool shared = (use & DP_VARIANT_SHARED) != 0, stored = (use & DP_VARIANT_MATERIALISE) != 0;
    use &= ~(DP_VARIANT_SHARED | DP_VARIANT_MATERIALISE);
    const int mode = use == DP_WS_RECOMPUTE ? MODE_WEIGHTED : (stored ? MODE_MATERIALISE : MODE_NORM);
    if (g.kind == DP_CONV2D) return conv_variant_name(g, mode, shared);
    if (g.kind == DP_DENSE) return g.bf16 ? "dense<bf16>" : "dense<f32>";
    return g.bf16 ? "gn_affine<bf16>" : "gn_affine<f32>";
}

dp_status dp_per_example_grad(const dp_layer_desc *desc, const void *x, const void *dy, float *g_w, float *g_b,
                              size_t g_stride, float *sqnorm, void *ws, size_t ws_bytes, dp_stream stream)
{
    Geo g;
    DP_TRY(make_geo(desc, g));
    DP_TRY(check_ptr(x, "x", true));
    DP_TRY(check_ptr(dy, "dy", true));
    DP_TRY(check_ptr(g_w, "g_w", false));
    DP_TRY(check_ptr(g_b, "g_b", false));
    DP_TRY(check_ptr(sqnorm, "sqnorm", false, 4));
    if (!g_w && !sqnorm) return fail(DP_ERR_INVALID_ARG, "nothing to compute: g_w and sqnorm are both NULL");
    if (g_w && g.pb && !g_b) return fail(DP_ERR_INVALID_ARG, "g_w given but g_b is NULL for a layer with a bias");
    if (!g_w && g_b) return fail(DP_ERR_INVALID_ARG, "g_b given without g_w");
    if (g_stride) {
        if (g_stride % 4) return fail(DP_ERR_INVALID_ARG, "g_stride must be a multiple of 4");
        if (g_stride < g.pw || g_stride < g.pb) return fail(DP_ERR_INVALID_ARG, "g_stride smaller than the tensor");
    }
    DP_TRY(check_ws(g, MODE_NORM, ws, ws_bytes));
    const int mode = g_w ? MODE_MATERIALISE : MODE_NORM;
    hipStream_t s = static_cast<hipStream_t>(stream);
    g_err[0] = 0;
    return launch_layer(g, mode, x, dy, g_w, g_b, g_stride, sqnorm, nullptr, 0.0f, ws, s);
}

static size_t norm_partial_count_for(const Geo &g, int mode)
{
    if (g.kind == DP_CONV2D) return conv_norm_partial_count(g, mode);
    if (g.kind == DP_DENSE) return dense_norm_partial_count(g, mode);
    return gn_norm_partial_count(g);
}

size_t dp_norm_partial_count(const dp_layer_desc *desc, int materialise)
{
    Geo g;
    if (make_geo(desc, g) != DP_OK) return 0;
    return norm_partial_count_for(g, materialise ? MODE_MATERIALISE : MODE_NORM);
}

dp_status dp_per_example_grad_partials(const dp_layer_desc *desc, const void *x, const void *dy, float *g_w, float *g_b,
                                       size_t g_stride, void *ws, size_t ws_bytes, dp_stream stream)
{
    Geo g;
    DP_TRY(make_geo(desc, g));
    DP_TRY(check_ptr(x, "x", true));
    DP_TRY(check_ptr(dy, "dy", true));
    DP_TRY(check_ptr(g_w, "g_w", false));
    DP_TRY(check_ptr(g_b, "g_b", false));
    if (g_w && g.pb && !g_b) return fail(DP_ERR_INVALID_ARG, "g_w given but g_b is NULL for a layer with a bias");
    if (!g_w && g_b) return fail(DP_ERR_INVALID_ARG, "g_b given without g_w");
    if (g_stride) {
        if (g_stride % 4) return fail(DP_ERR_INVALID_ARG, "g_stride must be a multiple of 4");
        if (g_stride < g.pw || g_stride < g.pb) return fail(DP_ERR_INVALID_ARG, "g_stride smaller than the tensor");
    }
    DP_TRY(check_ws(g, MODE_NORM, ws, ws_bytes));
    const int mode = g_w ? MODE_MATERIALISE : MODE_NORM;
    hipStream_t s = static_cast<hipStream_t>(stream);
    g_err[0] = 0;
    // sqnorm == nullptr: the kernels leave their partial sums at the start of the workspace
    return launch_layer(g, mode, x, dy, g_w, g_b, g_stride, nullptr, nullptr, 0.0f, ws, s);
}

// ---- clipping units of several examples ----------------------------------------------------

// Geometry of a call with clipping units.  A dense layer's unit sum is the per-example gradient of one
// example that holds the tokens of the whole unit ([n, t, k] read as [n / unit, unit * t, k]).
static dp_status unit_geo(const dp_layer_desc *desc, int clip_unit, Geo &g)
{
    DP_TRY(make_geo(desc, g));
    if (clip_unit < 1) return fail(DP_ERR_INVALID_ARG, "clip_unit = %d (need >= 1)", clip_unit);
    if (g.n % clip_unit) return fail(DP_ERR_INVALID_ARG, "n = %d is not a multiple of clip_unit = %d", g.n, clip_unit);
    if (g.kind == DP_DENSE) {
        if ((long long)desc->h * clip_unit > 0x7FFFFFFFll) return fail(DP_ERR_UNSUPPORTED, "dense layer: unit * tokens too large");
        dp_layer_desc d2 = *desc;
        d2.n = desc->n / clip_unit;
        d2.h = desc->h * clip_unit;
        DP_TRY(make_geo(&d2, g));
    }
    return DP_OK;
}

static size_t unit_ws_kernels(const Geo &g, int kind, int clip_unit)
{
    if (kind == DP_DENSE) return align16_api(dense_ws_bytes(g, MODE_NORM));          // g is already the reshaped layer
    if (kind == DP_CONV2D) return align16_api(conv_unit_ws_bytes(g, clip_unit));
    return align16_api(gn_unit_ws_bytes(g, clip_unit));
}
static size_t unit_ws_need(const Geo &g, int kind, int clip_unit) { return unit_ws_kernels(g, kind, clip_unit) + layout_copy_bytes(g); }

static dp_status launch_layer_units(const Geo &g, int clip_unit, const void *x, const void *dy, float *g_w, float *g_b,
                                    size_t g_stride, float *sqnorm, void *ws, hipStream_t s)
{
    DP_TRY_ST(channels_first_inputs(g, unit_ws_kernels(g, g.kind, clip_unit), x, dy, ws, s));
    if (g.kind == DP_DENSE)
        return launch_dense(g, g_w ? MODE_MATERIALISE : MODE_NORM, x, dy, g_w, g_b, g_stride, sqnorm, nullptr, 0.0f, ws, s);
    if (g.kind == DP_CONV2D) return launch_conv_units(g, clip_unit, x, dy, g_w, g_b, g_stride, sqnorm, ws, s);
    return launch_gn_units(g, clip_unit, x, dy, g_w, g_b, g_stride, sqnorm, ws, s);
}

size_t dp_unit_workspace_bytes(const dp_layer_desc *desc, int clip_unit)
{
    Geo g;
    if (unit_geo(desc, clip_unit, g) != DP_OK) return 0;
    if (clip_unit == 1) return dp_workspace_bytes(desc, DP_WS_PER_EXAMPLE_GRAD);
    return unit_ws_need(g, desc->kind, clip_unit);
}

dp_status dp_unit_grad(const dp_layer_desc *desc, int clip_unit, const void *x, const void *dy, float *g_w,
                                  float *g_b, size_t g_stride, float *sqnorm, void *ws, size_t ws_bytes, dp_stream stream)
{
    Geo g;
    DP_TRY(unit_geo(desc, clip_unit, g));
    if (clip_unit == 1) return dp_per_example_grad(desc, x, dy, g_w, g_b, g_stride, sqnorm, ws, ws_bytes, stream);
    DP_TRY(check_ptr(x, "x", true));
    DP_TRY(check_ptr(dy, "dy", true));
    DP_TRY(check_ptr(g_w, "g_w", false));
    DP_TRY(check_ptr(g_b, "g_b", false));
    DP_TRY(check_ptr(sqnorm, "sqnorm", g_w == nullptr, 4));
    if (g_w && g.pb && !g_b) return fail(DP_ERR_INVALID_ARG, "g_w given but g_b is NULL for a layer with a bias");
    if (!g_w && g_b) return fail(DP_ERR_INVALID_ARG, "g_b given without g_w");
    if (g_stride) {
        if (g_stride % 4) return fail(DP_ERR_INVALID_ARG, "g_stride must be a multiple of 4");
        if (g_stride < g.pw || g_stride < g.pb) return fail(DP_ERR_INVALID_ARG, "g_stride smaller than the tensor");
    }
    const size_t need = unit_ws_need(g, desc->kind, clip_unit);
    if (need && (!ws || ws_bytes < need))
        return fail(DP_ERR_WORKSPACE, "workspace of %zu bytes needed (dp_unit_workspace_bytes), %zu given", need, ws ? ws_bytes : (size_t)0);
    if (need && !aligned16(ws)) return fail(DP_ERR_INVALID_ARG, "workspace is not 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    g_err[0] = 0;
    return launch_layer_units(g, clip_unit, x, dy, g_w, g_b, g_stride, sqnorm, ws, s);
}

// Work per workgroup a batch call plans for, in units of one 128x128x64 chunk: the convolutions' multiply-adds
// spread over about three rounds of workgroups on 256 compute units, but neither so little that a workgroup's
// start-up dominates nor so much that one workgroup becomes the critical path.
static int batch_target(const std::vector<Geo> &geo)
{
    if (geo.size() < 2) return 0;
    double macs = 0.0;
    for (const Geo &g : geo)
        if (g.kind == DP_CONV2D) macs += (double)g.n * g.cout * g.cin * g.kh * g.kw * g.oh * g.ow;
    const double per_wg = macs / (128.0 * 128.0 * 64.0) / 768.0;
    return per_wg < 4.0 ? 4 : (per_wg > 64.0 ? 64 : (int)per_wg);
}

dp_status dp_per_example_grad_batch(const dp_layer_desc *descs, const void *const *x, const void *const *dy,
                                    float *const *g_w, float *const *g_b, size_t g_stride, float *const *sqnorm,
                                    void *const *ws, const size_t *ws_bytes, int32_t *partial_counts, int n_layers,
                                    dp_stream stream)
{
    if (!descs || !x || !dy || !ws || !ws_bytes)
        return fail(DP_ERR_INVALID_ARG, "descs, x, dy, ws and ws_bytes must be non-NULL host arrays");
    if (!sqnorm && !partial_counts)
        return fail(DP_ERR_INVALID_ARG, "sqnorm is NULL (reduction left to the caller) but partial_counts is NULL too");
    if (n_layers < 1) return fail(DP_ERR_INVALID_ARG, "n_layers = %d (need >= 1)", n_layers);
    std::vector<Geo> geo((size_t)n_layers);
    for (int l = 0; l < n_layers; ++l) {             // everything is validated before anything is launched
        Geo &g = geo[(size_t)l];
        DP_TRY(make_geo(&descs[l], g));
        if (g.n != geo[0].n) return fail(DP_ERR_INVALID_ARG, "layer %d: n = %d differs from layer 0's %d", l, g.n, geo[0].n);
        DP_TRY(check_ptr(x[l], "x[l]", true));
        DP_TRY(check_ptr(dy[l], "dy[l]", true));
        float *gw = g_w ? g_w[l] : nullptr, *gb = g_b ? g_b[l] : nullptr;
        DP_TRY(check_ptr(gw, "g_w[l]", false));
        DP_TRY(check_ptr(gb, "g_b[l]", false));
        if (sqnorm) DP_TRY(check_ptr(sqnorm[l], "sqnorm[l]", true, 4));
        if (gw && g.pb && !gb) return fail(DP_ERR_INVALID_ARG, "layer %d: g_w given but g_b is NULL for a layer with a bias", l);
        if (!gw && gb) return fail(DP_ERR_INVALID_ARG, "layer %d: g_b given without g_w", l);
        if (g_stride) {
            if (g_stride % 4) return fail(DP_ERR_INVALID_ARG, "g_stride must be a multiple of 4");
            if (gw && (g_stride < g.pw || g_stride < g.pb)) return fail(DP_ERR_INVALID_ARG, "layer %d: g_stride smaller than the tensor", l);
        }
        DP_TRY(check_ws(g, MODE_NORM, ws[l], ws_bytes[l]));
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    g_err[0] = 0;
    LaunchQueue q;
    q.stream = s;
    q.crowd = batch_target(geo);
    q.fuse = geo[0].n <= 2 ? 2 : 1;
    set_open_queue(&q);
    std::vector<const float *> parts((size_t)n_layers);
    std::vector<int32_t> counts((size_t)n_layers);
    dp_status st = DP_OK;
    for (int l = 0; l < n_layers && st == DP_OK; ++l) {
        const Geo &g = geo[(size_t)l];
        float *gw = g_w ? g_w[l] : nullptr, *gb = g_b ? g_b[l] : nullptr;
        const int mode = gw ? MODE_MATERIALISE : MODE_NORM;
        // sqnorm == nullptr: the kernels leave their partial sums at the start of the workspace
        st = launch_layer(g, mode, x[l], dy[l], gw, gb, g_stride, nullptr, nullptr, 0.0f, ws[l], s);
        parts[(size_t)l] = static_cast<const float *>(ws[l]);
        counts[(size_t)l] = (int32_t)norm_partial_count_for(g, mode);       // the plan in force inside this batch
    }
    if (st == DP_OK) st = flush_queue(q);
    set_open_queue(nullptr);
    if (st != DP_OK) return st;
    if (partial_counts)
        for (int l = 0; l < n_layers; ++l) partial_counts[l] = counts[(size_t)l];
    if (!sqnorm) return DP_OK;
    return launch_layer_norms(parts.data(), counts.data(), sqnorm, n_layers, geo[0].n, s);
}

dp_status dp_unit_grad_batch(const dp_layer_desc *descs, int clip_unit, const void *const *x, const void *const *dy,
                             float *const *g_w, float *const *g_b, size_t g_stride, float *const *sqnorm,
                             void *const *ws, const size_t *ws_bytes, int n_layers, dp_stream stream)
{
    if (!descs || !x || !dy || !sqnorm || !ws || !ws_bytes)
        return fail(DP_ERR_INVALID_ARG, "descs, x, dy, sqnorm, ws and ws_bytes must be non-NULL host arrays");
    if (n_layers < 1) return fail(DP_ERR_INVALID_ARG, "n_layers = %d (need >= 1)", n_layers);
    if (clip_unit < 2) return fail(DP_ERR_INVALID_ARG, "clip_unit = %d (need >= 2; units of one example: dp_per_example_grad_batch)", clip_unit);
    std::vector<Geo> geo((size_t)n_layers);
    for (int l = 0; l < n_layers; ++l) {             // everything is validated before anything is launched
        Geo &g = geo[(size_t)l];
        DP_TRY(unit_geo(&descs[l], clip_unit, g));
        if (descs[l].n != descs[0].n) return fail(DP_ERR_INVALID_ARG, "layer %d: n = %d differs from layer 0's %d", l, descs[l].n, descs[0].n);
        DP_TRY(check_ptr(x[l], "x[l]", true));
        DP_TRY(check_ptr(dy[l], "dy[l]", true));
        float *gw = g_w ? g_w[l] : nullptr, *gb = g_b ? g_b[l] : nullptr;
        DP_TRY(check_ptr(gw, "g_w[l]", false));
        DP_TRY(check_ptr(gb, "g_b[l]", false));
        DP_TRY(check_ptr(sqnorm[l], "sqnorm[l]", true, 4));
        if (gw && g.pb && !gb) return fail(DP_ERR_INVALID_ARG, "layer %d: g_w given but g_b is NULL for a layer with a bias", l);
        if (!gw && gb) return fail(DP_ERR_INVALID_ARG, "layer %d: g_b given without g_w", l);
        if (g_stride) {
            if (g_stride % 4) return fail(DP_ERR_INVALID_ARG, "g_stride must be a multiple of 4");
            if (gw && (g_stride < g.pw || g_stride < g.pb)) return fail(DP_ERR_INVALID_ARG, "layer %d: g_stride smaller than the tensor", l);
        }
        const size_t need = unit_ws_need(g, descs[l].kind, clip_unit);
        if (need && (!ws[l] || ws_bytes[l] < need))
            return fail(DP_ERR_WORKSPACE, "layer %d: workspace of %zu bytes needed (dp_unit_workspace_bytes), %zu given", l, need,
                        ws[l] ? ws_bytes[l] : (size_t)0);
        if (need && !aligned16(ws[l])) return fail(DP_ERR_INVALID_ARG, "layer %d: workspace is not 16-byte aligned", l);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    g_err[0] = 0;
    const int units = descs[0].n / clip_unit;
    LaunchQueue q;
    q.stream = s;
    q.crowd = batch_target(geo);
    q.fuse = geo[0].n <= 2 ? 2 : 1;
    set_open_queue(&q);
    std::vector<const float *> parts((size_t)n_layers);
    std::vector<int32_t> counts((size_t)n_layers);
    dp_status st = DP_OK;
    for (int l = 0; l < n_layers && st == DP_OK; ++l) {
        const Geo &g = geo[(size_t)l];
        float *gw = g_w ? g_w[l] : nullptr, *gb = g_b ? g_b[l] : nullptr;
        const int mode = gw ? MODE_MATERIALISE : MODE_NORM;
        parts[(size_t)l] = static_cast<const float *>(ws[l]);
        // sqnorm == nullptr: the partial sums stay in the workspace for the one reduction launch below
        if (g.kind == DP_CONV2D) {
            counts[(size_t)l] = (int32_t)conv_unit_norm_partial_count(g, clip_unit);     // the plan in force inside this batch
            st = launch_layer_units(g, clip_unit, x[l], dy[l], gw, gb, g_stride, nullptr, ws[l], s);
        } else if (g.kind == DP_DENSE) {
            counts[(size_t)l] = (int32_t)dense_norm_partial_count(g, mode);
            st = launch_layer_units(g, clip_unit, x[l], dy[l], gw, gb, g_stride, nullptr, ws[l], s);
        } else {
            counts[(size_t)l] = (int32_t)gn_unit_norm_partial_count(g);
            parts[(size_t)l] = gn_unit_partials(g, ws[l]);
            st = launch_layer_units(g, clip_unit, x[l], dy[l], gw, gb, g_stride, nullptr, ws[l], s);
        }
    }
    if (st == DP_OK) st = flush_queue(q);
    set_open_queue(nullptr);
    if (st != DP_OK) return st;
    return launch_layer_norms(parts.data(), counts.data(), sqnorm, n_layers, units, s);
}

dp_status dp_layer_norms_from_partials(const float *const *partials, const int32_t *counts, float *const *sqnorm,
                                       int n_layers, int n, dp_stream stream)
{
    if (!partials || !counts || !sqnorm)
        return fail(DP_ERR_INVALID_ARG, "partials, counts and sqnorm must be non-NULL host arrays");
    if (n_layers < 1 || n < 1) return fail(DP_ERR_INVALID_ARG, "n_layers (%d) and n (%d) must be >= 1", n_layers, n);
    for (int l = 0; l < n_layers; ++l) {
        if (!partials[l] || (reinterpret_cast<uintptr_t>(partials[l]) & 3u))
            return fail(DP_ERR_INVALID_ARG, "partials[%d] is NULL or not 4-byte aligned", l);
        if (!sqnorm[l] || (reinterpret_cast<uintptr_t>(sqnorm[l]) & 3u))
            return fail(DP_ERR_INVALID_ARG, "sqnorm[%d] is NULL or not 4-byte aligned", l);
        if (counts[l] < 1) return fail(DP_ERR_INVALID_ARG, "counts[%d] = %d (need >= 1)", l, counts[l]);
    }
    g_err[0] = 0;
    return launch_layer_norms(partials, counts, sqnorm, n_layers, n, static_cast<hipStream_t>(stream));
}

dp_status dp_clip_accumulate_recompute_batch(const dp_layer_desc *descs, const void *const *x, const void *const *dy,
                                             const float *const *sqnorm, const float *clip_c, float *const *acc_w,
                                             float *const *acc_b, void *const *ws, const size_t *ws_bytes, int n_layers,
                                             dp_stream stream)
{
    if (!descs || !x || !dy || !sqnorm || !clip_c || !acc_w || !ws || !ws_bytes)
        return fail(DP_ERR_INVALID_ARG, "descs, x, dy, sqnorm, clip_c, acc_w, ws and ws_bytes must be non-NULL host arrays");
    if (n_layers < 1) return fail(DP_ERR_INVALID_ARG, "n_layers = %d (need >= 1)", n_layers);
    std::vector<Geo> geo((size_t)n_layers);
    for (int l = 0; l < n_layers; ++l) {
        Geo &g = geo[(size_t)l];
        DP_TRY(make_geo(&descs[l], g));
        DP_TRY(check_ptr(x[l], "x[l]", true));
        DP_TRY(check_ptr(dy[l], "dy[l]", true));
        DP_TRY(check_ptr(sqnorm[l], "sqnorm[l]", true, 4));
        DP_TRY(check_ptr(acc_w[l], "acc_w[l]", true));
        float *ab = acc_b ? acc_b[l] : nullptr;
        DP_TRY(check_ptr(ab, "acc_b[l]", g.pb != 0));
        if (!g.pb && ab) return fail(DP_ERR_INVALID_ARG, "layer %d: acc_b given for a layer without bias", l);
        DP_TRY(check_clip(clip_c[l]));
        DP_TRY(check_ws(g, MODE_WEIGHTED, ws[l], ws_bytes[l]));
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    g_err[0] = 0;
    LaunchQueue q;
    q.stream = s;
    q.crowd = batch_target(geo);
    q.fuse = geo[0].n <= 2 ? 2 : 1;
    set_open_queue(&q);
    dp_status st = DP_OK;
    for (int l = 0; l < n_layers && st == DP_OK; ++l) {
        const Geo &g = geo[(size_t)l];
        float *ab = acc_b ? acc_b[l] : nullptr;
        st = launch_layer(g, MODE_WEIGHTED, x[l], dy[l], acc_w[l], ab, 0, nullptr, sqnorm[l], clip_c[l], ws[l], s);
    }
    if (st == DP_OK) st = flush_queue(q);
    set_open_queue(nullptr);
    return st;
}

dp_status dp_norms_from_partials(const float *const *partials, const int32_t *counts, const int32_t *group_of_layer,
                                 int n_layers, int n, int n_groups, float *group_sqnorm, dp_stream stream)
{
    if (!partials || !counts || !group_of_layer)
        return fail(DP_ERR_INVALID_ARG, "partials, counts and group_of_layer must be non-NULL host arrays");
    DP_TRY(check_ptr(group_sqnorm, "group_sqnorm", true, 4));
    if (n_layers < 1 || n < 1 || n_groups < 1)
        return fail(DP_ERR_INVALID_ARG, "n_layers (%d), n (%d) and n_groups (%d) must be >= 1", n_layers, n, n_groups);
    if (n_groups > 65535) return fail(DP_ERR_UNSUPPORTED, "more than 65535 clipping groups");
    for (int l = 0; l < n_layers; ++l) {
        if (!partials[l] || (reinterpret_cast<uintptr_t>(partials[l]) & 3u))
            return fail(DP_ERR_INVALID_ARG, "partials[%d] is NULL or not 4-byte aligned", l);
        if (counts[l] < 1) return fail(DP_ERR_INVALID_ARG, "counts[%d] = %d (need >= 1)", l, counts[l]);
        if (group_of_layer[l] < 0 || group_of_layer[l] >= n_groups)
            return fail(DP_ERR_INVALID_ARG, "group_of_layer[%d] = %d outside [0, %d)", l, group_of_layer[l], n_groups);
    }
    g_err[0] = 0;
    return launch_norms_from_partials(partials, counts, group_of_layer, n_layers, n, n_groups, group_sqnorm,
                                      static_cast<hipStream_t>(stream));
}

dp_status dp_norms(const float *layer_sqnorm, const int32_t *group_of_layer, int n_layers, int n, int n_groups,
                   float *group_sqnorm, dp_stream stream)
{
    DP_TRY(check_ptr(layer_sqnorm, "layer_sqnorm", true, 4));
    DP_TRY(check_ptr(group_of_layer, "group_of_layer", true, 4));
    DP_TRY(check_ptr(group_sqnorm, "group_sqnorm", true, 4));
    if (n_layers < 1 || n < 1 || n_groups < 1)
        return fail(DP_ERR_INVALID_ARG, "n_layers (%d), n (%d) and n_groups (%d) must be >= 1", n_layers, n, n_groups);
    if (n_groups > 65535) return fail(DP_ERR_UNSUPPORTED, "more than 65535 clipping groups");
    g_err[0] = 0;
    return launch_norms(layer_sqnorm, group_of_layer, n_layers, n, n_groups, group_sqnorm, static_cast<hipStream_t>(stream));
}

dp_status dp_clip_factors(const float *sqnorm, float clip_c, int n, float *f, dp_stream stream)
{
    DP_TRY(check_ptr(sqnorm, "sqnorm", true, 4));
    DP_TRY(check_ptr(f, "f", true, 4));
    DP_TRY(check_clip(clip_c));
    if (n < 1) return fail(DP_ERR_INVALID_ARG, "n = %d (need >= 1)", n);
    g_err[0] = 0;
    return launch_clip_factors(sqnorm, clip_c, n, f, static_cast<hipStream_t>(stream));
}

dp_status dp_clip_accumulate(const float *g, size_t g_stride, const float *sqnorm, float clip_c, int n, size_t p,
                             float *acc, dp_stream stream)
{
    DP_TRY(check_ptr(g, "g", true));
    DP_TRY(check_ptr(sqnorm, "sqnorm", true, 4));
    DP_TRY(check_ptr(acc, "acc", true));
    DP_TRY(check_clip(clip_c));
    if (n < 1) return fail(DP_ERR_INVALID_ARG, "n = %d (need >= 1)", n);
    if (p < 1) return fail(DP_ERR_INVALID_ARG, "p = 0 parameters");
    if (g_stride == 0) g_stride = p;
    if (g_stride < p) return fail(DP_ERR_INVALID_ARG, "g_stride smaller than p");
    if (p >= ((size_t)1 << 40)) return fail(DP_ERR_UNSUPPORTED, "p too large");
    g_err[0] = 0;
    return launch_clip_accumulate(g, g_stride, sqnorm, clip_c, n, p, acc, static_cast<hipStream_t>(stream));
}

dp_status dp_clip_accumulate_segments(const float *g, size_t g_stride, const float *group_sqnorm, int n_groups,
                                      const size_t *seg_begin, const int32_t *seg_group, const float *seg_clip, int n_seg,
                                      int n, size_t p, float *acc, dp_stream stream)
{
    DP_TRY(check_ptr(g, "g", true));
    DP_TRY(check_ptr(group_sqnorm, "group_sqnorm", true, 4));
    DP_TRY(check_ptr(acc, "acc", true));
    if (!seg_begin || !seg_group || !seg_clip) return fail(DP_ERR_INVALID_ARG, "segment tables must be non-NULL host arrays");
    if (n < 1 || n_groups < 1 || n_seg < 1) return fail(DP_ERR_INVALID_ARG, "n, n_groups and n_seg must be >= 1");
    if (p < 4 || p % 4) return fail(DP_ERR_INVALID_ARG, "p must be a positive multiple of 4");
    if (g_stride == 0) g_stride = p;
    if (g_stride < p || g_stride % 4) return fail(DP_ERR_INVALID_ARG, "g_stride must be a multiple of 4 and at least p");
    if (p >= ((size_t)1 << 40)) return fail(DP_ERR_UNSUPPORTED, "p too large");
    if (seg_begin[0] != 0) return fail(DP_ERR_INVALID_ARG, "the first segment must start at column 0");
    for (int k = 0; k < n_seg; ++k) {
        const size_t end = k + 1 < n_seg ? seg_begin[k + 1] : p;
        if (seg_begin[k] % 4 || seg_begin[k] >= end) return fail(DP_ERR_INVALID_ARG, "segment %d: boundaries must be increasing multiples of 4 below p", k);
        if (seg_group[k] < 0 || seg_group[k] >= n_groups) return fail(DP_ERR_INVALID_ARG, "segment %d: group %d outside [0, %d)", k, seg_group[k], n_groups);
        DP_TRY(check_clip(seg_clip[k]));
    }
    g_err[0] = 0;
    return launch_clip_accumulate_segments(g, g_stride, group_sqnorm, seg_begin, seg_group, seg_clip, n_seg, n, p, acc,
                                           static_cast<hipStream_t>(stream));
}

dp_status dp_clip_accumulate_recompute(const dp_layer_desc *desc, const void *x, const void *dy, const float *sqnorm,
                                       float clip_c, float *acc_w, float *acc_b, void *ws, size_t ws_bytes,
                                       dp_stream stream)
{
    Geo g;
    DP_TRY(make_geo(desc, g));
    DP_TRY(check_ptr(x, "x", true));
    DP_TRY(check_ptr(dy, "dy", true));
    DP_TRY(check_ptr(sqnorm, "sqnorm", true, 4));
    DP_TRY(check_ptr(acc_w, "acc_w", true));
    DP_TRY(check_ptr(acc_b, "acc_b", g.pb != 0));
    if (!g.pb && acc_b) return fail(DP_ERR_INVALID_ARG, "acc_b given for a layer without bias");
    DP_TRY(check_clip(clip_c));
    DP_TRY(check_ws(g, MODE_WEIGHTED, ws, ws_bytes));
    hipStream_t s = static_cast<hipStream_t>(stream);
    g_err[0] = 0;
    return launch_layer(g, MODE_WEIGHTED, x, dy, acc_w, acc_b, 0, nullptr, sqnorm, clip_c, ws, s);
}

dp_status dp_add_noise_finalize(const float *acc, float *out, size_t p, float sigma, float clip_total,
                                uint64_t total_batch, uint64_t seed, uint64_t step, uint32_t tensor_id,
                                dp_stream stream)
{
    DP_TRY(check_ptr(acc, "acc", true));
    DP_TRY(check_ptr(out, "out", true));
    if (p < 1) return fail(DP_ERR_INVALID_ARG, "p = 0 parameters");
    if (std::isnan(sigma) || sigma < 0.0f || std::isinf(sigma)) return fail(DP_ERR_INVALID_ARG, "sigma must be finite and >= 0");
    if (!(clip_total > 0.0f) || (sigma > 0.0f && !std::isfinite(clip_total)))
        return fail(DP_ERR_INVALID_ARG, "clip_total must be > 0, and finite unless sigma is 0");
    if (total_batch < 1) return fail(DP_ERR_INVALID_ARG, "total_batch = 0");
    if (p >= ((size_t)1 << 40)) return fail(DP_ERR_UNSUPPORTED, "p too large");
    g_err[0] = 0;
    return launch_noise_finalize(acc, out, p, sigma, clip_total, total_batch, seed, step, tensor_id,
                                 static_cast<hipStream_t>(stream));
}

dp_status dp_add_example_noise(float *acc, size_t p, float sigma, float clip_total, uint64_t total_batch, uint64_t seed,
                               uint64_t step, uint32_t tensor_id, uint64_t first_example, int n_examples,
                               const uint64_t *step_dev, dp_stream stream)
{
    DP_TRY(check_ptr(acc, "acc", true));
    DP_TRY(check_ptr(step_dev, "step_dev", false, 8));
    if (p < 1) return fail(DP_ERR_INVALID_ARG, "p = 0 parameters");
    if (std::isnan(sigma) || sigma < 0.0f || std::isinf(sigma)) return fail(DP_ERR_INVALID_ARG, "sigma must be finite and >= 0");
    if (!(clip_total > 0.0f) || (sigma > 0.0f && !std::isfinite(clip_total)))
        return fail(DP_ERR_INVALID_ARG, "clip_total must be > 0, and finite unless sigma is 0");
    if (total_batch < 1) return fail(DP_ERR_INVALID_ARG, "total_batch = 0");
    if (n_examples < 1) return fail(DP_ERR_INVALID_ARG, "n_examples = %d (need >= 1)", n_examples);
    if (first_example + (uint64_t)n_examples > total_batch)
        return fail(DP_ERR_INVALID_ARG, "examples %llu..%llu are outside the step's %llu examples",
                    (unsigned long long)first_example, (unsigned long long)(first_example + n_examples - 1),
                    (unsigned long long)total_batch);
    if (total_batch > 0xFFFFFFFFull) return fail(DP_ERR_UNSUPPORTED, "more than 2^32 examples per step");
    if (p > ((size_t)1 << 34)) return fail(DP_ERR_UNSUPPORTED, "p too large for the per-example stream");
    g_err[0] = 0;
    return launch_example_noise(acc, p, sigma, clip_total, total_batch, seed, step, tensor_id, first_example, n_examples,
                                step_dev, static_cast<hipStream_t>(stream));
}

dp_status dp_add_noise_finalize_update(const float *acc, float *theta, float *velocity, float *out, size_t p, float sigma,
                                       float clip_total, uint64_t total_batch, uint64_t seed, uint64_t step,
                                       uint32_t tensor_id, float lr, float momentum, dp_stream stream)
{
    DP_TRY(check_ptr(acc, "acc", true));
    DP_TRY(check_ptr(theta, "theta", true));
    DP_TRY(check_ptr(velocity, "velocity", false));
    DP_TRY(check_ptr(out, "out", false));
    if (p < 1) return fail(DP_ERR_INVALID_ARG, "p = 0 parameters");
    if (std::isnan(sigma) || sigma < 0.0f || std::isinf(sigma)) return fail(DP_ERR_INVALID_ARG, "sigma must be finite and >= 0");
    if (!(clip_total > 0.0f) || (sigma > 0.0f && !std::isfinite(clip_total)))
        return fail(DP_ERR_INVALID_ARG, "clip_total must be > 0, and finite unless sigma is 0");
    if (total_batch < 1) return fail(DP_ERR_INVALID_ARG, "total_batch = 0");
    if (!std::isfinite(lr)) return fail(DP_ERR_INVALID_ARG, "lr must be finite");
    if (!std::isfinite(momentum) || momentum < 0.0f) return fail(DP_ERR_INVALID_ARG, "momentum must be finite and >= 0");
    if (momentum != 0.0f && !velocity) return fail(DP_ERR_INVALID_ARG, "momentum != 0 needs a velocity buffer");
    if (p >= ((size_t)1 << 40)) return fail(DP_ERR_UNSUPPORTED, "p too large");
    g_err[0] = 0;
    return launch_noise_finalize_update(acc, theta, velocity, out, p, sigma, clip_total, total_batch, seed, step,
                                        tensor_id, lr, momentum, static_cast<hipStream_t>(stream));
}

dp_status dp_add_noise_finalize_flat(const float *acc, float *out, float *theta, float *velocity,
                                     const uint64_t *seg_begin, const uint64_t *seg_size, const uint32_t *seg_tensor_id,
                                     int n_seg, float sigma, float clip_total, uint64_t total_batch, uint64_t seed,
                                     uint64_t step, const uint64_t *step_dev, float lr, float momentum, dp_stream stream)
{
    DP_TRY(check_ptr(acc, "acc", true));
    DP_TRY(check_ptr(out, "out", theta == nullptr));
    DP_TRY(check_ptr(theta, "theta", false));
    DP_TRY(check_ptr(velocity, "velocity", false));
    DP_TRY(check_ptr(step_dev, "step_dev", false, 8));
    if (!seg_begin || !seg_size || !seg_tensor_id) return fail(DP_ERR_INVALID_ARG, "segment tables must be non-NULL host arrays");
    if (n_seg < 1) return fail(DP_ERR_INVALID_ARG, "n_seg = %d (need >= 1)", n_seg);
    if (std::isnan(sigma) || sigma < 0.0f || std::isinf(sigma)) return fail(DP_ERR_INVALID_ARG, "sigma must be finite and >= 0");
    if (!(clip_total > 0.0f) || (sigma > 0.0f && !std::isfinite(clip_total)))
        return fail(DP_ERR_INVALID_ARG, "clip_total must be > 0, and finite unless sigma is 0");
    if (total_batch < 1) return fail(DP_ERR_INVALID_ARG, "total_batch = 0");
    if (velocity && !theta) return fail(DP_ERR_INVALID_ARG, "velocity given without theta");
    if (theta) {
        if (!std::isfinite(lr)) return fail(DP_ERR_INVALID_ARG, "lr must be finite");
        if (!std::isfinite(momentum) || momentum < 0.0f) return fail(DP_ERR_INVALID_ARG, "momentum must be finite and >= 0");
        if (momentum != 0.0f && !velocity) return fail(DP_ERR_INVALID_ARG, "momentum != 0 needs a velocity buffer");
    }
    uint64_t end = 0;
    for (int k = 0; k < n_seg; ++k) {
        if (seg_begin[k] % 4) return fail(DP_ERR_INVALID_ARG, "tensor %d: seg_begin must be a multiple of 4", k);
        if (seg_begin[k] < end) return fail(DP_ERR_INVALID_ARG, "tensor %d overlaps the one before it (or the order is not increasing)", k);
        if (seg_size[k] < 1) return fail(DP_ERR_INVALID_ARG, "tensor %d: seg_size = 0", k);
        if (seg_size[k] >= ((uint64_t)1 << 32)) return fail(DP_ERR_UNSUPPORTED, "tensor %d: 2^32 elements or more", k);
        end = seg_begin[k] + seg_size[k];
    }
    if (end >= ((uint64_t)1 << 40)) return fail(DP_ERR_UNSUPPORTED, "parameter vector too large");
    g_err[0] = 0;
    return launch_noise_finalize_flat(acc, out, theta, velocity, seg_begin, seg_size, seg_tensor_id, n_seg, sigma, clip_total,
                                      total_batch, seed, step, step_dev, lr, momentum, static_cast<hipStream_t>(stream));
}

dp_status dp_philox_raw(uint32_t *raw, size_t p, uint64_t seed, uint64_t step, uint32_t tensor_id, dp_stream stream)
{
    DP_TRY(check_ptr(raw, "raw", true, 4));
    if (p < 1) return fail(DP_ERR_INVALID_ARG, "p = 0");
    if (p >= ((size_t)1 << 40)) return fail(DP_ERR_UNSUPPORTED, "p too large");
    g_err[0] = 0;
    return launch_philox_raw(raw, p, seed, step, tensor_id, static_cast<hipStream_t>(stream));
}

}  // extern "C"
