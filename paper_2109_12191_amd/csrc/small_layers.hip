// Per-example gradients of dense layers and GroupNorm affine parameters (H1 for the layer
// kinds that are not convolutions).  With one token per example a dense weight gradient is
// the rank-one product dy_i (x) x_i: there is no contraction to put on MFMA, the kernel is a
// streaming outer product.  GroupNorm scale/shift gradients are two reductions over each
// channel of x and dy.
#include "internal.h"

namespace dp {

template <bool BF16> struct In;
template <> struct In<true> {
    typedef uint16_t type;
    static __device__ __forceinline__ float ld(const uint16_t *p) { return bf16_bits_to_float(*p); }
};
template <> struct In<false> {
    typedef float type;
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
};

// ------------------------------------------------------------------------------------------
// dense: dW_i[o,k] = sum_t dY_i[t,o] X_i[t,k];  db_i[o] = sum_t dY_i[t,o]
// Workgroup tile: DR rows (o) x 256 columns (k); a thread owns one column, so x loads and
// gradient stores are coalesced along k and dy values are wave-uniform.
constexpr int DR = 16;

struct DenseArgs {
    const void *x, *dy;
    float *out_w, *out_b;
    size_t out_stride_w, out_stride_b;
    float *partials;
    const float *group_sqnorm;
    float clip_c;
    int n, tokens, cin, cout, has_bias;
    int tiles_k, tiles_o;
};

template <bool BF16, bool WEIGHTED>
__global__ void __launch_bounds__(256) dense_kernel(const DenseArgs a)
{
    typedef typename In<BF16>::type E;
    __shared__ float red[4];
    const int tile_k = blockIdx.x, tile_o = blockIdx.y;
    const int k = tile_k * 256 + threadIdx.x;
    const int o0 = tile_o * DR;
    const bool k_ok = k < a.cin;
    const E *xg = static_cast<const E *>(a.x), *dyg = static_cast<const E *>(a.dy);
    const int i_begin = WEIGHTED ? 0 : blockIdx.z;
    const int i_end = WEIGHTED ? a.n : blockIdx.z + 1;
    const bool bias_thread = a.has_bias && tile_k == 0 && threadIdx.x < DR && o0 + threadIdx.x < a.cout;

    float acc[DR];
#pragma unroll
    for (int r = 0; r < DR; ++r) acc[r] = 0.0f;
    float accb = 0.0f;

    for (int i = i_begin; i < i_end; ++i) {
        const float f = WEIGHTED ? clip_factor(a.group_sqnorm[i], a.clip_c) : 1.0f;
        const E *xi = xg + (size_t)i * a.tokens * a.cin;
        const E *dyi = dyg + (size_t)i * a.tokens * a.cout;
        for (int t = 0; t < a.tokens; ++t) {
            const float xv = k_ok ? In<BF16>::ld(xi + (size_t)t * a.cin + k) * f : 0.0f;
#pragma unroll
            for (int r = 0; r < DR; ++r) {
                const int o = o0 + r;
                const float d = (o < a.cout) ? In<BF16>::ld(dyi + (size_t)t * a.cout + o) : 0.0f;
                acc[r] += d * xv;
            }
            if (bias_thread) accb += In<BF16>::ld(dyi + (size_t)t * a.cout + o0 + threadIdx.x) * f;
        }
    }

    if constexpr (!WEIGHTED) {
        const int i = i_begin;
        float ss = 0.0f;
#pragma unroll
        for (int r = 0; r < DR; ++r) {
            ss += acc[r] * acc[r];
            if (a.out_w && k_ok && o0 + r < a.cout)
                a.out_w[(size_t)i * a.out_stride_w + (size_t)(o0 + r) * a.cin + k] = acc[r];
        }
        if (bias_thread) {
            ss += accb * accb;
            if (a.out_w) a.out_b[(size_t)i * a.out_stride_b + o0 + threadIdx.x] = accb;
        }
        const float tot = block_sum<4>(ss, red);
        if (threadIdx.x == 0)
            a.partials[(size_t)i * (a.tiles_k * a.tiles_o) + tile_o * a.tiles_k + tile_k] = tot;
    } else {
#pragma unroll
        for (int r = 0; r < DR; ++r)
            if (k_ok && o0 + r < a.cout) a.out_w[(size_t)(o0 + r) * a.cin + k] += acc[r];
        if (bias_thread) a.out_b[o0 + threadIdx.x] += accb;
    }
}

// One token per example: the gradient is the rank-one product dy_i (x) x_i (plus db_i = dy_i), so
// its squared Frobenius norm is |dy_i|^2 |x_i|^2 (+ |dy_i|^2) -- the same number H2 defines, from
// two short reductions instead of Cout*Cin products.  One workgroup per example.
template <bool BF16>
__global__ void __launch_bounds__(256) dense_rank1_norm_kernel(const DenseArgs a, float *sqnorm)
{
    typedef typename In<BF16>::type E;
    __shared__ float red[4];
    const int i = blockIdx.x;
    const E *xi = static_cast<const E *>(a.x) + (size_t)i * a.cin;
    const E *dyi = static_cast<const E *>(a.dy) + (size_t)i * a.cout;
    float sx = 0.0f, sd = 0.0f;
    for (int k = threadIdx.x; k < a.cin; k += 256) { const float v = In<BF16>::ld(xi + k); sx += v * v; }
    for (int o = threadIdx.x; o < a.cout; o += 256) { const float v = In<BF16>::ld(dyi + o); sd += v * v; }
    sx = block_sum<4>(sx, red);
    sd = block_sum<4>(sd, red);
    if (threadIdx.x == 0) sqnorm[i] = sd * sx + (a.has_bias ? sd : 0.0f);
}

// One token per example, clip-weighted sum: acc[o, k] += sum_i (f_i dy_i[o]) x_i[k].  Same tile
// as dense_kernel (DR rows x 256 columns, a thread owns a column); the examples are taken 32 at
// a time: their scaled dy values go through LDS, a thread keeps eight x loads in flight, and
// the sum over examples runs in example order.
template <bool BF16>
__global__ void __launch_bounds__(256) dense_rank1_weighted_kernel(const DenseArgs a)
{
    typedef typename In<BF16>::type E;
    constexpr int EB = 32;
    __shared__ float sd[EB][DR];
    const int tile_k = blockIdx.x, tile_o = blockIdx.y;
    const int k = tile_k * 256 + threadIdx.x;
    const int o0 = tile_o * DR;
    const bool k_ok = k < a.cin;
    const E *xg = static_cast<const E *>(a.x), *dyg = static_cast<const E *>(a.dy);
    const bool bias_thread = a.has_bias && tile_k == 0 && threadIdx.x < DR && o0 + threadIdx.x < a.cout;
    float acc[DR];
#pragma unroll
    for (int r = 0; r < DR; ++r) acc[r] = 0.0f;
    float accb = 0.0f;
    for (int i0 = 0; i0 < a.n; i0 += EB) {
        __syncthreads();
        for (int q = threadIdx.x; q < EB * DR; q += 256) {
            const int ii = q / DR, r = q - ii * DR;
            const int i = i0 + ii, o = o0 + r;
            float v = 0.0f;
            if (i < a.n && o < a.cout)
                v = In<BF16>::ld(dyg + (size_t)i * a.cout + o) * clip_factor(a.group_sqnorm[i], a.clip_c);
            sd[ii][r] = v;
        }
        __syncthreads();
#pragma unroll 1
        for (int ib = 0; ib < EB; ib += 8) {          // eight x loads in flight at a time
            float xv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                xv[u] = (k_ok && i0 + ib + u < a.n) ? In<BF16>::ld(xg + (size_t)(i0 + ib + u) * a.cin + k) : 0.0f;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
#pragma unroll
                for (int r = 0; r < DR; ++r) acc[r] += sd[ib + u][r] * xv[u];
            }
        }
        if (bias_thread) {
#pragma unroll
            for (int ii = 0; ii < EB; ++ii) accb += sd[ii][threadIdx.x];
        }
    }
#pragma unroll
    for (int r = 0; r < DR; ++r)
        if (k_ok && o0 + r < a.cout) a.out_w[(size_t)(o0 + r) * a.cin + k] += acc[r];
    if (bias_thread) a.out_b[o0 + threadIdx.x] += accb;
}

size_t dense_norm_partial_count(const Geo &g, int mode)
{
    if (mode == MODE_NORM && g.h == 1) return 1;      // rank-one closed form: one value per example
    return (size_t)((g.cin + 255) / 256) * ((g.cout + DR - 1) / DR);
}

size_t gn_norm_partial_count(const Geo &g) { return (size_t)g.gn_groups; }

size_t dense_ws_bytes(const Geo &g, int mode)
{
    if (mode == MODE_WEIGHTED) return 0;
    const size_t tiles = (size_t)((g.cin + 255) / 256) * ((g.cout + DR - 1) / DR);
    return (size_t)g.n * tiles * sizeof(float);
}

dp_status launch_dense(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                       size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c, void *ws,
                       hipStream_t s)
{
    DenseArgs a;
    a.x = x; a.dy = dy; a.out_w = out_w; a.out_b = out_b;
    a.out_stride_w = out_stride ? out_stride : g.pw;
    a.out_stride_b = out_stride ? out_stride : g.pb;
    a.partials = static_cast<float *>(ws);
    a.group_sqnorm = group_sqnorm; a.clip_c = clip_c;
    a.n = g.n; a.tokens = g.h; a.cin = g.cin; a.cout = g.cout; a.has_bias = g.has_bias;
    a.tiles_k = (g.cin + 255) / 256;
    a.tiles_o = (g.cout + DR - 1) / DR;
    const bool weighted = mode == MODE_WEIGHTED;
    if (!weighted && !out_w && a.tokens == 1) {
        if (!sqnorm) sqnorm = static_cast<float *>(ws);      // left as the single partial per example
        if (g.bf16) hipLaunchKernelGGL((dense_rank1_norm_kernel<true>), dim3(g.n), dim3(256), 0, s, a, sqnorm);
        else hipLaunchKernelGGL((dense_rank1_norm_kernel<false>), dim3(g.n), dim3(256), 0, s, a, sqnorm);
        return check_launch("dense_rank1_norm");
    }
    const dim3 grid(a.tiles_k, a.tiles_o, weighted ? 1 : g.n);
    if (weighted && a.tokens == 1) {
        if (g.bf16) hipLaunchKernelGGL((dense_rank1_weighted_kernel<true>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((dense_rank1_weighted_kernel<false>), grid, dim3(256), 0, s, a);
        return check_launch("dense_rank1_weighted");
    }
    if (g.bf16) {
        if (weighted) hipLaunchKernelGGL((dense_kernel<true, true>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((dense_kernel<true, false>), grid, dim3(256), 0, s, a);
    } else {
        if (weighted) hipLaunchKernelGGL((dense_kernel<false, true>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((dense_kernel<false, false>), grid, dim3(256), 0, s, a);
    }
    dp_status st = check_launch("dense");
    if (st != DP_OK || weighted || !sqnorm) return st;
    return launch_sum_partials(a.partials, g.n, a.tiles_k * a.tiles_o, sqnorm, s);
}

// ------------------------------------------------------------------------------------------
// GroupNorm affine, groups of more than GN_CMAX channels: one workgroup per (example, group).  Mean
// and biased variance of the group's (C/G)*H*W elements in two passes (the group is L2-resident
// after the first), then
// each wave takes channels of the group in turn and reduces sum dy*xhat and sum dy with
// shuffles.
struct GnArgs {
    const void *x, *dy;
    float *out_w, *out_b;           // [n, stride] rows of dgamma / dbeta (may be null)
    size_t out_stride_w, out_stride_b;
    float *partials;                // [n, groups]
    int n, c, hw, groups;
    float eps;
};

template <bool BF16>
__global__ void __launch_bounds__(256) gn_affine_3pass_kernel(const GnArgs a)
{
    typedef typename In<BF16>::type E;
    __shared__ float red[4];
    const int grp = blockIdx.x, i = blockIdx.y;
    const int cg = a.c / a.groups;
    const size_t first = ((size_t)i * a.c + (size_t)grp * cg) * a.hw;
    const int cnt = cg * a.hw;
    const E *xg = static_cast<const E *>(a.x) + first;
    const E *dyg = static_cast<const E *>(a.dy) + first;

    // the mean is taken about the group's first element, so that a group far from zero keeps its spread
    const float k = In<BF16>::ld(xg);
    float s = 0.0f;
    for (int p = threadIdx.x; p < cnt; p += 256) s += In<BF16>::ld(xg + p) - k;
    const float m1 = block_sum<4>(s, red) / (float)cnt;              // mean - k
    float v = 0.0f;
    for (int p = threadIdx.x; p < cnt; p += 256) {
        const float d = (In<BF16>::ld(xg + p) - k) - m1;
        v += d * d;
    }
    const float var = block_sum<4>(v, red) / (float)cnt;
    const float rstd = 1.0f / sqrtf(var + a.eps);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float ss = 0.0f;
    for (int cl = wave; cl < cg; cl += 4) {
        const E *xc = xg + (size_t)cl * a.hw, *dc = dyg + (size_t)cl * a.hw;
        float sg = 0.0f, sb = 0.0f;
        for (int p = lane; p < a.hw; p += 64) {
            const float d = In<BF16>::ld(dc + p);
            sg += d * (((In<BF16>::ld(xc + p) - k) - m1) * rstd);
            sb += d;
        }
        sg = wave_sum(sg);
        sb = wave_sum(sb);
        if (lane == 0) {
            const int c = grp * cg + cl;
            ss += sg * sg + sb * sb;
            if (a.out_w) {
                a.out_w[(size_t)i * a.out_stride_w + c] = sg;
                a.out_b[(size_t)i * a.out_stride_b + c] = sb;
            }
        }
    }
    const float tot = block_sum<4>(ss, red);
    if (threadIdx.x == 0) a.partials[(size_t)i * a.groups + grp] = tot;
}

// One sweep over x and dy (groups of at most GN_CMAX channels): with k = the group's first element as
// a shift (so that the variance does not cancel), every wave takes channels in turn and accumulates
//     sum (x-k), sum (x-k)^2 for the group statistics,   sum dy (x-k), sum dy for the channel;
// then dgamma_c = rstd (sum dy (x-k) - (mean-k) sum dy), dbeta_c = sum dy.  Four independent loads per
// lane and stream are in flight.
constexpr int GN_CMAX = 256;

template <bool BF16>
__global__ void __launch_bounds__(256) gn_affine_kernel(const GnArgs a)
{
    typedef typename In<BF16>::type E;
    __shared__ float red[4];
    __shared__ float s_dx[GN_CMAX], s_d[GN_CMAX];
    const int grp = blockIdx.x, i = blockIdx.y;
    const int cg = a.c / a.groups;
    const size_t first = ((size_t)i * a.c + (size_t)grp * cg) * a.hw;
    const int cnt = cg * a.hw;
    const E *xg = static_cast<const E *>(a.x) + first;
    const E *dyg = static_cast<const E *>(a.dy) + first;
    const float k = In<BF16>::ld(xg);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    float sx = 0.0f, sxx = 0.0f;
    for (int cl = wave; cl < cg; cl += 4) {
        const E *xc = xg + (size_t)cl * a.hw, *dc = dyg + (size_t)cl * a.hw;
        float dx[4] = {0.0f, 0.0f, 0.0f, 0.0f}, d1[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        float x1[4] = {0.0f, 0.0f, 0.0f, 0.0f}, x2[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        int p = lane;
        for (; p + 192 < a.hw; p += 256) {
            float xv[4], dv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { xv[u] = In<BF16>::ld(xc + p + 64 * u) - k; dv[u] = In<BF16>::ld(dc + p + 64 * u); }
#pragma unroll
            for (int u = 0; u < 4; ++u) { dx[u] += dv[u] * xv[u]; d1[u] += dv[u]; x1[u] += xv[u]; x2[u] += xv[u] * xv[u]; }
        }
        for (; p < a.hw; p += 64) {
            const float xv = In<BF16>::ld(xc + p) - k, dv = In<BF16>::ld(dc + p);
            dx[0] += dv * xv; d1[0] += dv; x1[0] += xv; x2[0] += xv * xv;
        }
        const float sdx = wave_sum((dx[0] + dx[1]) + (dx[2] + dx[3]));
        const float sd = wave_sum((d1[0] + d1[1]) + (d1[2] + d1[3]));
        sx += (x1[0] + x1[1]) + (x1[2] + x1[3]);
        sxx += (x2[0] + x2[1]) + (x2[2] + x2[3]);
        if (lane == 0) { s_dx[cl] = sdx; s_d[cl] = sd; }
    }
    const float m1 = block_sum<4>(sx, red) / (float)cnt;               // mean - k
    const float m2 = block_sum<4>(sxx, red) / (float)cnt;
    const float var = fmaxf(m2 - m1 * m1, 0.0f);
    const float rstd = 1.0f / sqrtf(var + a.eps);
    float ss = 0.0f;
    for (int cl = threadIdx.x; cl < cg; cl += 256) {                   // block_sum's barriers made s_dx / s_d visible
        const float sg = rstd * (s_dx[cl] - m1 * s_d[cl]), sb = s_d[cl];
        const int c = grp * cg + cl;
        ss += sg * sg + sb * sb;
        if (a.out_w) {
            a.out_w[(size_t)i * a.out_stride_w + c] = sg;
            a.out_b[(size_t)i * a.out_stride_b + c] = sb;
        }
    }
    const float tot = block_sum<4>(ss, red);
    if (threadIdx.x == 0) a.partials[(size_t)i * a.groups + grp] = tot;
}

size_t gn_ws_bytes(const Geo &g, int mode)
{
    size_t b = (size_t)g.n * g.gn_groups * sizeof(float);
    b = (b + 15) & ~(size_t)15;
    if (mode == MODE_WEIGHTED) b += (size_t)g.n * 2 * g.cin * sizeof(float);
    return b;
}

dp_status launch_gn(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                    size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c, void *ws,
                    hipStream_t s)
{
    GnArgs a;
    a.x = x; a.dy = dy;
    a.partials = static_cast<float *>(ws);
    a.n = g.n; a.c = g.cin; a.hw = g.h * g.w; a.groups = g.gn_groups; a.eps = g.gn_eps;
    const bool weighted = mode == MODE_WEIGHTED;
    float *gw = out_w, *gb = out_b;
    if (weighted) {
        const size_t head = (((size_t)g.n * g.gn_groups * sizeof(float)) + 15) & ~(size_t)15;
        gw = reinterpret_cast<float *>(static_cast<char *>(ws) + head);
        gb = gw + (size_t)g.n * g.cin;
        a.out_stride_w = a.out_stride_b = (size_t)g.cin;
    } else {
        a.out_stride_w = out_stride ? out_stride : g.pw;
        a.out_stride_b = out_stride ? out_stride : g.pb;
    }
    a.out_w = gw; a.out_b = gb;
    const dim3 grid(g.gn_groups, g.n);
    const bool one_sweep = g.cin / g.gn_groups <= GN_CMAX;
    if (g.bf16) {
        if (one_sweep) hipLaunchKernelGGL(gn_affine_kernel<true>, grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL(gn_affine_3pass_kernel<true>, grid, dim3(256), 0, s, a);
    } else {
        if (one_sweep) hipLaunchKernelGGL(gn_affine_kernel<false>, grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL(gn_affine_3pass_kernel<false>, grid, dim3(256), 0, s, a);
    }
    dp_status st = check_launch("gn_affine");
    if (st != DP_OK) return st;
    if (weighted) {
        st = launch_clip_accumulate(gw, (size_t)g.cin, group_sqnorm, clip_c, g.n, (size_t)g.cin, out_w, s);
        if (st != DP_OK) return st;
        return launch_clip_accumulate(gb, (size_t)g.cin, group_sqnorm, clip_c, g.n, (size_t)g.cin, out_b, s);
    }
    if (!sqnorm) return st;
    return launch_sum_partials(a.partials, g.n, g.gn_groups, sqnorm, s);
}

// Clipping units: rows[u*unit .. (u+1)*unit) of the per-example scale / shift gradients are added (in example
// order), stored if wanted, and squared.  One workgroup per (256 channels, unit).
struct UnitRowsArgs {
    const float *gw, *gb;          // [n, c] per-example gradients
    float *out_w, *out_b;          // unit sums (may be null)
    size_t out_stride_w, out_stride_b;
    float *partials;               // [units, gridDim.x]
    int c, unit;
};

__global__ void __launch_bounds__(256) unit_rows_kernel(const UnitRowsArgs a)
{
    __shared__ float red[4];
    const int c = blockIdx.x * 256 + threadIdx.x, u = blockIdx.y;
    float sw = 0.0f, sb = 0.0f;
    if (c < a.c) {
        for (int e = 0; e < a.unit; ++e) {
            const size_t row = (size_t)(u * a.unit + e) * a.c + c;
            sw += a.gw[row];
            sb += a.gb[row];
        }
        if (a.out_w) {
            a.out_w[(size_t)u * a.out_stride_w + c] = sw;
            a.out_b[(size_t)u * a.out_stride_b + c] = sb;
        }
    }
    const float tot = block_sum<4>(sw * sw + sb * sb, red);
    if (threadIdx.x == 0) a.partials[(size_t)u * gridDim.x + blockIdx.x] = tot;
}

static size_t gn_unit_head(const Geo &g) { return gn_ws_bytes(g, MODE_WEIGHTED); }

size_t gn_unit_ws_bytes(const Geo &g, int unit)
{
    return gn_unit_head(g) + (size_t)(g.n / unit) * ((g.cin + 255) / 256) * sizeof(float);
}

const float *gn_unit_partials(const Geo &g, const void *ws) { return reinterpret_cast<const float *>(static_cast<const char *>(ws) + gn_unit_head(g)); }
size_t gn_unit_norm_partial_count(const Geo &g) { return (size_t)((g.cin + 255) / 256); }

dp_status launch_gn_units(const Geo &g, int unit, const void *x, const void *dy, float *out_w, float *out_b,
                          size_t out_stride, float *sqnorm, void *ws, hipStream_t s)
{
    // per-example gradients into the workspace (where the clip-weighted call keeps them), then the unit sums
    const size_t head = (((size_t)g.n * g.gn_groups * sizeof(float)) + 15) & ~(size_t)15;
    float *gw = reinterpret_cast<float *>(static_cast<char *>(ws) + head);
    float *gb = gw + (size_t)g.n * g.cin;
    dp_status st = launch_gn(g, MODE_MATERIALISE, x, dy, gw, gb, (size_t)g.cin, nullptr, nullptr, 0.0f, ws, s);
    if (st != DP_OK) return st;
    UnitRowsArgs a;
    a.gw = gw; a.gb = gb; a.out_w = out_w; a.out_b = out_b;
    a.out_stride_w = out_stride ? out_stride : g.pw;
    a.out_stride_b = out_stride ? out_stride : g.pb;
    a.partials = reinterpret_cast<float *>(static_cast<char *>(ws) + gn_unit_head(g));
    a.c = g.cin; a.unit = unit;
    const int blocks = (g.cin + 255) / 256, units = g.n / unit;
    hipLaunchKernelGGL(unit_rows_kernel, dim3(blocks, units), dim3(256), 0, s, a);
    st = check_launch("unit_rows");
    if (st != DP_OK || !sqnorm) return st;
    return launch_sum_partials(a.partials, units, blocks, sqnorm, s);
}

}  // namespace dp
