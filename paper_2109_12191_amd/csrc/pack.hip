// Operand packing for the clip-weighted contraction (the recomputation form of H4):
//     acc[co, j] += sum_i f_i sum_k dY_i[co, k] * Xcol_i[j, k],   f_i = min(1, C / |g_i|)
// is one GEMM whose K axis runs over (example, output position).  For layers with small
// feature maps the operands are first rewritten K-contiguous and 16-byte aligned:
//     dYp[grp][co][e * SP + k] = bf16(f_i * dY_i[co, k])            i = grp * EG + e
//     Xp [grp][j ][e * SP + k] = Xpad_i[ci, oh*s + kh - p, ow*s + kw - p]   (im2col row j = (ci,kh,kw))
// with SP = S rounded up to 8 and zeros in the padding, so that the contraction kernel streams
// plain aligned pieces with no masks, gathers or per-example scaling, whatever the stride, kernel
// size or parity of S.  The clip factor is applied here, in fp32, and rounded to bf16 once
// (nearest even) -- the same arithmetic the in-kernel scaling performs.
// `grp` splits the examples into ranges that different workgroups contract (the K slices).
#include "group.h"
#include "internal.h"
#include "pieces.h"

namespace dp {

namespace {

struct PackArgs {
    const uint16_t *x, *dy;
    uint16_t *xp, *dyp;
    const float *group_sqnorm;
    float clip_c;
    int n, cin, cout, h, w, kh, kw, stride, pad, oh, ow;
    int S, SP, J;
    int groups, eg;                 // example ranges and examples per range
    int kg8;                        // pieces per packed row: eg * SP / 8
    long long x_pieces, dy_pieces;
};

__global__ void __launch_bounds__(256) pack_weighted_kernel(const Grouped<PackArgs> layers)
{
    unsigned bid;
    const PackArgs &a = layers.a[group_pick(layers, bid)];
    const long long q = (long long)bid * 256 + threadIdx.x;
    uint32_t out[4] = {0u, 0u, 0u, 0u};
    if (q < a.x_pieces) {
        const int kk8 = (int)(q % a.kg8);
        const long long row = q / a.kg8;
        const int j = (int)(row % a.J), grp = (int)(row / a.J);
        const int kk = kk8 * 8;
        const int e = kk / a.SP, k0 = kk - e * a.SP;
        const int i = grp * a.eg + e;
        if (i < a.n) {
            const int taps = a.kh * a.kw;
            const int ci = j / taps, t = j - ci * taps;
            const int kh = t / a.kw, kw = t - kh * a.kw;
            const uint16_t *src = a.x + ((size_t)i * a.cin + ci) * a.h * a.w;
            if (taps == 1 && a.stride == 1 && a.pad == 0) {
                // 1x1 stride 1: the im2col row is the channel itself -- eight consecutive elements from whole dwords
                // (the run may start on an odd element), element by element only where that window would leave the tensor
                const long long e0 = ((long long)i * a.cin + ci) * a.S + k0;
                const int hi = min(8, a.S - k0);
                if ((e0 & ~1ll) + 10 <= (long long)a.n * a.cin * a.S) {
                    const Raw<5> raw = piece_load_words(reinterpret_cast<const uint32_t *>(a.x) + (e0 >> 1));
                    piece_finish<true, 1>(out, raw, (uint32_t)(e0 & 1), 0, hi);
                } else {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const uint32_t v = (k0 + u < a.S) ? src[k0 + u] : 0u;
                        out[u >> 1] |= v << ((u & 1) * 16);
                    }
                }
                *reinterpret_cast<uint4 *>(a.xp + q * 8) = make_uint4(out[0], out[1], out[2], out[3]);
                return;
            }
            int oh = k0 / a.ow, ow = k0 - oh * a.ow;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                uint32_t v = 0u;
                if (k0 + u < a.S) {
                    const int ih = oh * a.stride + kh - a.pad, iw = ow * a.stride + kw - a.pad;
                    if (ih >= 0 && ih < a.h && iw >= 0 && iw < a.w) v = src[ih * a.w + iw];
                }
                out[u >> 1] |= v << ((u & 1) * 16);
                if (++ow == a.ow) { ow = 0; ++oh; }
            }
        }
        *reinterpret_cast<uint4 *>(a.xp + q * 8) = make_uint4(out[0], out[1], out[2], out[3]);
        return;
    }
    const long long qd = q - a.x_pieces;
    if (qd >= a.dy_pieces) return;
    const int kk8 = (int)(qd % a.kg8);
    const long long row = qd / a.kg8;
    const int co = (int)(row % a.cout), grp = (int)(row / a.cout);
    const int kk = kk8 * 8;
    const int e = kk / a.SP, k0 = kk - e * a.SP;
    const int i = grp * a.eg + e;
    if (i < a.n) {
        const float f = clip_factor(a.group_sqnorm[i], a.clip_c);
        const uint16_t *src = a.dy + ((size_t)i * a.cout + co) * a.S;
        const long long e0 = ((long long)i * a.cout + co) * a.S + k0;
        const int hi = min(8, a.S - k0);
        if (hi > 0 && (e0 & ~1ll) + 10 <= (long long)a.n * a.cout * a.S) {
            const Raw<5> raw = piece_load_words(reinterpret_cast<const uint32_t *>(a.dy) + (e0 >> 1));
            piece_finish<true, 1>(out, raw, (uint32_t)(e0 & 1), 0, hi);
            scale_regs<true, 4>(out, f);                 // f * dY in fp32, rounded to bf16 once (nearest even)
        } else {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                uint32_t v = 0u;
                if (k0 + u < a.S) v = float_to_bf16_bits(bf16_bits_to_float(src[k0 + u]) * f);
                out[u >> 1] |= v << ((u & 1) * 16);
            }
        }
    }
    *reinterpret_cast<uint4 *>(a.dyp + qd * 8) = make_uint4(out[0], out[1], out[2], out[3]);
}

// Strided 1x1 convolutions only look at every stride-th row and column of X: this copies those
// into a compact [n*cin][OH*OW] tensor so that the contraction runs its plain aligned loader on
// half (a quarter, with both strides) of the bytes.  One thread per pair of output elements.
struct SubArgs {
    const uint16_t *x;
    uint16_t *out;
    long long rows;
    int h, w, oh, ow, stride;
};

__global__ void __launch_bounds__(256) subsample_kernel(const Grouped<SubArgs> grp)
{
    unsigned bid;
    const SubArgs &a = grp.a[group_pick(grp, bid)];
    const uint16_t *__restrict__ x = a.x;
    uint16_t *__restrict__ out = a.out;
    const long long rows = a.rows;
    const int w = a.w, ow = a.ow, stride = a.stride;
    const int S = a.oh * ow, pairs = (S + 1) / 2;
    const long long t = (long long)bid * 256 + threadIdx.x;
    if (t >= rows * pairs) return;
    const long long row = t / pairs;
    const int k = (int)(t - row * pairs) * 2;
    const uint16_t *src = x + (size_t)row * a.h * w;
    const int r0 = k / ow, c0 = k - r0 * ow;
    const uint32_t lo = src[(size_t)r0 * stride * w + c0 * stride];
    uint16_t *dst = out + (size_t)row * S + k;
    if (k + 1 < S) {
        const int k1 = k + 1, r1 = k1 / ow, c1 = k1 - r1 * ow;
        const uint32_t hi = src[(size_t)r1 * stride * w + c1 * stride];
        if (((size_t)row * S) % 2 == 0) *reinterpret_cast<uint32_t *>(dst) = lo | (hi << 16);
        else { dst[0] = (uint16_t)lo; dst[1] = (uint16_t)hi; }
    } else {
        dst[0] = (uint16_t)lo;
    }
}

}  // namespace

namespace {

// Channels-last inputs: [n][positions][channels] -> [n][channels][positions], 32 x 32 tiles through LDS (both the
// reads and the writes are runs of 32 consecutive elements).  One workgroup of 256 threads per tile.
struct TrArgs {
    const void *in;
    void *out;
    int positions, channels, tiles_p, tiles_c;
};

template <typename T>
__global__ void __launch_bounds__(256) channels_first_kernel(const Grouped<TrArgs> layers)
{
    __shared__ T tile[32][33];
    unsigned bid;
    const TrArgs &a = layers.a[group_pick(layers, bid)];
    const int per_ex = a.tiles_p * a.tiles_c;
    const int i = (int)(bid / (unsigned)per_ex), t = (int)(bid - (unsigned)i * (unsigned)per_ex);
    const int tc = t / a.tiles_p, tp = t - tc * a.tiles_p;
    const size_t ex = (size_t)i * a.positions * a.channels;
    const T *in = static_cast<const T *>(a.in) + ex;
    T *out = static_cast<T *>(a.out) + ex;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int p = tp * 32 + r, c = tc * 32 + tx;
        if (p < a.positions && c < a.channels) tile[r][tx] = in[(size_t)p * a.channels + c];
    }
    __syncthreads();
#pragma unroll
    for (int r = ty; r < 32; r += 8) {
        const int c = tc * 32 + r, p = tp * 32 + tx;
        if (p < a.positions && c < a.channels) out[(size_t)c * a.positions + p] = tile[tx][r];
    }
}

}  // namespace

dp_status launch_to_channels_first(const void *in, void *out, int n, int positions, int channels, int elem_bytes, hipStream_t s)
{
    TrArgs a;
    a.in = in; a.out = out; a.positions = positions; a.channels = channels;
    a.tiles_p = (positions + 31) / 32; a.tiles_c = (channels + 31) / 32;
    const long long blocks = (long long)n * a.tiles_p * a.tiles_c;
    if (blocks > 0x7FFFFFFFll) return fail(DP_ERR_UNSUPPORTED, "channels-last input too large");
    const void *fn = elem_bytes == 2 ? reinterpret_cast<const void *>(&channels_first_kernel<uint16_t>)
                                     : reinterpret_cast<const void *>(&channels_first_kernel<uint32_t>);
    return submit_kernel<TrArgs>(TIER_LAYOUT, fn, a, (unsigned)blocks, 256, 0, s, "channels_first");
}

dp_status launch_subsample(const Geo &g, const void *x, void *out, hipStream_t s)
{
    const long long rows = (long long)g.n * g.cin;
    const long long threads = rows * ((g.oh * g.ow + 1) / 2);
    const long long blocks = (threads + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(DP_ERR_UNSUPPORTED, "subsample: layer too large");
    SubArgs a;
    a.x = static_cast<const uint16_t *>(x); a.out = static_cast<uint16_t *>(out); a.rows = rows;
    a.h = g.h; a.w = g.w; a.oh = g.oh; a.ow = g.ow; a.stride = g.stride;
    return submit_kernel<SubArgs>(TIER_PRE, reinterpret_cast<const void *>(&subsample_kernel), a, (unsigned)blocks, 256, 0,
                                  s, "subsample");
}

PackPlan pack_plan(const Geo &g, int groups)
{
    PackPlan p;
    p.S = g.oh * g.ow;
    p.SP = (p.S + 7) / 8 * 8;
    p.J = g.cin * g.kh * g.kw;
    p.groups = groups;
    p.eg = (g.n + groups - 1) / groups;
    p.groups = (g.n + p.eg - 1) / p.eg;          // no empty trailing range
    p.kg = p.eg * p.SP;
    p.x_bytes = (size_t)p.groups * p.J * p.kg * 2;
    p.dy_bytes = (size_t)p.groups * g.cout * p.kg * 2;
    return p;
}

dp_status launch_pack_weighted(const Geo &g, const PackPlan &p, const void *x, const void *dy,
                               const float *group_sqnorm, float clip_c, void *xp, void *dyp, hipStream_t s)
{
    PackArgs a;
    a.x = static_cast<const uint16_t *>(x);
    a.dy = static_cast<const uint16_t *>(dy);
    a.xp = static_cast<uint16_t *>(xp);
    a.dyp = static_cast<uint16_t *>(dyp);
    a.group_sqnorm = group_sqnorm; a.clip_c = clip_c;
    a.n = g.n; a.cin = g.cin; a.cout = g.cout; a.h = g.h; a.w = g.w; a.kh = g.kh; a.kw = g.kw;
    a.stride = g.stride; a.pad = g.pad; a.oh = g.oh; a.ow = g.ow;
    a.S = p.S; a.SP = p.SP; a.J = p.J; a.groups = p.groups; a.eg = p.eg; a.kg8 = p.kg / 8;
    a.x_pieces = (long long)p.groups * p.J * a.kg8;
    a.dy_pieces = (long long)p.groups * g.cout * a.kg8;
    const long long blocks = (a.x_pieces + a.dy_pieces + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return fail(DP_ERR_UNSUPPORTED, "pack: layer too large");
    return submit_kernel<PackArgs>(TIER_PRE, reinterpret_cast<const void *>(&pack_weighted_kernel), a, (unsigned)blocks,
                                   256, 0, s, "pack_weighted");
}

}  // namespace dp
