// Per-example weight gradients of the network's first convolution: 7x7, stride 2, pad 3, a handful of input
// channels (bf16), H1 of the path:
//     dW_i[co, ci, kh, kw] = sum_{oh, ow} dY_i[co, oh, ow] * Xpad_i[ci, 2 oh + kh - 3, 2 ow + kw - 3].
// With Cin = 3 the matrix is 64 x 147 but K is the whole 112 x 112 output map, and the im2col rows are 147 strided,
// shifted views of the same few image rows: the general kernel spends its time gathering them.  Here a workgroup of
// five waves takes a range of output rows of one example, two rows per step.  A step stages dY[2][64][OW] and the nine
// image rows 4 s - 3 .. 4 s + 5 of every channel into LDS through registers (the next step's loads are issued before
// the current step's MFMAs); an image row is split by column parity on the way,
//     E[c + 2] = X[2c]      O[c + 2] = X[2c + 1]      (zero outside the image),
// so that tap kw of output column ow is E[ow + (kw+1)/2] (kw odd) or O[ow + kw/2] (kw even): a contiguous run in ow.
// Wave w multiplies the 64 output channels with columns j = 32 w .. 32 w + 31 of the gradient (j = (ci, kh, kw)): a
// lane reads its own run of eight positions per K step, five dwords from a dword-aligned address, shifted by one
// element in registers where its run starts on an odd element.
// The ranges of an example meet in the workspace; a second kernel adds them in order, squares and stores.
#include "group.h"
#include "internal.h"
#include "pieces.h"

namespace dp {

namespace {

typedef uint32_t st_u32x4 __attribute__((ext_vector_type(4)));

constexpr int ST_THREADS = 320;                // five waves: columns 0 .. 159 of the gradient
constexpr int ST_COLS = 160;
constexpr int ST_COUT = 64;
constexpr int ST_FIX_BLOCKS = ST_COUT * ST_COLS / 256;       // 40 workgroups (and partial norms) per example
constexpr int ST_PT = 8;                       // 16-byte pieces a thread moves per step
constexpr int ST_LINES = 9;                    // image rows per channel and step: two output rows, seven taps

struct StemArgs {
    const uint16_t *x;              // [n][cin][H][W]
    const uint16_t *dy;             // [n][64][OH][OW]
    float *part;                    // [n][slices][64][160] partial blocks
    float *out_w;                   // [n] rows of out_stride floats, or null
    size_t out_stride;
    float *partials;                // [n][40]
    int n, cin, h, w, oh, ow, J;
    int slices, rows_per_slice;     // rows_per_slice is even
};

// a / d for 0 <= a < 4096, 1 <= d < 4096: (a + 1/2) / d is at least 1 / (2d) away from an integer, far more than the
// rounding of the reciprocal and the product
__device__ __forceinline__ int small_div(int a, int d) { return (int)(((float)a + 0.5f) * __builtin_amdgcn_rcpf((float)d)); }

__host__ __device__ inline int st_odd16(int b) { const int p = (b + 15) / 16; return (p | 1) * 16; }

// KSTEPS: K steps of 16 output columns per output row when known at compile time (the loop over them is unrolled and
// its LDS reads run ahead of the MFMAs), 0 for any width
template <int KSTEPS>
__global__ void __launch_bounds__(ST_THREADS) conv_stem_kernel(const Grouped<StemArgs> grp)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    unsigned bid;
    const StemArgs &a = grp.a[group_pick(grp, bid)];
    const int i = (int)bid / a.slices, sl = (int)bid - i * a.slices;
    const int oh_begin = sl * a.rows_per_slice, oh_end = min(a.oh, oh_begin + a.rows_per_slice);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int OW = a.ow, W = a.w, H = a.h;
    const int PA = st_odd16(OW * 2);                      // bytes per output channel in LDS (odd multiple of 16)
    const int EL = OW + 8;                                // elements of E (and of O) per staged image row
    const int XL = EL * 4;                                // bytes per staged image row: E, then O
    const int lines = a.cin * ST_LINES;
    char *sA = lds, *sX = lds + 2 * ST_COUT * PA;
    const int ppr = OW / 8, xpr = W / 8;                  // 16-byte pieces per dY row / image row
    const int n_a = 2 * ST_COUT * ppr, n_all = n_a + lines * xpr;

    // What this thread moves per step: source offset at output row 0 (elements, from the example's dY or image; the
    // offset of an image row above the image is negative and never used), where it goes in LDS, and a tag:
    // 0 nothing, 1 / 2 dY of the first / second row, 3 + k image row k of the step.
    int off[ST_PT], meta[ST_PT];
#pragma unroll
    for (int u = 0; u < ST_PT; ++u) {
        const int idx = (int)threadIdx.x + ST_THREADS * u;
        off[u] = 0; meta[u] = 0;
        if (idx < n_a) {
            // consecutive threads run along the two rows of one channel, which are contiguous in memory
            const int co = small_div(idx, 2 * ppr), q = idx - co * 2 * ppr, r = q >= ppr ? 1 : 0, pc = q - r * ppr;
            off[u] = (co * a.oh + r) * OW + pc * 8;
            meta[u] = ((r * ST_COUT + co) * PA + pc * 16) | ((1 + r) << 20);
        } else if (idx < n_all) {
            const int q = idx - n_a, line = small_div(q, xpr), pc = q - line * xpr, c = small_div(line, ST_LINES), k = line - c * ST_LINES;
            off[u] = (c * H + k - 3) * W + pc * 8;
            meta[u] = (2 * ST_COUT * PA + line * XL + (4 * pc + 2) * 2) | ((3 + k) << 20);
        }
    }
    const uint16_t *dy_ex = a.dy + (size_t)i * ST_COUT * a.oh * OW;
    const uint16_t *x_ex = a.x + (size_t)i * a.cin * H * W;

    // this lane's column of the gradient and where its runs start in a staged image row
    const int j = min(wave * 32 + (lane & 31), a.J - 1);  // columns beyond J compute a copy of the last one (never stored)
    const int ci = j / 49, tap = j - ci * 49, kh = tap / 7, kw = tap - kh * 7;
    const int e0 = ((kw & 1) ? (kw + 1) / 2 : EL + kw / 2) + 8 * (lane >> 5);     // element of the row at K step 0
    const unsigned sh = (e0 & 1) ? 2u : 0u;               // bytes to shift: the run starts on an odd element
    const char *bx = sX + (ci * ST_LINES + kh) * XL + (e0 & ~1) * 2;
    const char *pa = sA + (lane & 31) * PA + (lane >> 5) * 16;

    f32x16 acc[2];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[m][r] = 0.0f;

    // the image rows' margins stay zero: clear the whole region once
    for (int t = (int)threadIdx.x * 16; t < lines * XL; t += ST_THREADS * 16)
        *reinterpret_cast<st_u32x4 *>(sX + t) = st_u32x4{0u, 0u, 0u, 0u};

    st_u32x4 raw[ST_PT];
    auto fetch = [&](st_u32x4 (&raw)[ST_PT], int oh) {
#pragma unroll
        for (int u = 0; u < ST_PT; ++u) {
            const int tag = meta[u] >> 20;
            bool ok;
            const uint16_t *src;
            if (tag <= 2) {
                ok = tag != 0 && oh + (tag - 1) < oh_end;
                src = dy_ex + off[u] + oh * OW;
            } else {
                const int row = 2 * oh + (tag - 3) - 3;
                ok = row >= 0 && row < H && oh < oh_end;
                src = x_ex + off[u] + 2 * oh * W;
            }
            raw[u] = st_u32x4{0u, 0u, 0u, 0u};
            if (ok) raw[u] = *reinterpret_cast<const st_u32x4 *>(src);
        }
    };
    auto stage = [&](const st_u32x4 (&raw)[ST_PT]) {
#pragma unroll
        for (int u = 0; u < ST_PT; ++u) {
            const int tag = meta[u] >> 20;
            char *dst = lds + (meta[u] & 0xfffff);
            if (tag == 1 || tag == 2) {
                *reinterpret_cast<st_u32x4 *>(dst) = raw[u];
            } else if (tag >= 3) {
                uint32_t *pe = reinterpret_cast<uint32_t *>(dst), *po = reinterpret_cast<uint32_t *>(dst + EL * 2);
                pe[0] = __builtin_amdgcn_perm(raw[u].y, raw[u].x, 0x05040100u);
                pe[1] = __builtin_amdgcn_perm(raw[u].w, raw[u].z, 0x05040100u);
                po[0] = __builtin_amdgcn_perm(raw[u].y, raw[u].x, 0x07060302u);
                po[1] = __builtin_amdgcn_perm(raw[u].w, raw[u].z, 0x07060302u);
            }
        }
    };

    const int ksteps = KSTEPS ? KSTEPS : OW / 16;
    struct Operands { st_u32x4 a0, a1; uint32_t d[5]; };
    auto step_operands = [&](int t, Operands &o) {
        const int r = t >= ksteps ? 1 : 0, ks = t - r * ksteps;
        const uint32_t *p = reinterpret_cast<const uint32_t *>(bx + 2 * r * XL + ks * 32);
        const char *par = pa + r * ST_COUT * PA + ks * 32;
#pragma unroll
        for (int k = 0; k < 5; ++k) o.d[k] = p[k];
        o.a0 = *reinterpret_cast<const st_u32x4 *>(par);
        o.a1 = *reinterpret_cast<const st_u32x4 *>(par + 32 * PA);
    };
    auto step_mfma = [&](const Operands &o) {
        st_u32x4 b;
        b.x = __builtin_amdgcn_alignbyte(o.d[1], o.d[0], sh);
        b.y = __builtin_amdgcn_alignbyte(o.d[2], o.d[1], sh);
        b.z = __builtin_amdgcn_alignbyte(o.d[3], o.d[2], sh);
        b.w = __builtin_amdgcn_alignbyte(o.d[4], o.d[3], sh);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o.a0), __builtin_bit_cast(bf16x8, b), acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, o.a1), __builtin_bit_cast(bf16x8, b), acc[1], 0, 0, 0);
    };
    fetch(raw, oh_begin);
    for (int oh = oh_begin; oh < oh_end; oh += 2) {       // one step: output rows oh and oh + 1
        __syncthreads();                                  // the previous step has been read (first pass: the clearing is done)
        stage(raw);
        __syncthreads();
        fetch(raw, oh + 2);                               // in flight during the MFMAs (nothing beyond the range)
        // 2 ksteps K steps: the first row, then the second
        if constexpr (KSTEPS > 0) {
#pragma unroll
            for (int t = 0; t < 2 * KSTEPS; ++t) {
                Operands o;
                step_operands(t, o);
                step_mfma(o);
            }
        } else {
            // operands of the next step are read from LDS before this one's MFMAs
            const int T = 2 * ksteps;
            Operands cur, nxt;
            step_operands(0, cur);
            for (int t = 0; t < T; t += 2) {
                step_operands(t + 1, nxt);
                step_mfma(cur);
                step_operands(t + 2 < T ? t + 2 : t, cur);    // past the end: read something valid, never used
                step_mfma(nxt);
            }
        }
    }

    // this range's block: [64][160] floats, row co, column j (all 160 columns are written)
    float *mine = a.part + ((size_t)i * a.slices + sl) * (ST_COUT * ST_COLS);
    const int col = wave * 32 + (lane & 31);
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = m * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            mine[co * ST_COLS + col] = acc[m][r];
        }
}

// One thread per (example, co, column): the ranges in order, then the square and the store.
__global__ void __launch_bounds__(256) conv_stem_fixup_kernel(const Grouped<StemArgs> grp)
{
    __shared__ float red[4];
    unsigned bid;
    const StemArgs &a = grp.a[group_pick(grp, bid)];
    const int i = (int)bid / ST_FIX_BLOCKS, b = (int)bid - i * ST_FIX_BLOCKS;
    const int e = b * 256 + (int)threadIdx.x;
    const int co = e / ST_COLS, j = e - co * ST_COLS;
    const float *src = a.part + (size_t)i * a.slices * (ST_COUT * ST_COLS) + e;
    float v = 0.0f;
    for (int s = 0; s < a.slices; ++s) v += src[(size_t)s * (ST_COUT * ST_COLS)];
    float ss = 0.0f;
    if (j < a.J) {
        ss = v * v;
        if (a.out_w) a.out_w[(size_t)i * a.out_stride + (size_t)co * a.J + j] = v;
    }
    const float tot = block_sum<4>(ss, red);
    if (threadIdx.x == 0) a.partials[(size_t)i * ST_FIX_BLOCKS + b] = tot;
}

int stem_rows_per_slice(const Geo &g)
{
    // about one workgroup per compute unit; a range is an even number of output rows, at least four
    int slices = (256 + g.n - 1) / g.n;
    if (slices > g.oh / 4) slices = g.oh / 4;
    if (slices < 1) slices = 1;
    const int rows = (g.oh + slices - 1) / slices;
    return (rows + 1) & ~1;
}
int stem_slices(const Geo &g) { const int r = stem_rows_per_slice(g); return (g.oh + r - 1) / r; }
size_t st_align16(size_t b) { return (b + 15) & ~(size_t)15; }
unsigned stem_lds_bytes(const Geo &g) { return (unsigned)(2 * ST_COUT * st_odd16(g.ow * 2) + g.cin * ST_LINES * (g.ow + 8) * 4); }

}  // namespace

bool stem_applicable(const Geo &g, int mode)
{
    if (mode == MODE_WEIGHTED || !g.bf16 || g.has_bias || g.nhwc) return false;
    if (g.kh != 7 || g.kw != 7 || g.stride != 2 || g.pad != 3) return false;
    if (g.cout != ST_COUT || g.cin < 1 || g.cin * 49 > ST_COLS) return false;
    if (g.h % 2 || g.w % 2 || g.oh * 2 != g.h || g.ow * 2 != g.w || g.ow % 16 || g.oh < 4) return false;
    // the pieces of one step fit the staging registers, its rows fit LDS, offsets fit 32 bits
    const int pieces = 2 * ST_COUT * (g.ow / 8) + g.cin * ST_LINES * (g.w / 8);
    if (pieces > ST_PT * ST_THREADS || stem_lds_bytes(g) > 64 * 1024) return false;
    return (size_t)g.cin * g.h * g.w < ((size_t)1 << 30) && (size_t)g.cout * g.oh * g.ow < ((size_t)1 << 30);
}

size_t stem_norm_partial_count(void) { return ST_FIX_BLOCKS; }

// [n][40] partial norms, the partial blocks
size_t stem_ws_bytes(const Geo &g)
{
    return st_align16((size_t)g.n * ST_FIX_BLOCKS * sizeof(float)) + (size_t)g.n * stem_slices(g) * ST_COUT * ST_COLS * sizeof(float);
}

dp_status launch_stem(const Geo &g, const void *x, const void *dy, float *out_w, size_t out_stride, float *sqnorm, void *ws,
                      hipStream_t s)
{
    StemArgs a;
    char *w = static_cast<char *>(ws);
    a.partials = reinterpret_cast<float *>(w);
    w += st_align16((size_t)g.n * ST_FIX_BLOCKS * sizeof(float));
    a.part = reinterpret_cast<float *>(w);
    a.x = static_cast<const uint16_t *>(x);
    a.dy = static_cast<const uint16_t *>(dy);
    a.out_w = out_w;
    a.out_stride = out_stride ? out_stride : g.pw;
    a.n = g.n; a.cin = g.cin; a.h = g.h; a.w = g.w; a.oh = g.oh; a.ow = g.ow; a.J = g.cin * 49;
    a.rows_per_slice = stem_rows_per_slice(g);
    a.slices = stem_slices(g);
    const void *fn = g.ow == 112 ? reinterpret_cast<const void *>(&conv_stem_kernel<7>) : reinterpret_cast<const void *>(&conv_stem_kernel<0>);
    dp_status st = submit_main<StemArgs>(fn, a, (unsigned)(g.n * a.slices), ST_THREADS,
                                         stem_lds_bytes(g), s, "conv_stem");
    if (st != DP_OK) return st;
    st = submit_kernel<StemArgs>(TIER_POST, reinterpret_cast<const void *>(&conv_stem_fixup_kernel), a,
                                 (unsigned)(g.n * ST_FIX_BLOCKS), 256, 0, s, "conv_stem_fixup");
    if (st != DP_OK || !sqnorm) return st;
    const float *parts = a.partials;
    const int n = g.n;
    return submit_post([=]() -> dp_status { return launch_sum_partials(parts, n, ST_FIX_BLOCKS, sqnorm, s); });
}

}  // namespace dp
