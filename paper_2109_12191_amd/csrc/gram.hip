// Squared norms of per-example convolution gradients on small feature maps (1x1 stride 1; 3x3 pad 1 with
// stride 1 or 2), without forming the gradients (H2 for the layers whose gradients are recomputed later,
// never stored).
//
// For a 1x1 stride-1 convolution dW_i = A_i B_i^T with A_i = dY_i [Cout x S], B_i = X_i [Cin x S], so
//     ||dW_i||_F^2 = sum_{k,k'} (A_i^T A_i)[k,k'] * (B_i^T B_i)[k,k']
// -- the same number as the sum of squares of dW_i's entries, from two S x S Gram matrices instead
// of a Cout x Cin x S contraction.  With S <= 64 (7x7 maps: S = 49) that is ~8x fewer flops and no
// large tile to square.  Both Grams are contractions over CHANNELS, so each operand is transposed
// on its way into LDS (T[k][c], channels contiguous) and then feeds v_mfma_f32_32x32x16_bf16 like
// any K-contiguous operand.  For a 3x3 convolution B_i is the im2col matrix (rows (ci, kh, kw)), gathered
// from the image while it is transposed.
//
// Kernel 1: a workgroup takes one example and a slice of at most 256 channels of one operand and leaves
// its partial 64x64 Gram (accumulator register layout) in the workspace.  Kernel 2: one
// workgroup per example adds the slices in order, multiplies the Grams element by element and
// reduces.  Fixed order everywhere: same bits on every run.
#include "group.h"
#include "internal.h"
#include "pieces.h"

namespace dp {

namespace {

constexpr int GR_THREADS = 256;
constexpr int GR_CB = 256;                         // channels staged at a time
constexpr int GR_PT = GR_CB * 2 + 16;              // bytes per LDS row k (odd multiple of 16)

struct GramArgs {
    const uint16_t *a, *b;                         // dY [n][ca][S], X [n][cb][S]
    float *part;                                   // [n][sa + sb][4096]: slices of the dY Gram, then of the X Gram
    float *out;                                    // [n][GR_PARTS] partial squared norms
    int n, ca, cb, S;
    int sa, sb;                                    // channel slices (of at most `slice` channels) of dY and of X
    int slice;                                     // channels a workgroup takes: a multiple of 256
    int total_a, total_b;                          // elements in each tensor
    // 3x3 pad-1 convolutions: the rows of the second operand are im2col rows (ci, kh, kw) gathered from the
    // image X [n][cin][h][w]; cb = cin * 9 then.  taps == 1: X is the operand itself.
    int taps, cin, h, w, ow, stride;
};

// Gram of channels [c0, c1) of one example's matrix src[c][S] (element offset `base` from the
// tensor start): acc += T^T T restricted to this wave's 32x32 block (kb, kb2).
__device__ __forceinline__ void gram_part(f32x16 &acc, const uint16_t *tensor, int base, int total, int c0, int c1, int S,
                                          char *lds, int kb, int kb2, int lane)
{
    const uint32_t *words = reinterpret_cast<const uint32_t *>(tensor);
    for (int cblk = c0; cblk < c1; cblk += GR_CB) {
        __syncthreads();                           // the previous block has been consumed
        // ---- stage T[k][c]: thread -> (channel c = id % 256, piece pc = id / 256 of 8 positions)
        constexpr int NP = 8;                      // pieces per channel (64 positions)
        Raw<5> raw[NP];
#pragma unroll
        for (int pc = 0; pc < NP; ++pc) {
            const int c = cblk + (int)threadIdx.x;
            const int e0 = base + c * S + pc * 8;  // element index in the tensor
            const bool need = c < c1 && pc * 8 < S;
            const bool safe = need && (e0 & ~1) + 10 <= total;
            raw[pc] = piece_load_words(words + ((safe ? e0 : base) >> 1));
        }
#pragma unroll
        for (int pc = 0; pc < NP; ++pc) {
            const int c = cblk + (int)threadIdx.x;
            const int e0 = base + c * S + pc * 8;
            const bool need = c < c1 && pc * 8 < S;
            const bool safe = need && (e0 & ~1) + 10 <= total;
            const int hi = need ? min(8, S - pc * 8) : 0;
            uint32_t v[4];
            piece_finish<true, 1>(v, raw[pc], (uint32_t)(e0 & 1), 0, safe ? hi : 0);
            if (need && !safe) {                   // the last rows of the tensor: element by element
                v[0] = v[1] = v[2] = v[3] = 0u;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (e < hi) v[e >> 1] |= (uint32_t)tensor[e0 + e] << ((e & 1) * 16);
            }
            uint16_t *col = reinterpret_cast<uint16_t *>(lds + (pc * 8) * GR_PT) + threadIdx.x;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                *reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(col) + e * GR_PT) =
                    (uint16_t)(v[e >> 1] >> ((e & 1) * 16));
        }
        __syncthreads();
        // ---- MFMAs over the channels of this block
        const int nks = (min(GR_CB, c1 - cblk) + 15) / 16;
        const char *pa = lds + (kb * 32 + (lane & 31)) * GR_PT + (lane >> 5) * 16;
        const char *pb = lds + (kb2 * 32 + (lane & 31)) * GR_PT + (lane >> 5) * 16;
        for (int ks = 0; ks < nks; ++ks) {
            const bf16x8 va = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pa + ks * 32));
            const bf16x8 vb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pb + ks * 32));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, vb, acc, 0, 0, 0);
        }
    }
}

// The same for im2col rows [c0, c1) of a 3x3 pad-1 convolution (row j = (ci, kh, kw), column k = (oh, ow)):
//     T[k][j] = Xpad[ci][oh * stride + kh - 1][ow * stride + kw - 1],
// gathered element by element (the nine taps of a channel re-read the same few bytes, from L1).
__device__ __forceinline__ void gram_part_im2col(f32x16 &acc, const GramArgs &a, int i, int c0, int c1, char *lds, int kb,
                                                 int kb2, int lane)
{
    for (int cblk = c0; cblk < c1; cblk += GR_CB) {
        __syncthreads();
        const int j = cblk + (int)threadIdx.x;
        const bool live = j < c1;
        const int ci = j / 9, tap = j - ci * 9;
        const int dh = tap / 3 - 1, dw = tap - (tap / 3) * 3 - 1;
        const uint16_t *img = a.b + ((size_t)i * a.cin + (live ? ci : 0)) * a.h * a.w;
        uint16_t vals[64];
        int oh = 0, owc = 0;
#pragma unroll
        for (int k = 0; k < 64; ++k) {
            const int ih = oh * a.stride + dh, iw = owc * a.stride + dw;
            const bool ok = live && k < a.S && ih >= 0 && ih < a.h && iw >= 0 && iw < a.w;
            vals[k] = ok ? img[ih * a.w + iw] : (uint16_t)0;
            if (++owc == a.ow) { owc = 0; ++oh; }
        }
        uint16_t *col = reinterpret_cast<uint16_t *>(lds) + threadIdx.x;
#pragma unroll
        for (int k = 0; k < 64; ++k) *reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(col) + k * GR_PT) = vals[k];
        __syncthreads();
        const int nks = (min(GR_CB, c1 - cblk) + 15) / 16;
        const char *pa = lds + (kb * 32 + (lane & 31)) * GR_PT + (lane >> 5) * 16;
        const char *pb = lds + (kb2 * 32 + (lane & 31)) * GR_PT + (lane >> 5) * 16;
        for (int ks = 0; ks < nks; ++ks) {
            const bf16x8 va = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pa + ks * 32));
            const bf16x8 vb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pb + ks * 32));
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, vb, acc, 0, 0, 0);
        }
    }
}

__global__ void __launch_bounds__(GR_THREADS) gram_partial_kernel(const Grouped<GramArgs> grp)
{
    __shared__ __attribute__((aligned(16))) char lds[64 * GR_PT];
    unsigned bid;
    const GramArgs &a = grp.a[group_pick(grp, bid)];
    const int slots = a.sa + a.sb;
    const int i = bid / slots, s = bid - i * slots;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kb = wave >> 1, kb2 = wave & 1;
    f32x16 gm;
#pragma unroll
    for (int r = 0; r < 16; ++r) gm[r] = 0.0f;
    // one slice of one operand per workgroup: one to four blocks of 256 channels (one memory round trip each)
    if (s < a.sa)
        gram_part(gm, a.a, i * a.ca * a.S, a.total_a, s * a.slice, min(a.ca, (s + 1) * a.slice), a.S, lds, kb, kb2, lane);
    else if (a.taps == 1)
        gram_part(gm, a.b, i * a.cb * a.S, a.total_b, (s - a.sa) * a.slice, min(a.cb, (s - a.sa + 1) * a.slice), a.S, lds, kb, kb2,
                  lane);
    else
        gram_part_im2col(gm, a, i, (s - a.sa) * a.slice, min(a.cb, (s - a.sa + 1) * a.slice), lds, kb, kb2, lane);
    float *mine = a.part + (size_t)bid * 4096;
#pragma unroll
    for (int r = 0; r < 16; ++r) mine[r * GR_THREADS + threadIdx.x] = gm[r];
}

// One workgroup per (example, accumulator register r): 256 Gram entries each; the slices are added in
// order, the two Grams multiplied entry by entry and the products reduced to one partial norm.
constexpr int GR_PARTS = 16;
constexpr int GR_SA_MAX = 16, GR_SB_MAX = 40;      // slices of 256 rows: Cout <= 4096, Cin*k*k <= 10240

__global__ void __launch_bounds__(GR_THREADS) gram_combine_kernel(const Grouped<GramArgs> grp)
{
    __shared__ float red[4];
    unsigned bid;
    const GramArgs &a = grp.a[group_pick(grp, bid)];
    const int i = bid / GR_PARTS, r = bid - i * GR_PARTS;
    const float *base = a.part + (size_t)i * (a.sa + a.sb) * 4096 + r * GR_THREADS + threadIdx.x;
    float va[GR_SA_MAX], vb[GR_SB_MAX];            // all loads in flight together
#pragma unroll
    for (int s = 0; s < GR_SA_MAX; ++s) va[s] = s < a.sa ? base[(size_t)s * 4096] : 0.0f;
#pragma unroll
    for (int s = 0; s < GR_SB_MAX; ++s) vb[s] = s < a.sb ? base[(size_t)(a.sa + s) * 4096] : 0.0f;
    float ga = 0.0f, gb = 0.0f;
#pragma unroll
    for (int s = 0; s < GR_SA_MAX; ++s) ga += va[s];
#pragma unroll
    for (int s = 0; s < GR_SB_MAX; ++s) gb += vb[s];
    const float tot = block_sum<4>(ga * gb, red);
    if (threadIdx.x == 0) a.out[bid] = tot;
}

int gram_rows_b(const Geo &g) { return g.cin * g.kh * g.kw; }
// Channels per workgroup: every slice leaves a 16 KB partial Gram in the workspace, which the second kernel reads back --
// with 256-channel slices that is more bytes than the operands themselves.  Inside a batch call (the launch is shared
// with other layers and has thousands of workgroups) a workgroup takes four blocks; a layer alone keeps one block per
// workgroup, for the parallelism.  Workspace sizes cover the one-block plan, the larger of the two.
int gram_slice(const Geo &g) { return (crowd_hint() > 0 && g.n >= 8) ? 4 * GR_CB : GR_CB; }
int gram_slots(const Geo &g) { return (g.cout + GR_CB - 1) / GR_CB + (gram_rows_b(g) + GR_CB - 1) / GR_CB; }

size_t gram_align16(size_t b) { return (b + 15) & ~(size_t)15; }

}  // namespace

bool gram_norm_applicable(const Geo &g, int mode)
{
    if (mode != MODE_NORM || !g.bf16 || g.has_bias) return false;
    const bool one = g.kh == 1 && g.kw == 1 && g.stride == 1 && g.pad == 0;
    const bool three = g.kh == 3 && g.kw == 3 && g.pad == 1 && (g.stride == 1 || g.stride == 2);
    if (!one && !three) return false;
    const long long S = (long long)g.oh * g.ow, J = (long long)g.cin * g.kh * g.kw;
    if (S > 64 || S < 8) return false;
    if (g.cin < 128 || g.cout < 128 || g.cout > GR_SA_MAX * GR_CB || J > GR_SB_MAX * GR_CB) return false;
    // the Gram route wins when S is small against the channel counts (S^2 (J+Cout) << S J Cout)
    if (S * (J + g.cout) * 4 > J * g.cout) return false;
    return (long long)g.n * g.cin * g.h * g.w < (1ll << 31) && (long long)g.n * g.cout * S < (1ll << 31);
}

size_t gram_ws_bytes(const Geo &g)
{
    return gram_align16((size_t)g.n * GR_PARTS * sizeof(float)) + (size_t)g.n * gram_slots(g) * 4096 * sizeof(float);
}

dp_status launch_gram_norm(const Geo &g, const void *x, const void *dy, float *sqnorm, void *ws, hipStream_t s)
{
    GramArgs a;
    a.a = static_cast<const uint16_t *>(dy);
    a.b = static_cast<const uint16_t *>(x);
    a.n = g.n; a.ca = g.cout; a.cb = gram_rows_b(g); a.S = g.oh * g.ow;
    a.slice = gram_slice(g);
    a.sa = (g.cout + a.slice - 1) / a.slice; a.sb = (a.cb + a.slice - 1) / a.slice;
    a.taps = g.kh * g.kw; a.cin = g.cin; a.h = g.h; a.w = g.w; a.ow = g.ow; a.stride = g.stride;
    a.total_a = g.n * g.cout * a.S;
    a.total_b = g.n * g.cin * g.h * g.w;
    // the partial norms [n][16] sit at the start of the workspace, the partial Grams after them
    a.out = static_cast<float *>(ws);
    a.part = reinterpret_cast<float *>(static_cast<char *>(ws) + gram_align16((size_t)g.n * GR_PARTS * sizeof(float)));
    // the kernel remap of the contraction launches does not apply here: any workgroup count will do
    dp_status st = submit_kernel<GramArgs>(TIER_MAIN, reinterpret_cast<const void *>(&gram_partial_kernel), a,
                                           (unsigned)(g.n * (a.sa + a.sb)), GR_THREADS, 0, s, "gram_partial");
    if (st != DP_OK) return st;
    st = submit_kernel<GramArgs>(TIER_POST, reinterpret_cast<const void *>(&gram_combine_kernel), a,
                                 (unsigned)(g.n * GR_PARTS), GR_THREADS, 0, s, "gram_combine");
    if (st != DP_OK || !sqnorm) return st;
    const float *parts = a.out;
    const int n = g.n;
    return submit_post([=]() -> dp_status { return launch_sum_partials(parts, n, GR_PARTS, sqnorm, s); });
}

size_t gram_norm_partial_count(void) { return GR_PARTS; }

}  // namespace dp
