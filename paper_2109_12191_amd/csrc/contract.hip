// Per-example conv weight gradients as batched implicit-GEMM contractions on MFMA (gfx950).
//
// GEMM view of one example i of one conv layer (H1 of the path):
//     D_i[m, j] = sum_k A_i[m, k] * B_i[j, k]
//     m = output channel (Cout rows), j = (ci, kh, kw) flattened (J = Cin*KH*KW columns, the
//     framework's [Cout, Cin, KH, KW] weight layout read as a Cout x J matrix),
//     k = output position (oh, ow) flattened (S = OH*OW, the contraction),
//     A_i[m, k] = dY_i[m, k]               -- contiguous in k in NCHW
//     B_i[j, k] = Xpad_i[ci, oh*s+kh-p, ow*s+kw-p]  (zero outside the image).
//
// One workgroup (4 waves) owns one MT x NT tile of D.  It walks K in chunks: each chunk of A
// and of the im2col view of B is staged through LDS with K contiguous (the operand order
// v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32 want), then every wave runs its share of
// 32x32 MFMA tiles out of LDS.  Three things can happen to a finished tile:
//   * per-example mode: its squares are summed in registers and reduced with wavefront
//     shuffles to one partial per (example, tile) -- the gradient never goes back to HBM for
//     the norm -- and, if asked, the tile is also stored (materialised per-example gradient);
//   * weighted mode: K runs over (example, position) with dY_i scaled by the clip factor f_i
//     while it is staged, so the tile is sum_i f_i dW_i; it is added to the accumulator.
// The bias gradient db_i[m] = sum_k dY_i[m, k] rides along as one more MFMA against a
// register of ones in the workgroups of tile column 0.
#include "internal.h"

namespace dp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int THREADS = 256;
constexpr int PITCH = 144;            // bytes per LDS row: 128 data + 16 pad (odd multiple of 16 B:
                                      // 8 consecutive rows hit 8 distinct 16-byte bank groups)
constexpr int ROW_BYTES = 128;        // K-chunk per row: 64 bf16 or 32 fp32

struct ConvArgs {
    const void *x, *dy;
    float *out_w, *out_b;             // per-example: g_w / g_b (may be null); weighted: acc or ws slices
    size_t out_stride_w, out_stride_b;  // per-example row stride / weighted per-split stride
    float *partials;                  // per-example: [n, tiles] partial squared norms
    const float *group_sqnorm;        // weighted: [n]
    float clip_c;
    int n, cin, cout, h, w, kh, kw, stride, pad, oh, ow;
    int J, S;
    int tiles_m, tiles_n;
    int ex_per_split, splits;
    int accumulate;                   // weighted: 1 = out += tile, 0 = out = tile (workspace slice)
    int va, vb;                       // elements per 16-byte-or-smaller vector access of A / B rows
    int b_direct;                     // 1x1, stride 1, no padding: B is a plain matrix
};

// Entry of the per-tile column table used by the im2col gather.
struct ColInfo {
    int off;        // ci*H*W + (kh-p)*W + (kw-p)
    short dh, dw;   // kh-p, kw-p; dh = -30000 marks a column beyond J
};

template <bool BF16> struct ElemTraits;
template <> struct ElemTraits<true> {
    typedef uint16_t type;
    static constexpr int KC = 64;      // elements per K-chunk
    static constexpr int ESIZE = 2;
};
template <> struct ElemTraits<false> {
    typedef float type;
    static constexpr int KC = 32;
    static constexpr int ESIZE = 4;
};

// Stage ROWS x KC elements of a K-contiguous matrix (row r at base + r*row_stride) into
// registers as raw dwords.  Thread t owns the 16-byte pieces {t + 256*q}; piece c covers row
// c / 8, bytes (c % 8)*16 .. +15 of the row's 128-byte chunk.  V = elements per global load.
// Rows >= rows_valid and k >= k_valid read as zero.
template <bool BF16, int ROWS, int V>
__device__ __forceinline__ void load_rows(uint32_t (&st)[ROWS * ROW_BYTES / 4 / THREADS],
                                          const typename ElemTraits<BF16>::type *base, size_t row_stride,
                                          int rows_valid, int k0, int k_valid)
{
    typedef typename ElemTraits<BF16>::type E;
    constexpr int ES = ElemTraits<BF16>::ESIZE;
    constexpr int PIECES = ROWS * 8 / THREADS;        // 16-byte pieces per thread
    constexpr int EPP = 16 / ES;                      // elements per piece
#pragma unroll
    for (int q = 0; q < PIECES; ++q) {
        const int c = threadIdx.x + THREADS * q;
        const int row = c >> 3;
        const int k = k0 + (c & 7) * EPP;
        const E *src = base + (size_t)row * row_stride + k;
        const bool row_ok = row < rows_valid;
        if constexpr (V == EPP) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (row_ok && k < k_valid) v = *reinterpret_cast<const uint4 *>(src);
            st[q * 4 + 0] = v.x; st[q * 4 + 1] = v.y; st[q * 4 + 2] = v.z; st[q * 4 + 3] = v.w;
        } else if constexpr (V * ES == 8) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint2 v = make_uint2(0, 0);
                if (row_ok && k + h * V < k_valid) v = *reinterpret_cast<const uint2 *>(src + h * V);
                st[q * 4 + 2 * h] = v.x; st[q * 4 + 2 * h + 1] = v.y;
            }
        } else {
            // element-wise
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if constexpr (BF16) {
                    uint32_t lo = 0, hi = 0;
                    if (row_ok && k + 2 * d < k_valid) lo = src[2 * d];
                    if (row_ok && k + 2 * d + 1 < k_valid) hi = src[2 * d + 1];
                    st[q * 4 + d] = lo | (hi << 16);
                } else {
                    uint32_t v = 0;
                    if (row_ok && k + d < k_valid) v = __float_as_uint(src[d]);
                    st[q * 4 + d] = v;
                }
            }
        }
    }
}

template <bool BF16, int ROWS>
__device__ __forceinline__ void load_rows_any(uint32_t (&st)[ROWS * ROW_BYTES / 4 / THREADS],
                                              const typename ElemTraits<BF16>::type *base, size_t row_stride,
                                              int rows_valid, int k0, int k_valid, int v)
{
    constexpr int EPP = 16 / ElemTraits<BF16>::ESIZE;
    if (v == EPP) load_rows<BF16, ROWS, EPP>(st, base, row_stride, rows_valid, k0, k_valid);
    else if (v == EPP / 2) load_rows<BF16, ROWS, EPP / 2>(st, base, row_stride, rows_valid, k0, k_valid);
    else load_rows<BF16, ROWS, 1>(st, base, row_stride, rows_valid, k0, k_valid);
}

// im2col gather of ROWS columns-of-D x KC positions for a general conv.
template <bool BF16, int ROWS>
__device__ __forceinline__ void gather_rows(uint32_t (&st)[ROWS * ROW_BYTES / 4 / THREADS],
                                            const typename ElemTraits<BF16>::type *xi, const ColInfo *cols,
                                            const ConvArgs &a, int k0)
{
    constexpr int ES = ElemTraits<BF16>::ESIZE;
    constexpr int PIECES = ROWS * 8 / THREADS;
    constexpr int EPP = 16 / ES;
    // positions of this thread's piece are the same for all its rows: decode them once
    const int kbase = k0 + (threadIdx.x & 7) * EPP;
    int ihs[EPP], iws[EPP];
#pragma unroll
    for (int e = 0; e < EPP; ++e) {
        const int k = kbase + e;
        const int oh = k / a.ow, ow = k - oh * a.ow;
        ihs[e] = (k < a.S) ? oh * a.stride : -60000;      // pushes ih out of range
        iws[e] = ow * a.stride;
    }
#pragma unroll
    for (int q = 0; q < PIECES; ++q) {
        const int row = (threadIdx.x >> 3) + (THREADS / 8) * q;
        const ColInfo ci = cols[row];
        uint32_t v[EPP];
#pragma unroll
        for (int e = 0; e < EPP; ++e) {
            const int ih = ihs[e] + ci.dh, iw = iws[e] + ci.dw;
            const bool ok = (unsigned)ih < (unsigned)a.h && (unsigned)iw < (unsigned)a.w;
            const int idx = ok ? ci.off + ihs[e] * a.w + iws[e] : 0;
            if constexpr (BF16) {
                const uint32_t t = xi[idx];
                v[e] = ok ? t : 0u;
            } else {
                const float t = xi[idx];
                v[e] = ok ? __float_as_uint(t) : 0u;
            }
        }
        if constexpr (BF16) {
#pragma unroll
            for (int d = 0; d < 4; ++d) st[q * 4 + d] = v[2 * d] | (v[2 * d + 1] << 16);
        } else {
#pragma unroll
            for (int d = 0; d < 4; ++d) st[q * 4 + d] = v[d];
        }
    }
}

template <bool BF16, int N>
__device__ __forceinline__ void scale_regs(uint32_t (&st)[N], float f)
{
#pragma unroll
    for (int d = 0; d < N; ++d) {
        if constexpr (BF16) {
            const float lo = __uint_as_float(st[d] << 16) * f;
            const float hi = __uint_as_float(st[d] & 0xFFFF0000u) * f;
            st[d] = (uint32_t)float_to_bf16_bits(lo) | ((uint32_t)float_to_bf16_bits(hi) << 16);
        } else {
            st[d] = __float_as_uint(__uint_as_float(st[d]) * f);
        }
    }
}

template <int ROWS>
__device__ __forceinline__ void store_rows(const uint32_t (&st)[ROWS * ROW_BYTES / 4 / THREADS], char *lds)
{
    constexpr int PIECES = ROWS * 8 / THREADS;
#pragma unroll
    for (int q = 0; q < PIECES; ++q) {
        const int c = threadIdx.x + THREADS * q;
        *reinterpret_cast<uint4 *>(lds + (c >> 3) * PITCH + (c & 7) * 16) =
            make_uint4(st[q * 4], st[q * 4 + 1], st[q * 4 + 2], st[q * 4 + 3]);
    }
}

// MT = NT = 128 (BIG) or 64; 2x2 waves; each wave TM x TN tiles of 32x32.
template <bool BF16, bool BIG, bool WEIGHTED, bool BIAS>
__global__ void __launch_bounds__(THREADS) conv_contract_kernel(const ConvArgs a)
{
    typedef typename ElemTraits<BF16>::type E;
    constexpr int KC = ElemTraits<BF16>::KC;
    constexpr int MT = BIG ? 128 : 64, NT = MT;
    constexpr int TM = BIG ? 2 : 1, TN = TM;
    constexpr int WT = 32 * TM;                         // wave tile edge
    constexpr int REGS = MT * ROW_BYTES / 4 / THREADS;  // staging dwords per operand per thread

    __shared__ __attribute__((aligned(16))) char sA[MT * PITCH];
    __shared__ __attribute__((aligned(16))) char sB[NT * PITCH];
    __shared__ ColInfo cols[NT];
    __shared__ float red[4];

    // ---- which tile / example range: consecutive hardware workgroup ids rotate over the 8
    // XCDs, so id -> (id % 8) * per_xcd + id / 8 keeps the tiles of one example (which share
    // its A and B rows) on one XCD's L2.
    const int tiles = a.tiles_m * a.tiles_n;
    const int units = WEIGHTED ? a.splits : a.n;
    const int total = tiles * units;
    const int per_xcd = (total + 7) >> 3;
    const int wg = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (wg >= total) return;
    const int unit = wg / tiles;
    const int tile = wg - unit * tiles;
    const int tile_m = tile / a.tiles_n, tile_n = tile - tile_m * a.tiles_n;
    const int m0 = tile_m * MT, n0 = tile_n * NT;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // column table for the gather
    if (!a.b_direct && threadIdx.x < NT) {
        const int j = n0 + threadIdx.x;
        ColInfo c;
        if (j < a.J) {
            const int kk = a.kh * a.kw;
            const int ci = j / kk, r = j - ci * kk;
            const int kh = r / a.kw, kw = r - kh * a.kw;
            c.dh = (short)(kh - a.pad);
            c.dw = (short)(kw - a.pad);
            c.off = ci * a.h * a.w + (kh - a.pad) * a.w + (kw - a.pad);
        } else {
            c.dh = -30000; c.dw = 0; c.off = 0;
        }
        cols[threadIdx.x] = c;
    }
    __syncthreads();

    const int i_begin = WEIGHTED ? unit * a.ex_per_split : unit;
    const int i_end = WEIGHTED ? min(a.n, i_begin + a.ex_per_split) : unit + 1;
    const int chunks_per_ex = (a.S + KC - 1) / KC;
    const int n_chunks = (i_end - i_begin) * chunks_per_ex;

    const size_t x_ex = (size_t)a.cin * a.h * a.w, dy_ex = (size_t)a.cout * a.S;
    const E *xg = static_cast<const E *>(a.x), *dyg = static_cast<const E *>(a.dy);

    f32x16 acc[TM][TN];
    f32x16 accb[TM];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) accb[tm][r] = 0.0f;
    }
    const bool bias_here = BIAS && tile_n == 0 && wn == 0;

    uint32_t stA[REGS], stB[REGS];
    auto fetch = [&](int chunk) {
        const int i = i_begin + chunk / chunks_per_ex;
        const int k0 = (chunk - (chunk / chunks_per_ex) * chunks_per_ex) * KC;
        load_rows_any<BF16, MT>(stA, dyg + (size_t)i * dy_ex + (size_t)m0 * a.S, (size_t)a.S, a.cout - m0, k0, a.S,
                                a.va);
        if constexpr (WEIGHTED) scale_regs<BF16, REGS>(stA, clip_factor(a.group_sqnorm[i], a.clip_c));
        if (a.b_direct)
            load_rows_any<BF16, NT>(stB, xg + (size_t)i * x_ex + (size_t)n0 * a.S, (size_t)a.S, a.J - n0, k0, a.S,
                                    a.vb);
        else
            gather_rows<BF16, NT>(stB, xg + (size_t)i * x_ex, cols, a, k0);
    };

    if (n_chunks > 0) fetch(0);
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        __syncthreads();                       // everyone is done reading the previous chunk
        store_rows<MT>(stA, sA);
        store_rows<NT>(stB, sB);
        __syncthreads();
        if (chunk + 1 < n_chunks) fetch(chunk + 1);   // global loads fly while the MFMAs run

        const char *pa = sA + (wm * WT + (lane & 31)) * PITCH + (lane >> 5) * 16;
        const char *pb = sB + (wn * WT + (lane & 31)) * PITCH + (lane >> 5) * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {       // 4 x 32 bytes of K per row
            uint4 fa[TM], fb[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) fa[tm] = *reinterpret_cast<const uint4 *>(pa + tm * 32 * PITCH + ks * 32);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) fb[tn] = *reinterpret_cast<const uint4 *>(pb + tn * 32 * PITCH + ks * 32);
            if constexpr (BF16) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    const bf16x8 va = __builtin_bit_cast(bf16x8, fa[tm]);
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            va, __builtin_bit_cast(bf16x8, fb[tn]), acc[tm][tn], 0, 0, 0);
                    if constexpr (BIAS) {
                        if (bias_here) {
                            const uint4 one = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
                            accb[tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, __builtin_bit_cast(bf16x8, one),
                                                                               accb[tm], 0, 0, 0);
                        }
                    }
                }
            } else {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    const float av[4] = {__uint_as_float(fa[tm].x), __uint_as_float(fa[tm].y),
                                         __uint_as_float(fa[tm].z), __uint_as_float(fa[tm].w)};
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const float bv[4] = {__uint_as_float(fb[tn].x), __uint_as_float(fb[tn].y),
                                             __uint_as_float(fb[tn].z), __uint_as_float(fb[tn].w)};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[e], bv[e], acc[tm][tn], 0, 0, 0);
                    }
                    if constexpr (BIAS) {
                        if (bias_here) {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                accb[tm] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[e], 1.0f, accb[tm], 0, 0, 0);
                        }
                    }
                }
            }
        }

    }

    if constexpr (!WEIGHTED) {
        // ---- epilogue of one example's tile: squared norm in registers, optional store
        const int i = i_begin;
        float ss = 0.0f;
        const bool store = a.out_w != nullptr;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int j = n0 + wn * WT + tn * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float v = acc[tm][tn][r];
                    ss += v * v;                  // rows/columns beyond the matrix are exact zeros
                    if (store) {
                        const int m = m0 + wm * WT + tm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                        if (m < a.cout && j < a.J)
                            a.out_w[(size_t)i * a.out_stride_w + (size_t)m * a.J + j] = v;
                    }
                }
            }
            if constexpr (BIAS) {
                if (bias_here && (lane & 31) == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = accb[tm][r];
                        ss += v * v;
                        const int m = m0 + wm * WT + tm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                        if (store && m < a.cout) a.out_b[(size_t)i * a.out_stride_b + m] = v;
                    }
                }
            }
        }
        const float tot = block_sum<4>(ss, red);
        if (threadIdx.x == 0) a.partials[(size_t)i * tiles + tile] = tot;
    }

    if constexpr (WEIGHTED) {
        float *ow = a.out_w + (size_t)unit * a.out_stride_w;
        float *ob = a.out_b ? a.out_b + (size_t)unit * a.out_stride_b : nullptr;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int j = n0 + wn * WT + tn * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm * WT + tm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                    if (m < a.cout && j < a.J) {
                        float *p = ow + (size_t)m * a.J + j;
                        *p = a.accumulate ? *p + acc[tm][tn][r] : acc[tm][tn][r];
                    }
                }
            }
            if constexpr (BIAS) {
                if (bias_here && (lane & 31) == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = m0 + wm * WT + tm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                        if (m < a.cout) ob[m] = a.accumulate ? ob[m] + accb[tm][r] : accb[tm][r];
                    }
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------ host

static int pow2_divisor(int s, int vmax)
{
    int v = vmax;
    while (v > 1 && (s % v) != 0) v >>= 1;
    return v;
}

ConvPlan conv_plan(const Geo &g, int mode)
{
    ConvPlan p;
    const int J = g.cin * g.kh * g.kw;
    p.big = (g.cout > 64 && J > 64) ? 1 : 0;
    const int t = p.big ? 128 : 64;
    p.tiles_m = (g.cout + t - 1) / t;
    p.tiles_n = (J + t - 1) / t;
    p.splits = 1;
    if (mode == MODE_WEIGHTED) {
        const int tiles = p.tiles_m * p.tiles_n;
        int want = (256 + tiles - 1) / tiles;
        if (want > g.n) want = g.n;
        if (want < 1) want = 1;
        const int per = (g.n + want - 1) / want;
        p.splits = (g.n + per - 1) / per;
    }
    return p;
}

size_t conv_ws_bytes(const Geo &g, int mode)
{
    const ConvPlan p = conv_plan(g, mode);
    if (mode == MODE_WEIGHTED) return p.splits > 1 ? (size_t)p.splits * (g.pw + g.pb) * sizeof(float) : 0;
    return (size_t)g.n * p.tiles_m * p.tiles_n * sizeof(float);
}

const char *conv_variant_name(const Geo &g, int mode)
{
    static const char *names[2][2][2][2] = {
        {{{"conv_contract<f32,64x64,per_example>", "conv_contract<f32,64x64,per_example,bias>"},
          {"conv_contract<f32,64x64,weighted>", "conv_contract<f32,64x64,weighted,bias>"}},
         {{"conv_contract<f32,128x128,per_example>", "conv_contract<f32,128x128,per_example,bias>"},
          {"conv_contract<f32,128x128,weighted>", "conv_contract<f32,128x128,weighted,bias>"}}},
        {{{"conv_contract<bf16,64x64,per_example>", "conv_contract<bf16,64x64,per_example,bias>"},
          {"conv_contract<bf16,64x64,weighted>", "conv_contract<bf16,64x64,weighted,bias>"}},
         {{"conv_contract<bf16,128x128,per_example>", "conv_contract<bf16,128x128,per_example,bias>"},
          {"conv_contract<bf16,128x128,weighted>", "conv_contract<bf16,128x128,weighted,bias>"}}}};
    const ConvPlan p = conv_plan(g, mode);
    return names[g.bf16 ? 1 : 0][p.big][mode == MODE_WEIGHTED ? 1 : 0][g.has_bias ? 1 : 0];
}

template <bool BF16, bool BIG, bool WEIGHTED>
static void launch_variant(const ConvArgs &a, bool bias, unsigned blocks, hipStream_t s)
{
    if (bias)
        hipLaunchKernelGGL((conv_contract_kernel<BF16, BIG, WEIGHTED, true>), dim3(blocks), dim3(THREADS), 0, s, a);
    else
        hipLaunchKernelGGL((conv_contract_kernel<BF16, BIG, WEIGHTED, false>), dim3(blocks), dim3(THREADS), 0, s, a);
}

dp_status launch_conv(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                      size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c, void *ws,
                      hipStream_t s)
{
    const ConvPlan p = conv_plan(g, mode);
    ConvArgs a;
    a.x = x; a.dy = dy;
    a.n = g.n; a.cin = g.cin; a.cout = g.cout; a.h = g.h; a.w = g.w; a.kh = g.kh; a.kw = g.kw;
    a.stride = g.stride; a.pad = g.pad; a.oh = g.oh; a.ow = g.ow;
    a.J = g.cin * g.kh * g.kw;
    a.S = g.oh * g.ow;
    a.tiles_m = p.tiles_m; a.tiles_n = p.tiles_n;
    a.splits = p.splits;
    a.ex_per_split = (g.n + p.splits - 1) / p.splits;
    a.group_sqnorm = group_sqnorm; a.clip_c = clip_c;
    a.b_direct = (g.kh == 1 && g.kw == 1 && g.stride == 1 && g.pad == 0) ? 1 : 0;
    const int vmax = g.bf16 ? 8 : 4;
    a.va = pow2_divisor(a.S, vmax);
    a.vb = a.b_direct ? pow2_divisor(g.h * g.w, vmax) : 1;
    a.partials = nullptr;
    a.accumulate = 0;
    const int tiles = p.tiles_m * p.tiles_n;
    int units;
    if (mode == MODE_WEIGHTED) {
        units = p.splits;
        if (p.splits == 1) {
            a.out_w = out_w; a.out_b = out_b; a.out_stride_w = 0; a.out_stride_b = 0; a.accumulate = 1;
        } else {
            float *w = static_cast<float *>(ws);
            a.out_w = w; a.out_stride_w = g.pw + g.pb;
            a.out_b = w + g.pw; a.out_stride_b = g.pw + g.pb;
        }
    } else {
        units = g.n;
        a.out_w = out_w; a.out_b = out_b;
        a.out_stride_w = out_stride ? out_stride : g.pw;
        a.out_stride_b = out_stride ? out_stride : g.pb;
        a.partials = static_cast<float *>(ws);
    }
    const unsigned blocks = (unsigned)(((tiles * units + 7) / 8) * 8);
    const bool bias = g.has_bias != 0;
    const bool weighted = mode == MODE_WEIGHTED;
    if (g.bf16) {
        if (p.big) { if (weighted) launch_variant<true, true, true>(a, bias, blocks, s); else launch_variant<true, true, false>(a, bias, blocks, s); }
        else       { if (weighted) launch_variant<true, false, true>(a, bias, blocks, s); else launch_variant<true, false, false>(a, bias, blocks, s); }
    } else {
        if (p.big) { if (weighted) launch_variant<false, true, true>(a, bias, blocks, s); else launch_variant<false, true, false>(a, bias, blocks, s); }
        else       { if (weighted) launch_variant<false, false, true>(a, bias, blocks, s); else launch_variant<false, false, false>(a, bias, blocks, s); }
    }
    dp_status st = check_launch("conv_contract");
    if (st != DP_OK) return st;
    if (weighted) {
        if (p.splits > 1) {
            // slices hold [w | b] back to back; w and b accumulators are separate tensors
            st = launch_add_partial_sums(static_cast<float *>(ws), p.splits, g.pw + g.pb, g.pw, out_w, out_b, s);
        }
    } else if (sqnorm) {
        st = launch_sum_partials(static_cast<float *>(ws), g.n, tiles, sqnorm, s);
    }
    return st;
}

}  // namespace dp
