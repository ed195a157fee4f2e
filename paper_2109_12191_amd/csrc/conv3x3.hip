// Per-example weight gradients of 3x3, stride-1, pad-1 convolutions (bf16) from raw image rows.
//
// Same contraction as the general kernel (H1 of the path; per example i
//     dW_i[co, ci, kh, kw] = sum_{oh, ow} dY_i[co, oh, ow] * Xpad_i[ci, oh + kh - 1, ow + kw - 1]),
// but the nine taps of one input channel are nine shifted views of the SAME rows of X, so a
// workgroup stages each row once and builds all nine MFMA operands from it:
//
//   * a workgroup owns 64 output channels x 64 input channels x 9 taps of one example (four
//     waves, each 32 co x 32 ci x 9 taps = nine 32x32 accumulator tiles) and walks chunks of R
//     output rows;
//   * per chunk it stages dY[64 co][R rows] (K-contiguous, rows padded to OWP = W rounded up to
//     8) and X[64 ci][R + 2 rows][WP = OWP + 8 columns] into LDS; X is stored with column
//     c = iw + 1, zeros for iw = -1, iw >= W and rows outside the image, so every tap reads
//     plain in-range LDS;
//   * per 16 values of K a lane reads 16 bytes of dY and, per kernel row kh, 20 bytes of X
//     starting at column ow0: tap kw = 0 is dwords 0..3, kw = 1 the same five dwords shifted by
//     one element, kw = 2 dwords 1..4 -- nine MFMAs from four LDS reads.
//
// Against the general kernel this cuts global/L2 reads of X by ~9x (each row is fetched once
// per workgroup instead of once per tap) and LDS reads per MFMA by ~3x.
//
// K may be sliced over workgroups (few tiles, long K): slices store their accumulators in the
// workspace and a second kernel adds them in slice order, so results are run-to-run identical.
#include "internal.h"
#include "group.h"
#include "pieces.h"

#include <atomic>
#include <cstdio>

namespace dp {

namespace {

constexpr int C3_THREADS = 256;

struct C3Args {
    const uint16_t *x, *dy;
    float *out_w;                     // per-example gradients (may be null) or, weighted, the accumulator
    size_t out_stride;
    float *partials;                  // [n, tiles] partial squared norms
    float *ws_part;                   // sliced K / example ranges: accumulators in register layout
    const float *group_sqnorm;        // weighted: [n]
    float clip_c;
    int n, cin, cout, h;              // h: OUTPUT height (= input height for stride 1)
    int hin;                          // input height
    int tiles_co, tiles_ci;
    int chunks;                       // ceil(H / R)
    int ksplit, chunks_per_split;     // per-example mode: K slices
    int ex_per_split;                 // weighted mode: examples per workgroup (ksplit = example ranges)
    int variant;                      // which body conv3x3_any_kernel runs for this layer (C3_ANY_* below)
    int unit_major;                   // weighted mode: every example range keeps its own result (clipping units): the
                                      // slices always go to the workspace, ordered (range, tile)
};

constexpr int odd16(int bytes) { return ((bytes / 16) | 1) * 16; }
constexpr int C3_RP = 292;                           // floats per row staged by the store epilogue: 288 + 4
constexpr int C3_STORE_LDS = 4 * 8 * C3_RP * 4;      // bytes the store epilogue needs: 4 waves x 8 rows

// W is the OUTPUT row width.  Stride 1 reads X itself (input width W).  Stride 2 reads a copy of X
// whose rows have been split by column parity (deinterleave2_kernel below): each row is
//     O'[c] = X[2c - 1], c = 0 .. OWP+7   (zero for 2c-1 outside the row)   then   E[c] = X[2c], c = 0 .. OWP-1,
// so that tap kw = 0 is O'[ow], kw = 1 is E[ow], kw = 2 is O'[ow + 1]: contiguous runs again.
template <int W, int STRIDE> struct C3Cfg {
    static constexpr int OWP = (W + 7) / 8 * 8;
    static constexpr int R = (STRIDE == 1) ? ((OWP == 8) ? 8 : 224 / OWP)            // output rows per chunk
                                           : ((OWP == 16) ? 5 : (OWP == 32 ? 3 : 8));
    static constexpr int KSTEPS = R * OWP / 16;
    static constexpr int WP = (STRIDE == 1) ? OWP + 8 : 2 * OWP + 8;                  // elements per staged X row
    static constexpr int E_OFF = OWP + 8;                                           // stride 2: where E starts in a row
    static constexpr int XROWS = (STRIDE == 1) ? R + 2 : 2 * R + 1;
    static constexpr int PPR = OWP / 8, XPR = WP / 8;         // 16-byte pieces per LDS row
    static constexpr int PA = odd16(R * OWP * 2);             // bytes per co in LDS (odd multiple of 16)
    static constexpr int PX = odd16(XROWS * WP * 2);          // bytes per ci in LDS
    static constexpr int NPA = 64 * R * PPR, NPX = 64 * XROWS * XPR;
    static constexpr int PA_T = (NPA + C3_THREADS - 1) / C3_THREADS;
    static constexpr int PX_T = (NPX + C3_THREADS - 1) / C3_THREADS;
    static constexpr int LDS = (64 * PA + 64 * PX > C3_STORE_LDS) ? 64 * PA + 64 * PX : C3_STORE_LDS;
    static constexpr bool ALIGNED_A = (W % 8 == 0);
    static_assert(OWP == 8 || OWP == 16 || OWP == 32 || OWP == 56, "supported row widths");
    static_assert(R * OWP % 16 == 0, "whole MFMA K steps");
    static_assert(LDS <= 80 * 1024, "two workgroups per CU");
};

// What a workgroup does with finished accumulators (all of K of one example): squared norm of
// its 64 x 64 x 9 block and the optional store in the framework's [Cout, Cin, 3, 3] order.
//
// In the accumulator layout a lane holds, per tap, one input channel and sixteen output channels,
// so a direct store writes 4 bytes every 36.  When the layer's channel counts allow it the block
// goes through LDS instead (`lds`, free once the MFMAs are done): each wave lays down eight
// output-channel rows of 32 ci x 9 taps = 288 consecutive floats of the gradient, and reads them
// back as 16-byte pieces that leave as fully coalesced 1152-byte row segments.
__device__ __forceinline__ void c3_epilogue(const f32x16 (&acc)[9], const C3Args &a, int i, int unit, int co0, int ci0,
                                            int wm, int wn, int lane, float *red, char *lds)
{
    float ss = 0.0f;
    const bool store = a.out_w != nullptr;
    float *out = a.out_w + (size_t)i * a.out_stride;
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) ss += acc[t][r] * acc[t][r];     // channels beyond the layer are exact zeros
    // wave-uniform: whole 32-channel blocks, 16-byte aligned rows
    const bool via_lds = store && lds != nullptr && (a.cin % 32 == 0) && (a.out_stride % 4 == 0) &&
                         ((reinterpret_cast<uintptr_t>(a.out_w) & 15u) == 0);
    if (via_lds) {
        float *buf = reinterpret_cast<float *>(lds) + (threadIdx.x >> 6) * (8 * C3_RP);
        const int cil = lane & 31, half = lane >> 5;
        const int cib = ci0 + wn * 32;                                // first input channel of this wave
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            __syncthreads();                                          // previous pass read / MFMAs done with LDS
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int t = 0; t < 9; ++t) buf[(half * 4 + rr) * C3_RP + cil * 9 + t] = acc[t][q * 4 + rr];
            __syncthreads();
#pragma unroll
            for (int it = 0; it < 9; ++it) {
                const int f4 = it * 64 + lane;                        // 8 rows x 72 pieces
                const int row = f4 / 72, c4 = f4 - row * 72;
                const int co = co0 + wm * 32 + q * 8 + row;
                const float4 v = *reinterpret_cast<const float4 *>(buf + row * C3_RP + c4 * 4);
                if (co < a.cout && cib < a.cin)
                    *reinterpret_cast<float4 *>(out + ((size_t)co * a.cin + cib) * 9 + c4 * 4) = v;
            }
        }
    } else if (store) {
        const int ci = ci0 + wn * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = co0 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            const bool ok = co < a.cout && ci < a.cin;
            const size_t base = ((size_t)co * a.cin + ci) * 9;
#pragma unroll
            for (int t = 0; t < 9; ++t)
                if (ok) out[base + t] = acc[t][r];
        }
    }
    const float tot = block_sum<4>(ss, red);
    if (threadIdx.x == 0) a.partials[unit] = tot;
}

// Weighted sum of one tile over all examples: acc[co, ci, tap] += block, through LDS in the same
// coalesced row form as the store above when the shapes allow, else element by element.
__device__ __forceinline__ void c3_add_to_accumulator(const f32x16 (&acc)[9], const C3Args &a, int co0, int ci0,
                                                      int wm, int wn, int lane, char *lds)
{
    float *out = a.out_w;
    const bool via_lds = (a.cin % 32 == 0) && ((reinterpret_cast<uintptr_t>(a.out_w) & 15u) == 0);
    if (via_lds) {
        float *buf = reinterpret_cast<float *>(lds) + (threadIdx.x >> 6) * (8 * C3_RP);
        const int cil = lane & 31, half = lane >> 5;
        const int cib = ci0 + wn * 32;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            __syncthreads();
#pragma unroll
            for (int rr = 0; rr < 4; ++rr)
#pragma unroll
                for (int t = 0; t < 9; ++t) buf[(half * 4 + rr) * C3_RP + cil * 9 + t] = acc[t][q * 4 + rr];
            __syncthreads();
#pragma unroll
            for (int it = 0; it < 9; ++it) {
                const int f4 = it * 64 + lane;
                const int row = f4 / 72, c4 = f4 - row * 72;
                const int co = co0 + wm * 32 + q * 8 + row;
                const float4 v = *reinterpret_cast<const float4 *>(buf + row * C3_RP + c4 * 4);
                if (co < a.cout && cib < a.cin) {
                    float4 *dst = reinterpret_cast<float4 *>(out + ((size_t)co * a.cin + cib) * 9 + c4 * 4);
                    float4 o = *dst;
                    o.x += v.x; o.y += v.y; o.z += v.z; o.w += v.w;
                    *dst = o;
                }
            }
        }
    } else {
        const int ci = ci0 + wn * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int co = co0 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
            const bool ok = co < a.cout && ci < a.cin;
            const size_t base = ((size_t)co * a.cin + ci) * 9;
#pragma unroll
            for (int t = 0; t < 9; ++t)
                if (ok) out[base + t] += acc[t][r];
        }
    }
}

// MODE 0: one workgroup = all of K of one (example, tile); 1: a K slice of it (accumulators to the
// workspace); 2: clip-weighted sum over a range of examples for one tile (dY scaled by f_i while it
// is staged; added to the accumulator, or to the workspace when the examples are split into ranges).
enum { C3_FULL = 0, C3_SLICED = 1, C3_WEIGHTED = 2 };

// What one workgroup does; `bid` is its number within its layer.
template <int W, int MODE, int STRIDE>
__device__ __forceinline__ void conv3x3_body(const C3Args &a, const unsigned bid)
{
    constexpr bool WEIGHTED = MODE == C3_WEIGHTED;
    using C = C3Cfg<W, STRIDE>;
    constexpr int XB = 6;                             // X pieces per thread in flight at once
    extern __shared__ __attribute__((aligned(16))) char lds[];
    __shared__ float red[4];
    char *sX = lds, *sA = lds + 64 * C::PX;

    // consecutive hardware workgroup ids rotate over the 8 XCDs; give each XCD a run of
    // consecutive logical ids (the slices and tiles of the same examples share its L2)
    const int tiles = a.tiles_co * a.tiles_ci;
    const int total = (WEIGHTED ? 1 : a.n) * tiles * a.ksplit;
    const int per_xcd = (total + 7) >> 3;
    const int wg = (int)(bid & 7u) * per_xcd + (int)(bid >> 3);
    if (wg >= total) return;
    const int split = wg % a.ksplit;
    const int unit = wg / a.ksplit;                   // (example, tile); weighted: tile
    const int i_first = WEIGHTED ? split * a.ex_per_split : unit / tiles;
    const int i_last = WEIGHTED ? min(a.n, i_first + a.ex_per_split) : i_first + 1;
    const int tile = WEIGHTED ? unit : unit - i_first * tiles;
    const int tco = tile / a.tiles_ci, tci = tile - tco * a.tiles_ci;
    const int co0 = tco * 64, ci0 = tci * 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int H = a.h;

    // element offsets count from the start of the whole tensor (all n examples, below 2^31):
    // whole-dword windows (10 elements from an even element index) may reach into the
    // neighbouring example but never outside the tensor
    constexpr int XROW = (STRIDE == 1) ? W : C::WP;               // elements per row of the X tensor read here
    const int x_ex = a.cin * a.hin * XROW, dy_ex = a.cout * H * W;    // elements per example
    const int x_end = a.n * x_ex, dy_end = a.n * dy_ex;
    const uint32_t *xw = reinterpret_cast<const uint32_t *>(a.x);
    const uint32_t *dyw = reinterpret_cast<const uint32_t *>(a.dy);

    f32x16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

    const int c_begin = WEIGHTED ? 0 : split * a.chunks_per_split;
    const int c_end = WEIGHTED ? a.chunks : min(a.chunks, c_begin + a.chunks_per_split);

    for (int i = i_first; i < i_last; ++i) {
    const int x_base = i * x_ex, dy_base = i * dy_ex;
    float f = 1.0f;
    if constexpr (WEIGHTED) f = a.group_sqnorm ? clip_factor(a.group_sqnorm[i], a.clip_c) : 1.0f;
    for (int chunk = c_begin; chunk < c_end; ++chunk) {
        const int oh0 = chunk * C::R;
        if (chunk != c_begin || i != i_first) __syncthreads();    // everyone is done reading the previous chunk

        // ---- issue global loads, then shift / mask / write LDS.  The piece -> address decode is
        // recomputed per chunk on purpose (the opaque copy of the thread id stops the compiler
        // from keeping ~80 registers of loop-invariant addresses alive across the MFMA loop).
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        struct PieceA { int rel, lds_off, hi; bool valid, fast; };
        auto piece_a = [&](int u) {
            PieceA p;
            const int id = tid + C3_THREADS * u;
            const int co = id / (C::R * C::PPR), q = id - co * (C::R * C::PPR);
            const int r = q / C::PPR, pc = q - r * C::PPR;
            const int oh = oh0 + r;
            p.valid = (id < C::NPA) && (co0 + co < a.cout) && (oh < H);
            p.rel = dy_base + ((co0 + co) * H + oh) * W + pc * 8;
            p.lds_off = co * C::PA + (r * C::OWP + pc * 8) * 2;
            p.hi = W - pc * 8;                        // the row's end
            p.fast = p.valid && (p.rel & ~1) + 10 <= dy_end;
            return p;
        };
        struct PieceX { int rel, lds_off, lo, hi; bool valid, fast, write; };
        auto piece_x = [&](int u) {
            PieceX p;
            const int id = tid + C3_THREADS * u;
            const int ch = id / (C::XROWS * C::XPR), q = id - ch * (C::XROWS * C::XPR);
            const int xr = q / C::XPR, pc = q - xr * C::XPR;
            p.write = id < C::NPX;
            p.lds_off = ch * C::PX + (xr * C::WP + pc * 8) * 2;
            if constexpr (STRIDE == 1) {
                const int ih = oh0 - 1 + xr;
                const int iw0 = pc * 8 - 1;
                p.lo = (pc == 0) ? 1 : 0;
                p.hi = W - iw0;                           // may be <= 0: an all-zero piece
                p.valid = p.write && (ci0 + ch < a.cin) && (ih >= 0) && (ih < H) && (p.hi > p.lo);
                p.rel = x_base + ((ci0 + ch) * H + ih) * W + iw0;
                p.fast = p.valid && p.rel >= 0 && (p.rel & ~1) + 10 <= x_end;
            } else {
                // rows of the parity-split copy: whole aligned pieces, zeros already in place
                const int ih = 2 * oh0 - 1 + xr;
                p.lo = 0; p.hi = 8;
                p.valid = p.write && (ci0 + ch < a.cin) && (ih >= 0) && (ih < a.hin);
                p.rel = x_base + ((ci0 + ch) * a.hin + ih) * C::WP + pc * 8;
                p.fast = p.valid;
            }
            return p;
        };

        // dY first, then X in batches of at most XB pieces per thread: the loads of a batch are all
        // issued before the first is used, and a batch is small enough to sit in registers beside
        // the 144 accumulators
        {
            uint4 ra4[C::ALIGNED_A ? C::PA_T : 1];
            Raw<5> ra[C::ALIGNED_A ? 1 : C::PA_T];
#pragma unroll
            for (int u = 0; u < C::PA_T; ++u) {
                const PieceA p = piece_a(u);
                if constexpr (C::ALIGNED_A) ra4[u] = *reinterpret_cast<const uint4 *>(a.dy + (p.valid ? p.rel : 0));
                else ra[u] = piece_load_words(dyw + ((p.fast ? p.rel : 0) >> 1));
            }
#pragma unroll
            for (int u = 0; u < C::PA_T; ++u) {
                const PieceA p = piece_a(u);
                uint4 v;
                if constexpr (C::ALIGNED_A) {
                    v = p.valid ? ra4[u] : make_uint4(0u, 0u, 0u, 0u);
                } else {
                    uint32_t t[4];
                    piece_finish<true, 1>(t, ra[u], (uint32_t)(p.rel & 1), 0, p.fast ? p.hi : 0);
                    v = make_uint4(t[0], t[1], t[2], t[3]);
                }
                if constexpr (WEIGHTED) {
                    uint32_t t[4] = {v.x, v.y, v.z, v.w};
                    scale_regs<true, 4>(t, f);
                    v = make_uint4(t[0], t[1], t[2], t[3]);
                }
                if (C::NPA % C3_THREADS == 0 || tid + C3_THREADS * u < C::NPA)
                    *reinterpret_cast<uint4 *>(sA + p.lds_off) = v;
            }
        }
        if constexpr (STRIDE == 1) {
#pragma unroll
            for (int u0 = 0; u0 < C::PX_T; u0 += XB) {
                Raw<5> rx[XB];
#pragma unroll
                for (int u = 0; u < XB; ++u) {
                    if (u0 + u < C::PX_T) {
                        const PieceX p = piece_x(u0 + u);
                        rx[u] = piece_load_words(xw + ((p.fast ? p.rel : 0) >> 1));
                    }
                }
#pragma unroll
                for (int u = 0; u < XB; ++u) {
                    if (u0 + u >= C::PX_T) continue;
                    const PieceX p = piece_x(u0 + u);
                    uint32_t t[4];
                    piece_finish<true, 1>(t, rx[u], (uint32_t)(p.rel & 1), p.fast ? p.lo : 0, p.fast ? p.hi : 0);
                    const uint4 v = make_uint4(t[0], t[1], t[2], t[3]);
                    if (p.write) *reinterpret_cast<uint4 *>(sX + p.lds_off) = v;
                }
            }
        } else {
            constexpr int XB2 = 8;                    // aligned 16-byte copies: four registers per piece
#pragma unroll
            for (int u0 = 0; u0 < C::PX_T; u0 += XB2) {
                uint4 rx[XB2];
#pragma unroll
                for (int u = 0; u < XB2; ++u) {
                    if (u0 + u < C::PX_T) {
                        const PieceX p = piece_x(u0 + u);
                        rx[u] = *reinterpret_cast<const uint4 *>(a.x + (p.valid ? p.rel : 0));
                    }
                }
#pragma unroll
                for (int u = 0; u < XB2; ++u) {
                    if (u0 + u >= C::PX_T) continue;
                    const PieceX p = piece_x(u0 + u);
                    if (p.write) *reinterpret_cast<uint4 *>(sX + p.lds_off) = p.valid ? rx[u] : make_uint4(0u, 0u, 0u, 0u);
                }
            }
        }
        // Pieces whose whole-dword window would have left the tensor (only the first rows of the
        // first example and the last rows of the last one) were written as zeros above: fill them
        // in element by element, touching nothing but the valid elements.
        if (i == 0 || i == a.n - 1) {
            if constexpr (!C::ALIGNED_A) {
#pragma unroll 1
                for (int u = 0; u < C::PA_T; ++u) {
                    const PieceA p = piece_a(u);
                    if (p.valid && !p.fast) {
                        uint16_t *dst = reinterpret_cast<uint16_t *>(sA + p.lds_off);
                        const int hi = min(8, p.hi);
#pragma unroll 1
                        for (int e = 0; e < hi; ++e) {
                            uint16_t val = a.dy[p.rel + e];
                            if constexpr (WEIGHTED) val = float_to_bf16_bits(bf16_bits_to_float(val) * f);
                            dst[e] = val;
                        }
                    }
                }
            }
#pragma unroll 1
            for (int u = 0; u < (STRIDE == 1 ? C::PX_T : 0); ++u) {
                const PieceX p = piece_x(u);
                if (p.valid && !p.fast) {
                    uint16_t *dst = reinterpret_cast<uint16_t *>(sX + p.lds_off);
                    const int hi = min(8, p.hi);
#pragma unroll 1
                    for (int e = p.lo; e < hi; ++e) dst[e] = a.x[p.rel + e];
                }
            }
        }
        __syncthreads();

        // ---- MFMAs of the chunk
        const char *pa = sA + (wm * 32 + (lane & 31)) * C::PA;
        const char *px = sX + (wn * 32 + (lane & 31)) * C::PX;
        const int half = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < C::KSTEPS; ++ks) {
            const int kk = ks * 16 + half * 8;
            const int r = kk / C::OWP, ow0 = kk - r * C::OWP;
            const bf16x8 va = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pa + kk * 2));
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) {
                const char *row = px + ((STRIDE * r + kh) * C::WP + ow0) * 2;
                const uint4 d = *reinterpret_cast<const uint4 *>(row);
                const uint32_t d4 = *reinterpret_cast<const uint32_t *>(row + 16);
                const uint4 sh = make_uint4(funnel(d.y, d.x, 16), funnel(d.z, d.y, 16), funnel(d.w, d.z, 16),
                                            funnel(d4, d.w, 16));                 // the same run one element on
                uint4 b0, b1, b2;
                if constexpr (STRIDE == 1) {
                    b0 = d; b1 = sh; b2 = make_uint4(d.y, d.z, d.w, d4);
                } else {
                    b0 = d;                                                          // O'[ow]     = X[2 ow - 1]
                    b1 = *reinterpret_cast<const uint4 *>(row + C::E_OFF * 2);       // E[ow]      = X[2 ow]
                    b2 = sh;                                                         // O'[ow + 1] = X[2 ow + 1]
                }
                acc[kh * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, __builtin_bit_cast(bf16x8, b0), acc[kh * 3 + 0], 0, 0, 0);
                acc[kh * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, __builtin_bit_cast(bf16x8, b1), acc[kh * 3 + 1], 0, 0, 0);
                acc[kh * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, __builtin_bit_cast(bf16x8, b2), acc[kh * 3 + 2], 0, 0, 0);
            }
        }
    }
    }   // examples

    if constexpr (MODE == C3_FULL) {
        c3_epilogue(acc, a, i_first, unit, co0, ci0, wm, wn, lane, red, lds);
    } else if (WEIGHTED && a.ksplit == 1 && !a.unit_major) {
        c3_add_to_accumulator(acc, a, co0, ci0, wm, wn, lane, lds);
    } else {
        const size_t slot = (WEIGHTED && a.unit_major) ? (size_t)split * tiles + tile : (size_t)unit * a.ksplit + split;
        float *mine = a.ws_part + slot * (9 * 16 * C3_THREADS);
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[(t * 16 + r) * C3_THREADS + threadIdx.x] = acc[t][r];
    }
}

template <int W, int MODE, int STRIDE>
__global__ void __launch_bounds__(C3_THREADS, 2) conv3x3_kernel(const Grouped<C3Args> grp)
{
    unsigned bid;
    const C3Args &a = grp.a[group_pick(grp, bid)];
    conv3x3_body<W, MODE, STRIDE>(a, bid);
}

// The variants a ResNet of 224 x 224 images needs, in ONE kernel that dispatches on the layer's variant, so that all
// 3x3 layers of a batch call share a launch: at most four kernels run at a time on the chip, and the few workgroups of
// a narrow layer cost none of those four when they sit inside a wide launch.  Two sets (a body that is not needed is
// not compiled in: registers and LDS are those of the largest body of a set, and the finely sliced 56-wide body
// spills a few registers): set 0 for micro-steps of one or two examples (sliced variants: every launch is a few dozen
// workgroups and costs more than its work), set 1 for larger micro-steps (unsliced and clip-weighted variants).
enum { C3_ANY_56_SLICED = 0, C3_ANY_28_SLICED, C3_ANY_28_FULL, C3_ANY_14_FULL, C3_ANY_14_SLICED, C3_ANY_7_FULL,
       C3_ANY_14S2_SLICED, C3_ANY_14S2_FULL, C3_ANY_7S2_FULL, C3_ANY_56_FULL, C3_ANY_28_WEIGHTED, C3_ANY_14_WEIGHTED,
       C3_ANY_7_WEIGHTED, C3_ANY_28S2_FULL, C3_ANY_28S2_SLICED, C3_ANY_COUNT };

constexpr bool c3_any_in_set(int variant, int set)
{
    if (variant < 0) return false;
    if (set == 0) return variant <= C3_ANY_7S2_FULL || variant >= C3_ANY_28S2_FULL;
    return variant != C3_ANY_56_SLICED;
}

template <int SET>
__global__ void __launch_bounds__(C3_THREADS, 2) conv3x3_any_kernel(const Grouped<C3Args> grp)
{
    unsigned bid;
    const C3Args &a = grp.a[group_pick(grp, bid)];
    const int v = __builtin_amdgcn_readfirstlane(a.variant);
#define C3_ANY_CASE(ID, W, MODE, STRIDE)                                                  \
    if constexpr (c3_any_in_set(ID, SET)) {                                               \
        if (v == ID) { conv3x3_body<W, MODE, STRIDE>(a, bid); return; }                   \
    }
    C3_ANY_CASE(C3_ANY_56_SLICED, 56, C3_SLICED, 1)
    C3_ANY_CASE(C3_ANY_28_SLICED, 28, C3_SLICED, 1)
    C3_ANY_CASE(C3_ANY_28_FULL, 28, C3_FULL, 1)
    C3_ANY_CASE(C3_ANY_14_FULL, 14, C3_FULL, 1)
    C3_ANY_CASE(C3_ANY_14_SLICED, 14, C3_SLICED, 1)
    C3_ANY_CASE(C3_ANY_7_FULL, 7, C3_FULL, 1)
    C3_ANY_CASE(C3_ANY_14S2_SLICED, 14, C3_SLICED, 2)
    C3_ANY_CASE(C3_ANY_14S2_FULL, 14, C3_FULL, 2)
    C3_ANY_CASE(C3_ANY_7S2_FULL, 7, C3_FULL, 2)
    C3_ANY_CASE(C3_ANY_56_FULL, 56, C3_FULL, 1)
    C3_ANY_CASE(C3_ANY_28_WEIGHTED, 28, C3_WEIGHTED, 1)
    C3_ANY_CASE(C3_ANY_14_WEIGHTED, 14, C3_WEIGHTED, 1)
    C3_ANY_CASE(C3_ANY_7_WEIGHTED, 7, C3_WEIGHTED, 1)
    C3_ANY_CASE(C3_ANY_28S2_FULL, 28, C3_FULL, 2)
    C3_ANY_CASE(C3_ANY_28S2_SLICED, 28, C3_SLICED, 2)
#undef C3_ANY_CASE
}

constexpr int c3_max(int a, int b) { return a > b ? a : b; }
constexpr int C3_ANY_LDS = c3_max(c3_max(c3_max(C3Cfg<56, 1>::LDS, C3Cfg<28, 1>::LDS), c3_max(C3Cfg<14, 1>::LDS, C3Cfg<7, 1>::LDS)),
                                  c3_max(C3Cfg<28, 2>::LDS, c3_max(C3Cfg<14, 2>::LDS, C3Cfg<7, 2>::LDS)));

template <int W, int MODE, int STRIDE> constexpr int c3_any_variant()
{
    if (STRIDE == 1) {
        if (W == 56) return MODE == C3_SLICED ? C3_ANY_56_SLICED : (MODE == C3_FULL ? C3_ANY_56_FULL : -1);
        if (W == 28) return MODE == C3_SLICED ? C3_ANY_28_SLICED : (MODE == C3_FULL ? C3_ANY_28_FULL : C3_ANY_28_WEIGHTED);
        if (W == 14) return MODE == C3_SLICED ? C3_ANY_14_SLICED : (MODE == C3_FULL ? C3_ANY_14_FULL : C3_ANY_14_WEIGHTED);
        if (W == 7) return MODE == C3_FULL ? C3_ANY_7_FULL : (MODE == C3_WEIGHTED ? C3_ANY_7_WEIGHTED : -1);
        return -1;
    }
    if (W == 14) return MODE == C3_SLICED ? C3_ANY_14S2_SLICED : (MODE == C3_FULL ? C3_ANY_14S2_FULL : -1);
    if (W == 28) return MODE == C3_SLICED ? C3_ANY_28S2_SLICED : (MODE == C3_FULL ? C3_ANY_28S2_FULL : -1);
    if (W == 7 && MODE == C3_FULL) return C3_ANY_7S2_FULL;
    return -1;
}

// Parity split of the rows of X for the stride-2 kernel: out[row][0 .. OWP+8) = O'[c] = X[row][2c - 1],
// out[row][OWP+8 .. 2 OWP+8) = E[c] = X[row][2c]; zero where the column is outside the row.  `rows` =
// n * cin * hin rows of `win` (even) elements; one thread per 16-byte output piece, which needs
// the high (O') or low (E) halves of eight consecutive dwords of the input row.
struct DeintArgs {
    const uint16_t *x;
    uint16_t *out;
    long long rows;
    int win, owp;
};

__global__ void __launch_bounds__(256) deinterleave2_kernel(const Grouped<DeintArgs> grp)
{
    unsigned bid;
    const DeintArgs &a = grp.a[group_pick(grp, bid)];
    const uint16_t *__restrict__ x = a.x;
    uint16_t *__restrict__ out = a.out;
    const long long rows = a.rows;
    const int win = a.win, owp = a.owp;
    const int xpr = (2 * owp + 8) / 8, opr = (owp + 8) / 8;
    const long long q = (long long)bid * 256 + threadIdx.x;
    if (q >= rows * xpr) return;
    const long long row = q / xpr;
    const int pc = (int)(q - row * xpr);
    const bool odd_plane = pc < opr;
    const int first = odd_plane ? 8 * pc - 1 : 8 * (pc - opr);      // dword of element 0 of the piece
    const uint32_t *src = reinterpret_cast<const uint32_t *>(x + (size_t)row * win);
    const int nd = win / 2;
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int d = first + e;
        const uint32_t w = (d >= 0 && d < nd) ? src[d] : 0u;
        h[e] = odd_plane ? (w >> 16) : (w & 0xFFFFu);
    }
    *reinterpret_cast<uint4 *>(out + q * 8) =
        make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

// Slices of one (example, tile) meet here.  The sum is elementwise, so it is spread over many
// small workgroups: one per (example, tile, tap t, four of the tap's sixteen accumulator
// registers); each thread adds its four values in slice order with eight slices in flight, then
// squares / stores them like the unsliced epilogue.
constexpr int C3_FIX_R = 4, C3_FIX_PARTS = 16 / C3_FIX_R;

template <bool WEIGHTED>
__global__ void __launch_bounds__(C3_THREADS) conv3x3_fixup_kernel(const Grouped<C3Args> grp)
{
    __shared__ float red[4];
    unsigned bid;
    const C3Args &a = grp.a[group_pick(grp, bid)];
    const int tiles = a.tiles_co * a.tiles_ci;
    const int part = bid % C3_FIX_PARTS;
    const int t = (bid / C3_FIX_PARTS) % 9;
    const int unit = bid / (C3_FIX_PARTS * 9);                    // (example, tile); weighted: tile
    const int i = WEIGHTED ? 0 : unit / tiles, tile = unit - i * tiles;
    const int tco = tile / a.tiles_ci, tci = tile - tco * a.tiles_ci;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const size_t slice = (size_t)9 * 16 * C3_THREADS;
    const float *base = a.ws_part + (size_t)unit * a.ksplit * slice + (size_t)(t * 16 + part * C3_FIX_R) * C3_THREADS + threadIdx.x;
    float v[C3_FIX_R];
#pragma unroll
    for (int r = 0; r < C3_FIX_R; ++r) v[r] = 0.0f;
    int s = 0;
    for (; s + 8 <= a.ksplit; s += 8) {
        float tmp[8][C3_FIX_R];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < C3_FIX_R; ++r) tmp[u][r] = base[(size_t)(s + u) * slice + r * C3_THREADS];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < C3_FIX_R; ++r) v[r] += tmp[u][r];
    }
    for (; s < a.ksplit; ++s) {
        float tmp[C3_FIX_R];
#pragma unroll
        for (int r = 0; r < C3_FIX_R; ++r) tmp[r] = base[(size_t)s * slice + r * C3_THREADS];
#pragma unroll
        for (int r = 0; r < C3_FIX_R; ++r) v[r] += tmp[r];
    }
    const int ci = tci * 64 + wn * 32 + (lane & 31);
    float *out = WEIGHTED ? a.out_w : a.out_w + (size_t)i * a.out_stride;
    float ss = 0.0f;
#pragma unroll
    for (int rr = 0; rr < C3_FIX_R; ++rr) {
        const int r = part * C3_FIX_R + rr;
        const int co = tco * 64 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const bool ok = co < a.cout && ci < a.cin;
        const size_t idx = ((size_t)co * a.cin + ci) * 9 + t;
        if constexpr (WEIGHTED) {
            if (ok) out[idx] += v[rr];
        } else {
            ss += v[rr] * v[rr];
            if (a.out_w && ok) out[idx] = v[rr];
        }
    }
    if constexpr (!WEIGHTED) {
        const float tot = block_sum<4>(ss, red);
        if (threadIdx.x == 0) a.partials[bid] = tot;
    }
}

// ------------------------------------------------------------------------------------ host

struct C3Plan {
    int rows;           // R of the width case
    int tiles_co, tiles_ci, chunks;
    int ksplit, chunks_per_split;      // per-example modes: K slices; weighted: example ranges
    int ex_per_split;                  // weighted
};

int rows_of_width(int ow, int stride)
{
    const int owp = (ow + 7) / 8 * 8;
    if (stride == 2) return owp == 16 ? 5 : (owp == 32 ? 3 : 8);
    return owp == 8 ? 8 : 224 / owp;
}

// bytes of the parity-split copy of X the stride-2 kernel reads (0 for stride 1)
size_t c3_split_bytes(const Geo &g)
{
    if (g.stride != 2) return 0;
    const int owp = (g.ow + 7) / 8 * 8;
    return (size_t)g.n * g.cin * g.h * (2 * owp + 8) * sizeof(uint16_t);
}

// plans inside a batch call (the launch is shared with other layers) differ; workspace sizes cover both
thread_local int c3_forced_crowd = -1;
int c3_plan_crowd() { return c3_forced_crowd >= 0 ? c3_forced_crowd : crowd_hint(); }

C3Plan c3_plan(const Geo &g, int mode)
{
    C3Plan p;
    p.rows = rows_of_width(g.ow, g.stride);
    p.tiles_co = (g.cout + 63) / 64;
    p.tiles_ci = (g.cin + 63) / 64;
    p.chunks = (g.oh + p.rows - 1) / p.rows;
    p.ksplit = 1;
    p.chunks_per_split = p.chunks;
    p.ex_per_split = g.n;
    const long long tiles = (long long)p.tiles_co * p.tiles_ci;
    // inside a batch call: chunks per workgroup to plan for (a chunk here is about eight 128x128x64 chunks of work, but
    // slices cost a second pass over partial blocks: only very long walks are cut)
    int crowd = c3_plan_crowd(), tgt = crowd ? (crowd / 2 > 1 ? crowd / 2 : 1) : 0;
    // a layer that is small even chunk by chunk (micro-steps of one or two examples): a chunk per workgroup, the
    // walk of a workgroup is what such a launch waits for
    if (crowd && mode != MODE_WEIGHTED && (long long)g.n * tiles * p.chunks <= 128) tgt = 1;
    if (mode == MODE_WEIGHTED) {
        // example ranges: about 256 workgroups, partial blocks in the workspace kept below ~100 MB; in a launch
        // shared with other layers, ranges of at most 48 chunks
        long long want = (256 + tiles - 1) / tiles;
        // (measured in the replayed step: one range -- no partial blocks, no slice-sum launch, a narrow launch that the
        // other streams overlap -- beats four ranges by 4 % of the whole step; a walk is still capped at 48 chunks)
        // and a layer of few tiles still brings 32 workgroups
        if (crowd) {
            want = ((long long)g.n * p.chunks + 47) / 48;
            if (want * tiles < 32) want = (32 + tiles - 1) / tiles;
        }
        const long long cap = (long long)(96.0e6 / (4.0 * 9 * 16 * C3_THREADS * (double)tiles));
        if (want > cap) want = cap;
        if (want > g.n) want = g.n;
        if (want < 1) want = 1;
        p.ex_per_split = (int)((g.n + want - 1) / want);
        p.ksplit = (g.n + p.ex_per_split - 1) / p.ex_per_split;
        return p;
    }
    const long long units = (long long)g.n * tiles;
    // (measured in the replayed step, where other streams fill the compute units a narrow launch leaves free: the 56-wide
    // layers run 14 chunks per workgroup unsliced rather than in three slices + a slice-sum launch)
    if (p.chunks > 1 && (crowd ? p.chunks > 3 * tgt : units < 128)) {
        long long want = (128 + units - 1) / units;
        if (crowd) want = (p.chunks + tgt - 1) / tgt;
        if (want > p.chunks) want = p.chunks;
        p.chunks_per_split = (int)((p.chunks + want - 1) / want);
        p.ksplit = (p.chunks + p.chunks_per_split - 1) / p.chunks_per_split;
    }
    return p;
}

size_t c3_align16(size_t b) { return (b + 15) & ~(size_t)15; }

// partial squared norms per (example, tile): one, or one per fixup workgroup when K is sliced
size_t c3_partials_per_unit(const C3Plan &p) { return p.ksplit > 1 ? 9 * C3_FIX_PARTS : 1; }

template <int W, int MODE, int STRIDE>
dp_status c3_launch_mode(const C3Args &a, unsigned blocks, hipStream_t s)
{
    using C = C3Cfg<W, STRIDE>;
    constexpr int any = c3_any_variant<W, MODE, STRIDE>();
    const int set = fuse_hint() == 2 ? 0 : 1;
    if (fuse_hint() && (set == 0 ? c3_any_in_set(any, 0) : c3_any_in_set(any, 1))) {
        // inside a batch call: every row width in one launch
        const void *fn = set == 0 ? reinterpret_cast<const void *>(&conv3x3_any_kernel<0>)
                                  : reinterpret_cast<const void *>(&conv3x3_any_kernel<1>);
        static std::atomic<bool> any_attr_done[2];
        if (!any_attr_done[set].load()) {
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, C3_ANY_LDS) != hipSuccess)
                return fail(DP_ERR_DEVICE, "conv3x3: cannot reserve %d bytes of LDS", C3_ANY_LDS);
            any_attr_done[set].store(true);
        }
        C3Args b = a;
        b.variant = any;
        return submit_main<C3Args>(fn, b, blocks, C3_THREADS, C3_ANY_LDS, s, "conv3x3");
    }
    const void *fn = reinterpret_cast<const void *>(&conv3x3_kernel<W, MODE, STRIDE>);
    static std::atomic<bool> attr_done;              // zero-initialised; setting the attribute twice is harmless
    if (!attr_done.load()) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS) != hipSuccess)
            return fail(DP_ERR_DEVICE, "conv3x3: cannot reserve %d bytes of LDS", C::LDS);
        attr_done.store(true);
    }
    return submit_main<C3Args>(fn, a, blocks, C3_THREADS, C::LDS, s, "conv3x3");
}

template <int W, int STRIDE>
dp_status c3_launch_w(const C3Args &a, bool weighted, unsigned blocks, hipStream_t s)
{
    if constexpr (STRIDE == 1) {
        if (weighted) return c3_launch_mode<W, C3_WEIGHTED, STRIDE>(a, blocks, s);
    }
    if (a.ksplit > 1) return c3_launch_mode<W, C3_SLICED, STRIDE>(a, blocks, s);
    return c3_launch_mode<W, C3_FULL, STRIDE>(a, blocks, s);
}

}  // namespace

void c3_set_forced_crowd(int v) { c3_forced_crowd = v; }

bool conv3x3_applicable(const Geo &g, int mode)
{
    if (!g.bf16 || g.has_bias) return false;
    if (g.kh != 3 || g.kw != 3 || g.pad != 1) return false;
    if (g.cin < 64 || g.cout < 64) return false;
    if (g.stride == 1) {
        switch (g.w) {
        case 7: case 8: case 14: case 16: case 28: case 32: case 56: break;
        default: return false;
        }
    } else if (g.stride == 2) {
        // even images only (rows split by column parity, output exactly half the size)
        if (g.h % 2 || g.w % 2 || g.oh * 2 != g.h || g.ow * 2 != g.w) return false;
        // measured: worthwhile for the per-example calls on 14- and 7-wide outputs, and on 28-wide ones (chunks of
        // three rows) once a micro-step holds more than two examples: the layer then rides in the launch of the other
        // 3x3 layers (+ 0.4 % for the step; - 0.9 % with one example per micro-step); the clip-weighted form does
        // better in the general kernel / on packed operands
        if (mode == MODE_WEIGHTED || (g.ow != 7 && g.ow != 14 && g.ow != 28)) return false;
        if (g.ow == 28 && g.n <= 2) return false;
        if ((long long)g.n * g.cin * g.h * (2 * ((g.ow + 7) / 8 * 8) + 8) >= (1ll << 31)) return false;
    } else {
        return false;
    }
    // 32-bit element offsets inside the whole tensor
    return (long long)g.n * g.cin * g.h * g.w < (1ll << 31) && (long long)g.n * g.cout * g.h * g.w < (1ll << 31);
}

static size_t conv3x3_ws_bytes_plan(const Geo &g, int mode);

size_t conv3x3_ws_bytes(const Geo &g, int mode)
{
    const int saved = c3_forced_crowd;
    c3_forced_crowd = 0;
    const size_t alone = conv3x3_ws_bytes_plan(g, mode);
    c3_forced_crowd = 4;                             // smallest target: most slices
    const size_t shared = conv3x3_ws_bytes_plan(g, mode);
    c3_forced_crowd = saved;
    return alone > shared ? alone : shared;
}

static size_t conv3x3_ws_bytes_plan(const Geo &g, int mode)
{
    const C3Plan p = c3_plan(g, mode);
    const size_t tiles = (size_t)p.tiles_co * p.tiles_ci;
    const size_t split = c3_align16(c3_split_bytes(g));
    if (mode == MODE_WEIGHTED) return split + (p.ksplit > 1 ? tiles * p.ksplit * 9 * 16 * C3_THREADS * sizeof(float) : 0);
    const size_t units = (size_t)g.n * tiles;
    size_t b = c3_align16(units * c3_partials_per_unit(p) * sizeof(float));
    if (p.ksplit > 1) b += units * p.ksplit * 9 * 16 * C3_THREADS * sizeof(float);
    return b + split;
}

size_t conv3x3_norm_partial_count(const Geo &g)
{
    const C3Plan p = c3_plan(g, MODE_NORM);
    return (size_t)p.tiles_co * p.tiles_ci * c3_partials_per_unit(p);
}

const char *conv3x3_variant_name(const Geo &g, int mode)
{
    static const int widths[7] = {7, 8, 14, 16, 28, 32, 56};
    struct Names {
        char v[2][2][7][56];
        Names()
        {
            for (int st = 0; st < 2; ++st)
                for (int wt = 0; wt < 2; ++wt)
                    for (int k = 0; k < 7; ++k)
                        snprintf(v[st][wt][k], 56, "conv3x3_rows<bf16,w%d%s,%s>", widths[k], st ? ",s2" : "",
                                 wt ? "weighted" : "per_example");
        }
    };
    static const Names names;               // initialised once, thread-safe
    int slot = 6;
    for (int k = 0; k < 7; ++k)
        if (widths[k] == g.ow) slot = k;
    return names.v[g.stride == 2 ? 1 : 0][mode == MODE_WEIGHTED ? 1 : 0][slot];
}

// workspace of a call with clipping units: [units, tiles, 36] partial norms, then one accumulator block per (unit, tile)
size_t conv3x3_unit_ws_bytes(const Geo &g, int unit)
{
    const size_t tiles = (size_t)((g.cout + 63) / 64) * ((g.cin + 63) / 64), units = (size_t)(g.n / unit);
    return c3_align16(units * tiles * 9 * C3_FIX_PARTS * sizeof(float)) + units * tiles * 9 * 16 * C3_THREADS * sizeof(float);
}

size_t conv3x3_unit_norm_partial_count(const Geo &g)
{
    return (size_t)((g.cout + 63) / 64) * ((g.cin + 63) / 64) * 9 * C3_FIX_PARTS;
}

dp_status launch_conv3x3(const Geo &g, int mode, const void *x, const void *dy, float *out_w, size_t out_stride,
                         float *sqnorm, const float *group_sqnorm, float clip_c, void *ws, hipStream_t s, int unit)
{
    // unit > 0 (stride 1 only): sums over clipping units.  The clip-weighted kernel runs with factor 1 and one
    // example range per unit; the per-example slice-sum kernel then finishes every unit's block like an example's.
    const bool weighted = mode == MODE_WEIGHTED || unit > 0;
    C3Plan p = c3_plan(g, weighted ? MODE_WEIGHTED : mode);
    if (unit) { p.ex_per_split = unit; p.ksplit = g.n / unit; }
    C3Args a;
    a.variant = -1;
    a.unit_major = unit ? 1 : 0;
    a.x = static_cast<const uint16_t *>(x);
    a.dy = static_cast<const uint16_t *>(dy);
    a.out_w = out_w;
    a.out_stride = out_stride ? out_stride : g.pw;
    a.group_sqnorm = group_sqnorm; a.clip_c = clip_c;
    a.n = g.n; a.cin = g.cin; a.cout = g.cout; a.h = g.oh; a.hin = g.h;
    a.tiles_co = p.tiles_co; a.tiles_ci = p.tiles_ci;
    a.chunks = p.chunks; a.ksplit = p.ksplit; a.chunks_per_split = p.chunks_per_split;
    a.ex_per_split = p.ex_per_split;
    const size_t tiles = (size_t)p.tiles_co * p.tiles_ci;
    const size_t units = weighted ? tiles : (size_t)g.n * tiles;
    char *w = static_cast<char *>(ws);
    a.partials = nullptr;
    if (!weighted) {
        a.partials = reinterpret_cast<float *>(w);
        w += c3_align16(units * c3_partials_per_unit(p) * sizeof(float));
    } else if (unit) {
        a.partials = reinterpret_cast<float *>(w);
        w += c3_align16((size_t)(g.n / unit) * tiles * 9 * C3_FIX_PARTS * sizeof(float));
    }
    a.ws_part = (p.ksplit > 1 || unit) ? reinterpret_cast<float *>(w) : nullptr;
    if (p.ksplit > 1 || unit) w += units * p.ksplit * 9 * 16 * C3_THREADS * sizeof(float);
    const long long total = (long long)units * p.ksplit;
    const unsigned blocks = (unsigned)(((total + 7) / 8) * 8);
    dp_status st;
    if (g.stride == 2) {
        // rows of X split by column parity, after everything else in the workspace
        const int owp = (g.ow + 7) / 8 * 8;
        const long long rows = (long long)g.n * g.cin * g.h;
        const long long pieces = rows * ((2 * owp + 8) / 8);
        DeintArgs da;
        da.x = a.x; da.out = reinterpret_cast<uint16_t *>(w); da.rows = rows; da.win = g.w; da.owp = owp;
        st = submit_kernel<DeintArgs>(TIER_PRE, reinterpret_cast<const void *>(&deinterleave2_kernel), da,
                                      (unsigned)((pieces + 255) / 256), 256, 0, s, "deinterleave2");
        if (st != DP_OK) return st;
        a.x = reinterpret_cast<const uint16_t *>(w);
    }
    if (g.stride == 2) {
        if (g.ow == 7) st = c3_launch_w<7, 2>(a, weighted, blocks, s);
        else if (g.ow == 28) st = c3_launch_w<28, 2>(a, weighted, blocks, s);
        else st = c3_launch_w<14, 2>(a, weighted, blocks, s);
    } else {
        switch (g.w) {
        case 7: st = c3_launch_w<7, 1>(a, weighted, blocks, s); break;
        case 8: st = c3_launch_w<8, 1>(a, weighted, blocks, s); break;
        case 14: st = c3_launch_w<14, 1>(a, weighted, blocks, s); break;
        case 16: st = c3_launch_w<16, 1>(a, weighted, blocks, s); break;
        case 28: st = c3_launch_w<28, 1>(a, weighted, blocks, s); break;
        case 32: st = c3_launch_w<32, 1>(a, weighted, blocks, s); break;
        default: st = c3_launch_w<56, 1>(a, weighted, blocks, s); break;
        }
    }
    if (st != DP_OK) return st;
    // what follows the main kernel: at once, or after the grouped launch of a batch call
    if (unit) {
        C3Args u = a;
        u.n = g.n / unit; u.ksplit = 1;
        const size_t per_unit = tiles * 9 * C3_FIX_PARTS;
        st = submit_kernel<C3Args>(TIER_POST, reinterpret_cast<const void *>(&conv3x3_fixup_kernel<false>), u,
                                   (unsigned)((size_t)u.n * per_unit), C3_THREADS, 0, s, "conv3x3_fixup");
        if (st != DP_OK || !sqnorm) return st;
        const float *partials = a.partials;
        const int n_units = u.n, per = (int)per_unit;
        return submit_post([=]() -> dp_status { return launch_sum_partials(partials, n_units, per, sqnorm, s); });
    }
    if (p.ksplit > 1) {
        const unsigned fix_blocks = (unsigned)(units * 9 * C3_FIX_PARTS);
        const void *fix = weighted ? reinterpret_cast<const void *>(&conv3x3_fixup_kernel<true>)
                                   : reinterpret_cast<const void *>(&conv3x3_fixup_kernel<false>);
        st = submit_kernel<C3Args>(TIER_POST, fix, a, fix_blocks, C3_THREADS, 0, s, "conv3x3_fixup");
        if (st != DP_OK) return st;
    }
    if (weighted || !sqnorm) return DP_OK;
    const int n = g.n, per_example = p.tiles_co * p.tiles_ci * (int)c3_partials_per_unit(p);
    const float *partials = a.partials;
    return submit_post([=]() -> dp_status { return launch_sum_partials(partials, n, per_example, sqnorm, s); });
}

}  // namespace dp
