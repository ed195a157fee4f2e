// Per-example conv weight gradients as batched implicit-GEMM contractions on MFMA (gfx950).
//
// GEMM view of one example i of one conv layer (H1 of the path):
//     D_i[m, j] = sum_k A_i[m, k] * B_i[j, k]
//     m = output channel (Cout rows), j = (ci, kh, kw) flattened (J = Cin*KH*KW columns, the
//     framework's [Cout, Cin, KH, KW] weight layout read as a Cout x J matrix),
//     k = output position (oh, ow), the contraction,
//     A_i[m, k] = dY_i[m, oh, ow]                      -- contiguous along ow in NCHW
//     B_i[j, k] = Xpad_i[ci, oh*s+kh-p, ow*s+kw-p]     -- zero outside the image.
//
// K is laid out "row padded": k' = oh * OWp + ow with OWp = OW rounded up to the 16-byte
// piece (8 bf16 / 4 fp32), so that a piece never straddles two image rows and every piece of
// either operand is a run of consecutive (or stride-2) elements of one row of one tensor.
// A 1x1 stride-1 conv is passed in as the degenerate geometry H = 1, W = S (one long row).
//
// One workgroup (4 waves) owns one MT x NT tile of D and walks chunks of 128 bytes of K per
// row.  Each thread stages 16-byte pieces: one dword-aligned 16-byte global load (+1 dword
// when the run starts on an odd bf16), a funnel shift, and an edge mask; stride-2 rows are
// de-interleaved in registers.  Pieces go to LDS with K contiguous (the operand order of
// v_mfma_f32_32x32x16_bf16 / v_mfma_f32_32x32x2_f32) and every wave runs its 32x32 MFMA
// tiles out of LDS while the next chunk's loads are in flight.
//
// What happens to a finished tile:
//   * per-example mode: its squares are summed in registers and reduced with wavefront
//     shuffles to one partial per (example, tile) -- the gradient is never re-read for the
//     norm -- and, if asked, the tile is stored (materialised per-example gradient).  A
//     workgroup may take several examples in a row (short K) so loads stream across example
//     boundaries, or a slice of one example's K (long K, few tiles); slices store their tiles
//     in a workspace and a second kernel adds them in slice order and runs the epilogue.
//   * weighted mode: K runs over (example, position) with dY_i scaled by the clip factor f_i
//     while it is staged, so the tile is sum_i f_i dW_i; example ranges meet the same way and
//     the sum is added to the accumulator.
// The bias gradient db_i[m] = sum_k dY_i[m, k] rides along as one more MFMA against a
// register of ones in the workgroups of tile column 0.
#include "internal.h"
#include "group.h"
#include "pieces.h"

#include <atomic>
#include <cstdio>
#include <type_traits>

namespace dp {

constexpr int THREADS = 256;
constexpr int PITCH = 144;            // bytes per LDS row: 128 data + 16 pad (odd multiple of 16 B:
                                      // 8 consecutive rows hit 8 distinct 16-byte bank groups)

struct ConvArgs {
    const void *x, *dy;
    float *out_w, *out_b;             // per-example: g_w / g_b (may be null); weighted: accumulators
    size_t out_stride_w, out_stride_b;  // per-example row stride
    float *partials;                  // per-example: [n, tiles] partial squared norms
    const float *group_sqnorm;        // weighted: [n]
    float clip_c;
    float *ws_part;                   // split partial tiles
    int n, cin, cout, h, w, kh, kw, stride, pad, oh, ow;
    int J, S;
    int tiles_m, tiles_n;
    int kcolsp;                       // OW rounded up to a piece
    int chunks_per_ex;                // ceil(OH * kcolsp / KC)
    int ksplit;                       // per-example: K slices per (example, tile); weighted: example ranges
    int chunks_per_split;             // per-example mode
    int ex_per_split;                 // weighted mode
    int ex_per_wg;                    // per-example mode, ksplit == 1: consecutive examples per workgroup
    int force_slow;                   // stride other than 1 or 2: stage every chunk element by element
    int unit_major;                   // weighted mode, > 0: clipping units, each made of unit_major example ranges; the
                                      // ranges' blocks always go to the workspace, ordered (unit, tile, range in unit)
};

struct ColInfo {
    int off;        // ci*H*W + (kh-p)*W + (kw-p)
    short dh, dw;   // kh-p, kw-p; dh = -30000 marks a column beyond J
};

// ceil(a / b) for b > 0 and any sign of a
__device__ __forceinline__ int ceil_div(int a, int b) { return (a >= 0) ? (a + b - 1) / b : -((-a) / b); }

// Epilogue of one finished tile held in the MFMA accumulator layout (full K of one example, or
// the weighted sum over examples): squared norm + optional store, or add into the accumulator.
//
// In the accumulator layout register r of a lane is row (r >> 2) * 8 + (r & 3) (+ 4 for the upper half
// of the wave) and column lane & 31 of a 32x32 block, so the address of a value is a wave-uniform part
// (example, block, r: scalar arithmetic) plus a per-lane byte offset that never changes.  Tiles that
// lie wholly inside the matrix -- all of them when the channel counts are multiples of the tile --
// take that path: one store per value and no per-value compares or branches.  Ragged tiles check every
// value (rows / columns beyond the matrix hold no gradient: neither stored nor counted in the norm).
// Global accesses whose address is a wave-uniform base (scalar register pair) plus a 32-bit per-lane byte
// offset: no vector address arithmetic at all.  `base` must be the same in every lane.
__device__ __forceinline__ unsigned long long uniform_bits(const void *p)
{
    const unsigned long long v = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ void store_f32_uniform_base(unsigned long long base, unsigned byte_off, float v)
{
    asm volatile("global_store_dword %0, %1, %2" ::"v"(byte_off), "v"(v), "s"(base) : "memory");
}
// the same store with the non-temporal hint: per-example gradients are written once and read back much later by the
// streaming accumulate, so they should not push the operands (re-read by the neighbouring tiles) out of L2
__device__ __forceinline__ void store_f32_uniform_base_nt(unsigned long long base, unsigned byte_off, float v)
{
    asm volatile("global_store_dword %0, %1, %2 nt" ::"v"(byte_off), "v"(v), "s"(base) : "memory");
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a constant expression
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>{});
    }
}
template <int AT>
__device__ __forceinline__ void store_f32_uniform_base_nt_at(unsigned long long base, unsigned byte_off, float v)
{
    static_assert(AT >= 0 && AT < 4096, "immediate offset of a global store");
    asm volatile("global_store_dword %0, %1, %2 offset:%3 nt" ::"v"(byte_off), "v"(v), "s"(base), "n"(AT) : "memory");
}
__device__ __forceinline__ float load_f32_uniform_base(unsigned long long base, unsigned byte_off)
{
    float v;
    asm volatile("global_load_dword %0, %1, %2" : "=v"(v) : "v"(byte_off), "s"(base) : "memory");
    return v;                               // valid only after wait_loaded()
}
// wait for every outstanding load; the values pass through so that no use can move above the wait
__device__ __forceinline__ void wait_loaded(float (&v)[16])
{
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]), "+v"(v[8]),
                   "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
                 :
                 : "memory");
}

// Per-example mode returns this thread's share of the tile's squared norm (the caller reduces it: every
// (example, tile) owns four partial-norm slots, one per wave).
// EXACT: the host only sends layers whose tiles are all whole (no ragged path, MT / NT below are not used).
template <int WAVES_N, int TM, int TN, bool WEIGHTED, bool BIAS, bool EXACT = false, int NACC>
__device__ __forceinline__ float tile_epilogue(const f32x16 (&acc)[NACC], const ConvArgs &a, int i, int m0, int n0, int wm,
                                               int wn, int lane, bool bias_here)
{
    constexpr int WAVES_M = 4 / WAVES_N;
    constexpr int MT = WAVES_M * TM * 32, NT = WAVES_N * TN * 32;
    const int cout = __builtin_amdgcn_readfirstlane(a.cout), J = __builtin_amdgcn_readfirstlane(a.J);
    m0 = __builtin_amdgcn_readfirstlane(m0);
    n0 = __builtin_amdgcn_readfirstlane(n0);
    const bool inside_tile = EXACT || (m0 + MT <= cout && n0 + NT <= J);            // uniform
    // per lane: row and column of register 0 of block (0, 0) of this wave
    const int m_lane = m0 + wm * TM * 32 + (lane >> 5) * 4, j_lane = n0 + wn * TN * 32 + (lane & 31);
    const unsigned lane_off = ((unsigned)(m_lane - m0) * (unsigned)J + (unsigned)(j_lane - n0)) * 4u;   // bytes from the tile's corner
    float ss = 0.0f;
    if constexpr (!WEIGHTED) {
        const bool store = a.out_w != nullptr;
        const unsigned long long corner = uniform_bits(a.out_w + (size_t)i * a.out_stride_w + (size_t)m0 * J + n0);
        if (inside_tile) {
#pragma unroll
            for (int t = 0; t < TM * TN; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) ss += acc[t][r] * acc[t][r];
            if (store) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            store_f32_uniform_base_nt(corner + 4ull * ((unsigned)(tm * 32 + (r >> 2) * 8 + (r & 3)) * (unsigned)J + (unsigned)(tn * 32)),
                                                      lane_off, acc[tm * TN + tn][r]);
            }
        } else {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int j = j_lane + tn * 32;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = acc[tm * TN + tn][r];
                        const int m = m_lane + tm * 32 + (r >> 2) * 8 + (r & 3);
                        const bool inside = m < cout && j < J;
                        ss += inside ? v * v : 0.0f;
                        if (store && inside) a.out_w[(size_t)i * a.out_stride_w + (size_t)m * J + j] = v;
                    }
                }
        }
        if constexpr (BIAS) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                if (bias_here && (lane & 31) == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = acc[TM * TN + tm][r];
                        const int m = m_lane + tm * 32 + (r >> 2) * 8 + (r & 3);
                        ss += m < cout ? v * v : 0.0f;
                        if (store && m < cout) a.out_b[(size_t)i * a.out_stride_b + m] = v;
                    }
                }
            }
        }
    } else {
        const unsigned long long corner = uniform_bits(a.out_w + (size_t)m0 * J + n0);
        if (inside_tile) {
            // all loads of a block first, then the adds and stores
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    float old[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        old[r] = load_f32_uniform_base(corner + 4ull * ((unsigned)(tm * 32 + (r >> 2) * 8 + (r & 3)) * (unsigned)J + (unsigned)(tn * 32)), lane_off);
                    wait_loaded(old);
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        store_f32_uniform_base(corner + 4ull * ((unsigned)(tm * 32 + (r >> 2) * 8 + (r & 3)) * (unsigned)J + (unsigned)(tn * 32)),
                                               lane_off, old[r] + acc[tm * TN + tn][r]);
                }
        } else {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int j = j_lane + tn * 32;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = m_lane + tm * 32 + (r >> 2) * 8 + (r & 3);
                        if (m < cout && j < J) a.out_w[(size_t)m * J + j] += acc[tm * TN + tn][r];
                    }
                }
        }
        if constexpr (BIAS) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                if (bias_here && (lane & 31) == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int m = m_lane + tm * 32 + (r >> 2) * 8 + (r & 3);
                        if (m < cout) a.out_b[m] += acc[TM * TN + tm][r];
                    }
                }
            }
        }
    }
    return ss;
}

// Workgroup tile MT x NT = (WAVES_M*TM*32) x (WAVES_N*TN*32), WAVES_M*WAVES_N = 4 waves.
// Element-by-element staging of one operand's chunk straight into LDS, touching only valid
// elements.  Used for the few chunks whose whole-dword reads could leave the tensor (first rows
// of the first example, last rows of the last example), for tensors too small to have slack, and
// for strides other than 1 and 2.  Compact on purpose: it is rarely taken.
template <bool BF16, int ROWS, bool WEIGHTED>
__device__ __noinline__ void slow_stage_a(char *lds, const typename ElemTraits<BF16>::type *dy_i, int cout, int S,
                                          int oh_n, int ow_n, int kcolsp, int m0, int k0, float f)
{
    struct { int cout, S, oh, ow, kcolsp; } a = {cout, S, oh_n, ow_n, kcolsp};
    typedef typename ElemTraits<BF16>::type E;
    constexpr int KC = ElemTraits<BF16>::KC;
    for (int idx = threadIdx.x; idx < ROWS * KC; idx += THREADS) {
        const int row = idx / KC, kk = idx - row * KC;
        const int kprime = k0 + kk;
        const int oh = kprime / a.kcolsp, ow = kprime - oh * a.kcolsp;
        const int m = m0 + row;
        E val = 0;
        if (m < a.cout && oh < a.oh && ow < a.ow) {
            val = dy_i[(size_t)m * a.S + (size_t)oh * a.ow + ow];
            if constexpr (WEIGHTED) {
                if constexpr (BF16) val = float_to_bf16_bits(bf16_bits_to_float(val) * f);
                else val = val * f;
            }
        }
        *reinterpret_cast<E *>(lds + row * PITCH + kk * (int)sizeof(E)) = val;
    }
}

template <bool BF16, int ROWS>
__device__ __noinline__ void slow_stage_b(char *lds, const typename ElemTraits<BF16>::type *x_i, const ColInfo *cols,
                                          int h, int w, int oh_n, int ow_n, int stride, int kcolsp, int k0)
{
    struct { int h, w, oh, ow, stride, kcolsp; } a = {h, w, oh_n, ow_n, stride, kcolsp};
    typedef typename ElemTraits<BF16>::type E;
    constexpr int KC = ElemTraits<BF16>::KC;
    for (int idx = threadIdx.x; idx < ROWS * KC; idx += THREADS) {
        const int row = idx / KC, kk = idx - row * KC;
        const int kprime = k0 + kk;
        const int oh = kprime / a.kcolsp, ow = kprime - oh * a.kcolsp;
        const ColInfo ci = cols[row];
        const int ih = oh * a.stride + ci.dh, iw = ow * a.stride + ci.dw;
        E val = 0;
        if (oh < a.oh && ow < a.ow && (unsigned)ih < (unsigned)a.h && (unsigned)iw < (unsigned)a.w)
            val = x_i[ci.off + oh * a.stride * a.w + ow * a.stride];
        *reinterpret_cast<E *>(lds + row * PITCH + kk * (int)sizeof(E)) = val;
    }
}

// LOADER 0: the geometry is one long row per channel whose length is a multiple of the piece
// (1x1 stride-1 conv with S % 8 == 0 for bf16): every piece is a single aligned 16-byte load.
// LOADER 1 / 2: general geometry with stride 1 / 2 (any other stride runs LOADER 1 with every
// chunk staged element by element).
template <bool BF16, int WAVES_M, int WAVES_N, int TM, int TN, bool WEIGHTED, bool BIAS, int LOADER>
__global__ void __launch_bounds__(THREADS, 2) conv_contract_kernel(const Grouped<ConvArgs> grp)
{
    unsigned bid;                                   // workgroup number within this workgroup's layer
    const ConvArgs &a = grp.a[group_pick(grp, bid)];
    typedef typename ElemTraits<BF16>::type E;
    constexpr int KC = ElemTraits<BF16>::KC;
    constexpr int EPP = ElemTraits<BF16>::EPP;
    constexpr int MT = WAVES_M * TM * 32, NT = WAVES_N * TN * 32;
    constexpr int PA = MT / 32, PB = NT / 32;           // 16-byte pieces per thread per chunk
    constexpr int NACC = TM * TN + (BIAS ? TM : 0);     // 32x32 accumulator tiles per wave
    static_assert(WAVES_M * WAVES_N == 4, "four waves");

    __shared__ __attribute__((aligned(16))) char sA[2 * MT * PITCH];     // two buffers each
    __shared__ __attribute__((aligned(16))) char sB[2 * NT * PITCH];
    __shared__ ColInfo cols[NT];
    __shared__ float red[4];

    // ---- which tile and which slice of work.  Consecutive hardware workgroup ids rotate over
    // the 8 XCDs, so id -> (id % 8) * per_xcd + id / 8 puts runs of consecutive logical ids
    // (the slices of one tile; the tiles of one example) behind one XCD's L2.
    const int tiles = a.tiles_m * a.tiles_n;
    int total, tile, unit;
    if constexpr (WEIGHTED) {
        total = tiles * a.ksplit;
    } else {
        const int ex_groups = (a.n + a.ex_per_wg - 1) / a.ex_per_wg;
        total = ex_groups * tiles * a.ksplit;
    }
    const int per_xcd = (total + 7) >> 3;
    const int wg = (int)(bid & 7u) * per_xcd + (int)(bid >> 3);
    if (wg >= total) return;
    int split;
    if constexpr (WEIGHTED) {
        tile = wg / a.ksplit;               // slices of one tile are neighbours
        split = wg - tile * a.ksplit;
        unit = 0;
    } else {
        split = wg % a.ksplit;
        const int r = wg / a.ksplit;
        unit = r / tiles;                   // example group
        tile = r - unit * tiles;
    }
    const int tile_m = tile / a.tiles_n, tile_n = tile - tile_m * a.tiles_n;
    const int m0 = tile_m * MT, n0 = tile_n * NT;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WAVES_N, wn = wave - wm * WAVES_N;

    if (threadIdx.x < NT) {
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

    // ---- the stream of chunks this workgroup walks
    int i_begin, i_end, c_begin, c_end;     // examples [i_begin, i_end), chunks [c_begin, c_end) of each
    if constexpr (WEIGHTED) {
        i_begin = split * a.ex_per_split;
        i_end = min(a.n, i_begin + a.ex_per_split);
        c_begin = 0;
        c_end = a.chunks_per_ex;
    } else {
        i_begin = unit * a.ex_per_wg;
        i_end = min(a.n, i_begin + a.ex_per_wg);
        c_begin = split * a.chunks_per_split;
        c_end = min(a.chunks_per_ex, c_begin + a.chunks_per_split);
    }
    const int cpe = c_end - c_begin;
    const int n_chunks = (i_end - i_begin) * cpe;

    const size_t x_ex = (size_t)a.cin * a.h * a.w, dy_ex = (size_t)a.cout * a.S;
    const E *xg = static_cast<const E *>(a.x), *dyg = static_cast<const E *>(a.dy);

    // per-thread constants of the staging map: piece c = tid + 256 q -> row c / 8, K-piece c % 8.
    // Everything that does not change from chunk to chunk is computed here, once.
    const int kp = (threadIdx.x & 7) * EPP;
    const int row0 = threadIdx.x >> 3;
    int a_row_off[PA];                       // (m0 + row) * S, or -1 beyond Cout
#pragma unroll
    for (int q = 0; q < PA; ++q) {
        const int m = m0 + row0 + 32 * q;
        a_row_off[q] = (m < a.cout) ? m * a.S : -1;
    }
    int b_off[PB], b_dhw[PB];                // B rows: element offset of the tap, packed (dh, dw)
#pragma unroll
    for (int q = 0; q < PB; ++q) {
        if constexpr (LOADER == 0) {
            const int j = n0 + row0 + 32 * q;
            b_off[q] = (j < a.J) ? j * a.S : -1;
            b_dhw[q] = 0;
        } else {
            const ColInfo ci = cols[row0 + 32 * q];
            b_off[q] = ci.off;
            b_dhw[q] = ((int)ci.dh << 16) | ((int)ci.dw & 0xFFFF);
        }
    }

    f32x16 acc[NACC];
#pragma unroll
    for (int t = 0; t < NACC; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    const bool bias_here = BIAS && tile_n == 0 && wn == 0;

    // Raw loaded dwords of a chunk in flight and, per piece, the packed (odd, lo, hi) needed to
    // finish it.  Two sets: while chunk c is in the MFMAs, chunk c+1 waits in one set and the
    // loads of chunk c+2 are issued into the other.
    constexpr int LS = (LOADER == 2) ? 2 : 1;
    constexpr int RA = (LOADER == 0) ? 4 : raw_n<BF16, 1>();
    constexpr int RB = (LOADER == 0) ? 4 : raw_n<BF16, LS>();
    constexpr int EPD = BF16 ? 2 : 1;                  // elements per dword
    struct RawSet {
        Raw<RA> ra[PA];
        Raw<RB> rb[PB];
        uint32_t ma[PA], mb[PB];
        int i, c;                            // example and chunk (within the example) held by this set
        int oh, ow0;                         // this thread's output position in that chunk (gather loaders)
    };
    RawSet set0, set1;

    // Whole-dword reads touch a few bytes around the elements they need.  That is harmless inside
    // the tensor (a neighbouring row or example) but the window of a piece must not leave it:
    //   LOADER 0: the partial last piece of a row is read from a window moved back to end with the
    //     row, and rotated down in registers;
    //   LOADER 1 / 2: a piece whose window would start before the first example or end after the
    //     last one is staged as zeros and then filled in element by element (a handful of pieces
    //     in the workgroups of the first and the last example).
    // Tensors too small to have slack, and strides other than 1 and 2, stage every chunk element
    // by element.
    const bool all_slow = a.force_slow || x_ex < 512 || dy_ex < 512 || a.S < EPP;
    constexpr uint32_t UNSAFE = 2u;          // bit 1 of a piece's meta word

    // Position of the next chunk to fetch: example, chunk within it, and this thread's (oh, ow0);
    // advanced incrementally (no division in the loop).
    int f_i = i_begin, f_c = c_begin;
    const int kprime0 = c_begin * KC + kp;
    const int oh0 = (LOADER == 0) ? 0 : kprime0 / a.kcolsp;
    const int ow00 = (LOADER == 0) ? kprime0 : kprime0 - oh0 * a.kcolsp;
    const int step_oh = (LOADER == 0) ? 0 : KC / a.kcolsp, step_ow = (LOADER == 0) ? KC : KC - step_oh * a.kcolsp;
    int f_oh = oh0, f_ow = ow00;

    // dword pointer and element parity of example i's first element (tensors are 16-byte aligned)
    auto ex_words = [&](const E *base, size_t ex_elems, int i, int &par) -> const uint32_t * {
        const size_t eb = (size_t)i * ex_elems;
        par = (int)(eb % EPD);
        return reinterpret_cast<const uint32_t *>(base) + eb / EPD;
    };

    // Issue every global load of the next chunk (no use of the data here, so no wait either).
    auto fetch = [&](RawSet &R) {
        const int i = f_i, c = f_c;
        R.i = i; R.c = c;
        if (!all_slow) {
            if constexpr (LOADER == 0) {
                // one long row per channel; a piece is 16 bytes at a dword-aligned address.  Only the
                // last piece of a row can be partial: its window is moved back by `back` elements
                const int kprime = f_ow;
                const int hi = min(EPP, a.S - kprime);
                const int back = (hi > 0 && hi < EPP) ? EPP - hi : 0;
                const uint32_t meta = (uint32_t)max(hi, 0) | ((uint32_t)back << 8);
                const E *pa_ = dyg + (size_t)i * dy_ex + (kprime - back);
#pragma unroll
                for (int q = 0; q < PA; ++q) {
                    u32x4_a4 v = {0u, 0u, 0u, 0u};
                    if (hi > 0 && a_row_off[q] >= 0) v = *reinterpret_cast<const u32x4_a4 *>(pa_ + a_row_off[q]);
                    R.ra[q].d[0] = v.x; R.ra[q].d[1] = v.y; R.ra[q].d[2] = v.z; R.ra[q].d[3] = v.w;
                    R.ma[q] = meta;
                }
                const E *pb_ = xg + (size_t)i * x_ex + (kprime - back);
#pragma unroll
                for (int q = 0; q < PB; ++q) {
                    u32x4_a4 v = {0u, 0u, 0u, 0u};
                    if (hi > 0 && b_off[q] >= 0) v = *reinterpret_cast<const u32x4_a4 *>(pb_ + b_off[q]);
                    R.rb[q].d[0] = v.x; R.rb[q].d[1] = v.y; R.rb[q].d[2] = v.z; R.rb[q].d[3] = v.w;
                    R.mb[q] = meta;
                }
            } else {
                const int oh = f_oh, ow0 = f_ow;
                R.oh = oh; R.ow0 = ow0;
                const bool k_ok = oh < a.oh;
                const bool first = (i == 0), last = (i == a.n - 1);
                {
                    // A: dY_i[m, oh, ow0 .. ow0+EPP)
                    int par;
                    const uint32_t *wa = ex_words(dyg, dy_ex, i, par);
                    const int koff = k_ok ? oh * a.ow + ow0 : 0;
                    const int hi_a = k_ok ? min(a.ow - ow0, EPP) : 0;
#pragma unroll
                    for (int q = 0; q < PA; ++q) {
                        const bool ok = a_row_off[q] >= 0 && hi_a > 0;
                        const int e = (ok ? a_row_off[q] + koff : 0) + par;          // relative to wa, in elements
                        const int ws = (e / EPD) * EPD - par, we = ws + RA * EPD;     // window, relative to the example
                        const bool safe = (!first || ws >= 0) && (!last || we <= (int)dy_ex);
                        const uint32_t *src = wa + (safe ? e / EPD : 0);
                        if constexpr (BF16) {
                            R.ra[q] = piece_load_words(src);
                        } else {
                            const u32x4_a4 v = *reinterpret_cast<const u32x4_a4 *>(src);
                            R.ra[q].d[0] = v.x; R.ra[q].d[1] = v.y; R.ra[q].d[2] = v.z; R.ra[q].d[3] = v.w;
                        }
                        R.ma[q] = (uint32_t)(e & (EPD - 1)) | ((ok && !safe) ? UNSAFE : 0u) | ((uint32_t)(ok ? hi_a : 0) << 16);
                    }
                }
                {
                    // B: X_i[ci, oh*s + dh, (ow0 + e)*s + dw]; only the image edge is masked here,
                    // positions past OW meet the zeros of A
                    int par;
                    const uint32_t *wb = ex_words(xg, x_ex, i, par);
                    const int ihs = oh * a.stride, iws = ow0 * a.stride;
                    const int koff = ihs * a.w + iws;
#pragma unroll
                    for (int q = 0; q < PB; ++q) {
                        const int ih = ihs + (b_dhw[q] >> 16);
                        const int first_col = iws + (int)(short)(b_dhw[q] & 0xFFFF);   // input column of e = 0
                        int lo, hi;
                        if constexpr (LOADER == 1) { lo = -first_col; hi = a.w - first_col; }
                        else { lo = (1 - first_col) >> 1; hi = (a.w - first_col + 1) >> 1; }   // ceil(-first/2), ceil((W-first)/2)
                        lo = min(max(lo, 0), EPP);
                        hi = min(max(hi, lo), EPP);
                        const bool ok = k_ok && (unsigned)ih < (unsigned)a.h && hi > lo;
                        const int e = (ok ? b_off[q] + koff : 0) + par;
                        // floor division: the first tap of the first row may start one element early
                        const int ed = (e >= 0) ? e / EPD : -((-e + EPD - 1) / EPD);
                        const int ws = ed * EPD - par, we = ws + RB * EPD;
                        const bool safe = (!first || ws >= 0) && (!last || we <= (int)x_ex);
                        const uint32_t *src = wb + (safe ? ed : 0);
                        if constexpr (BF16 && LS == 1) {
                            R.rb[q] = piece_load_words(src);
                        } else {
                            const u32x4_a4 v0 = *reinterpret_cast<const u32x4_a4 *>(src);
                            R.rb[q].d[0] = v0.x; R.rb[q].d[1] = v0.y; R.rb[q].d[2] = v0.z; R.rb[q].d[3] = v0.w;
                            if constexpr (LS == 2) {
                                const u32x4_a4 v1 = *reinterpret_cast<const u32x4_a4 *>(src + 4);
                                R.rb[q].d[4] = v1.x; R.rb[q].d[5] = v1.y; R.rb[q].d[6] = v1.z; R.rb[q].d[7] = v1.w;
                            }
                        }
                        R.mb[q] = (uint32_t)(e & (EPD - 1)) | ((ok && !safe) ? UNSAFE : 0u) | ((uint32_t)lo << 8) |
                                  ((uint32_t)(ok ? hi : lo) << 16);
                    }
                }
            }
        }
        // advance to the next chunk of this workgroup's stream
        ++f_c;
        f_oh += step_oh;
        f_ow += step_ow;
        if (LOADER != 0 && f_ow >= a.kcolsp) { f_ow -= a.kcolsp; ++f_oh; }
        if (f_c == c_end) { f_c = c_begin; ++f_i; f_oh = oh0; f_ow = ow00; }
    };

    // the partial last piece of a flat row was read `back` elements early: move it down (whole
    // dwords: `back` is even for bf16) and zero what is shifted in
    auto rotate_down = [&](uint32_t (&v)[4], int back) {
        const int sh = back / EPD;
        if (sh & 1) { v[0] = v[1]; v[1] = v[2]; v[2] = v[3]; v[3] = 0u; }
        if (sh & 2) { v[0] = v[2]; v[1] = v[3]; v[2] = 0u; v[3] = 0u; }
    };

    // Finish the fetched pieces in registers and put the chunk into one LDS buffer.
    auto stage = [&](const RawSet &R, char *bufA, char *bufB) {
        const int i = R.i, c = R.c, k0 = c * KC;
        float f = 1.0f;
        if constexpr (WEIGHTED) f = a.group_sqnorm ? clip_factor(a.group_sqnorm[i], a.clip_c) : 1.0f;
        if (all_slow) {
            slow_stage_a<BF16, MT, WEIGHTED>(bufA, dyg + (size_t)i * dy_ex, a.cout, a.S, a.oh, a.ow, a.kcolsp, m0, k0, f);
            slow_stage_b<BF16, NT>(bufB, xg + (size_t)i * x_ex, cols, a.h, a.w, a.oh, a.ow, a.stride, a.kcolsp, k0);
            return;
        }
        const int lds_col = (threadIdx.x & 7) * 16;
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            uint32_t v[4];
            if constexpr (LOADER == 0) {
                v[0] = R.ra[q].d[0]; v[1] = R.ra[q].d[1]; v[2] = R.ra[q].d[2]; v[3] = R.ra[q].d[3];
                rotate_down(v, (int)(R.ma[q] >> 8));
                mask_piece<BF16>(v, 0, (int)(R.ma[q] & 0xFFu));
            } else {
                const int hi = (R.ma[q] & UNSAFE) ? 0 : (int)(R.ma[q] >> 16);
                if constexpr (BF16) {
                    piece_finish<BF16, 1>(v, R.ra[q], R.ma[q] & 1u, 0, hi);
                } else {
                    v[0] = R.ra[q].d[0]; v[1] = R.ra[q].d[1]; v[2] = R.ra[q].d[2]; v[3] = R.ra[q].d[3];
                    mask_piece<BF16>(v, 0, hi);
                }
            }
            if constexpr (WEIGHTED) scale_regs<BF16, 4>(v, f);
            *reinterpret_cast<uint4 *>(bufA + (row0 + 32 * q) * PITCH + lds_col) = make_uint4(v[0], v[1], v[2], v[3]);
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            uint32_t v[4];
            if constexpr (LOADER == 0) {
                v[0] = R.rb[q].d[0]; v[1] = R.rb[q].d[1]; v[2] = R.rb[q].d[2]; v[3] = R.rb[q].d[3];
                rotate_down(v, (int)(R.mb[q] >> 8));
            } else {
                const int lo = (int)((R.mb[q] >> 8) & 0xFFu);
                const int hi = (R.mb[q] & UNSAFE) ? lo : (int)(R.mb[q] >> 16);
                piece_finish<BF16, LS>(v, R.rb[q], R.mb[q] & 1u, lo, hi);
            }
            *reinterpret_cast<uint4 *>(bufB + (row0 + 32 * q) * PITCH + lds_col) = make_uint4(v[0], v[1], v[2], v[3]);
        }
        if constexpr (LOADER != 0) {
            // the few pieces staged as zeros because their window would have left the tensor
            if (i == 0 || i == a.n - 1) {
                const int oh = R.oh, ow0 = R.ow0;
                const E *ex_a = dyg + (size_t)i * dy_ex;
                const E *ex_b = xg + (size_t)i * x_ex;
#pragma unroll
                for (int q = 0; q < PA; ++q) {
                    if (R.ma[q] & UNSAFE) {
                        const E *src = ex_a + a_row_off[q] + oh * a.ow + ow0;
                        E *dst = reinterpret_cast<E *>(bufA + (row0 + 32 * q) * PITCH + lds_col);
                        const int hi = (int)(R.ma[q] >> 16);
#pragma unroll 1
                        for (int e = 0; e < hi; ++e) {
                            E val = src[e];
                            if constexpr (WEIGHTED) {
                                if constexpr (BF16) val = float_to_bf16_bits(bf16_bits_to_float(val) * f);
                                else val = val * f;
                            }
                            dst[e] = val;
                        }
                    }
                }
#pragma unroll
                for (int q = 0; q < PB; ++q) {
                    if (R.mb[q] & UNSAFE) {
                        const E *src = ex_b + b_off[q] + oh * a.stride * a.w + ow0 * a.stride;
                        E *dst = reinterpret_cast<E *>(bufB + (row0 + 32 * q) * PITCH + lds_col);
                        const int lo = (int)((R.mb[q] >> 8) & 0xFFu), hi = (int)(R.mb[q] >> 16);
#pragma unroll 1
                        for (int e = lo; e < hi; ++e) dst[e] = src[e * LS];
                    }
                }
            }
        }
    };

    auto finish = [&](int i) {
        // The epilogue may sit inside the chunk loop (several examples per workgroup).  Its index
        // arithmetic is loop-invariant; passing the tile origin through an opaque copy keeps the
        // compiler from hoisting ~100 registers of addresses across the MFMA loop.
        int m0v = __builtin_amdgcn_readfirstlane(m0), n0v = __builtin_amdgcn_readfirstlane(n0);
        asm volatile("" : "+s"(m0v), "+s"(n0v));
        const float ss = tile_epilogue<WAVES_N, TM, TN, WEIGHTED, BIAS>(acc, a, i, m0v, n0v, wm, wn, lane, bias_here);
        if constexpr (!WEIGHTED) {
            // four partial-norm slots per (example, tile): this kernel fills the first with the workgroup's sum
            const float tot = block_sum<4>(ss, red);
            if (threadIdx.x < 4) a.partials[((size_t)i * tiles + tile) * 4 + threadIdx.x] = threadIdx.x == 0 ? tot : 0.0f;
        }
    };

    // MFMAs of one chunk out of one LDS buffer; then, in per-example mode without K slices, the
    // epilogue of an example whose K has run out.
    int chunk_in_ex = 0, ex = i_begin;
    auto compute = [&](const char *bufA, const char *bufB) {
        const char *pa = bufA + (wm * TM * 32 + (lane & 31)) * PITCH + (lane >> 5) * 16;
        const char *pb = bufB + (wn * TN * 32 + (lane & 31)) * PITCH + (lane >> 5) * 16;
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
                        acc[tm * TN + tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            va, __builtin_bit_cast(bf16x8, fb[tn]), acc[tm * TN + tn], 0, 0, 0);
                    if constexpr (BIAS) {
                        if (bias_here) {
                            const uint4 one = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
                            acc[TM * TN + tm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                va, __builtin_bit_cast(bf16x8, one), acc[TM * TN + tm], 0, 0, 0);
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
                            acc[tm * TN + tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[e], bv[e], acc[tm * TN + tn], 0, 0, 0);
                    }
                    if constexpr (BIAS) {
                        if (bias_here) {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                acc[TM * TN + tm] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[e], 1.0f, acc[TM * TN + tm], 0, 0, 0);
                        }
                    }
                }
            }
        }
        if constexpr (!WEIGHTED) {
            if (a.ksplit == 1 && ++chunk_in_ex == cpe) {
                finish(ex);
                ++ex;
                chunk_in_ex = 0;
#pragma unroll
                for (int t = 0; t < NACC; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
            }
        }
    };

    // ---- software pipeline, one barrier per chunk:
    //   loads of chunk c+2 are issued, chunk c runs out of LDS buffer c%2, chunk c+1 (whose loads
    //   were issued one step earlier) is finished into buffer (c+1)%2, barrier.
    char *a0 = sA, *a1 = sA + MT * PITCH, *b0 = sB, *b1 = sB + NT * PITCH;
    if (n_chunks > 0) fetch(set0);
    if (n_chunks > 1) fetch(set1);
    if (n_chunks > 0) stage(set0, a0, b0);
    __syncthreads();
    for (int chunk = 0; chunk < n_chunks; chunk += 2) {
        if (chunk + 2 < n_chunks) fetch(set0);
        compute(a0, b0);
        if (chunk + 1 < n_chunks) stage(set1, a1, b1);
        __syncthreads();
        if (chunk + 1 >= n_chunks) break;
        if (chunk + 3 < n_chunks) fetch(set1);
        compute(a1, b1);
        if (chunk + 2 < n_chunks) stage(set0, a0, b0);
        __syncthreads();
    }

    if (a.ksplit == 1 && !(WEIGHTED && a.unit_major)) {
        if constexpr (WEIGHTED) finish(0);
        return;
    }

    // ---- slices of one tile meet in the workspace; a second kernel (conv_fixup_kernel) adds
    // them in slice order and runs the epilogue.  Plain stores: the kernel boundary orders them.
    const int group = WEIGHTED ? tile : (unit * tiles + tile);     // ex_per_wg == 1 when K is sliced
    size_t slot = (size_t)group * a.ksplit + split;
    if (WEIGHTED && a.unit_major) {                       // (unit, tile, range within the unit)
        const int u = split / a.unit_major;
        slot = ((size_t)u * tiles + tile) * a.unit_major + (split - u * a.unit_major);
    }
    float *mine = a.ws_part + slot * (NACC * 16 * THREADS);
#pragma unroll
    for (int t = 0; t < NACC; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(t * 16 + r) * THREADS + threadIdx.x] = acc[t][r];
}

// ---------------------------------------------------------------------------------------------
// The same contraction for the geometry of LOADER 0 (bf16, one long row of S >= 64 elements per
// channel, S even, no bias: the 1x1 stride-1 convolutions, and strided ones after the subsampling
// pre-pass) with the operands streamed global -> LDS by gfx950's 16-byte LDS-direct loads.
//
// Nothing is staged through registers: a wave instruction moves 64 x 16 bytes = eight 128-byte rows
// of one operand straight into LDS (lane L's 16 bytes land at base + 16 L).  The lane chooses WHICH
// piece of the row it fetches, so the bank-conflict-free layout is a permutation done on the global
// side: row r keeps its piece p in slot p ^ ((r >> 1) & 7); the MFMA operand reads of 16 consecutive
// rows at one k then touch 16 distinct 16-byte bank groups, with no padding in LDS.
// A load's address is a wave-uniform base (example, chunk: scalar registers) plus a per-lane byte
// offset that never changes (row and piece), so a chunk's loads cost no vector arithmetic.
// With no registers tied up by staging the pipeline is STAGES deep: the loads of chunk c + STAGES - 1
// are issued before the MFMAs of chunk c, one barrier per chunk; a workgroup that takes several
// examples in a row keeps that stream going across their boundaries (the epilogue of one example
// runs while the next one's chunks are in flight).  These layers are bound by HBM, and what a compute
// unit can keep in flight is what its LDS holds: STAGES - 1 chunks per workgroup.
// The wait for a chunk is a counted s_waitcnt vmcnt(N): every thread issues exactly the same number of
// LDS-direct loads per chunk, and loads complete in order.
// Rows beyond the matrix (ragged tiles) fetch a valid row instead; the epilogues leave them out of the
// norm and never store them.  Only the last chunk of an example can reach beyond the row (S % 64 != 0):
// its pieces at k >= S fetch an earlier piece of the row (nothing is read beyond the tensor) and are
// overwritten with zeros in LDS, the surplus of a partial last piece likewise, in an extra
// barrier-separated step; and that chunk runs only the MFMA steps that hold data.  The partial last
// piece of the tensor's very last row gets its valid bytes through registers.
// Weighted form: the clip factor is applied in fp32 to the finished per-example tile (a second set of
// accumulators), acc_total += f_i * acc_i -- no second rounding of dY to bf16.
// lane L: LDS[lds_base + 16 L .. +16) <- 16 bytes at base + byte_off.  base and lds_base are wave-uniform
// (already in scalar registers).
__device__ __forceinline__ void lds_direct_16(unsigned long long base, unsigned byte_off, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_base) : "memory");
}
// the same with only the lanes of `lanes` (wave-uniform, never empty) taking part: the others fetch nothing and leave
// their 16 bytes of LDS as they are.  The instruction is issued once either way, so counted waits stay exact.
__device__ __forceinline__ void lds_direct_16_lanes(unsigned long long base, unsigned byte_off, unsigned lds_base, unsigned long long lanes)
{
    unsigned long long saved;
    asm volatile("s_mov_b32 m0, %3\n\t"
                 "s_mov_b64 %0, exec\n\t"
                 "s_mov_b64 exec, %4\n\t"
                 "global_load_lds_dwordx4 %1, %2\n\t"
                 "s_mov_b64 exec, %0"
                 : "=&s"(saved)
                 : "v"(byte_off), "s"(base), "s"(lds_base), "s"(lanes)
                 : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Wait until at most `after` (wave-uniform) of this wave's vector memory operations are outstanding, rounded down to
// a count the instruction can encode (six bits) from a short menu: waiting for more than asked is always safe.
__device__ __forceinline__ void wait_outstanding(int after)
{
    if (after >= 63) wait_vmcnt<63>();
#define DP_WAIT_STEP(K) else if (after >= K) wait_vmcnt<K>();
    DP_WAIT_STEP(56) DP_WAIT_STEP(48) DP_WAIT_STEP(40) DP_WAIT_STEP(36) DP_WAIT_STEP(32) DP_WAIT_STEP(24) DP_WAIT_STEP(20)
    DP_WAIT_STEP(16) DP_WAIT_STEP(12) DP_WAIT_STEP(8) DP_WAIT_STEP(6) DP_WAIT_STEP(4)
#undef DP_WAIT_STEP
    else wait_vmcnt<0>();
}

// WM x 2 waves (WM = 2: 256 threads; WM = 4: 512 threads, a 256 x 128 tile whose eight waves share the X rows: a quarter
// fewer operand bytes into LDS per multiply-add, and with three stages in 144 KB two chunks are in flight instead of the
// one each that two resident 128 x 128 workgroups have -- the per-example form of these layers waits on memory, and what a
// compute unit keeps in flight is what its LDS holds).  WM = 4: whole tiles only, K never sliced, per-example form.
template <int WM, int TM, int TN, bool WEIGHTED, int STAGES>
__global__ void __launch_bounds__(WM * 128, (STAGES * (WM * TM + 2 * TN) * 4 <= 64 ? 2 : 1)) conv_flat_kernel(const Grouped<ConvArgs> grp)
{
    typedef uint16_t E;
    constexpr int KC = 64, EPP = 8;
    constexpr int NWAVES = WM * 2;
    constexpr int MT = WM * TM * 32, NT = 2 * TN * 32;
    constexpr int ROWS = MT + NT;                        // LDS rows of 128 bytes per stage: A rows, then B rows
    constexpr int STAGE_BYTES = ROWS * 128;
    constexpr int NLD = ROWS / (8 * NWAVES);             // LDS-direct loads per thread and chunk (eight rows per wave instruction)
    constexpr int NLA = MT / (8 * NWAVES);               // of which the first NLA fetch rows of A (dY)
    constexpr int NACC = TM * TN;
    static_assert(STAGES >= 2 && STAGES <= 5, "pipeline depth");
    static_assert(ROWS % (8 * NWAVES) == 0 && MT % (8 * NWAVES) == 0, "whole wave instructions");
    static_assert(WM == 2 || !WEIGHTED, "the wide workgroup is the per-example form");
    extern __shared__ __attribute__((aligned(16))) char lds[];

    unsigned bid;
    const ConvArgs &a = grp.a[group_pick(grp, bid)];

    const int tiles = a.tiles_m * a.tiles_n;
    int total, tile, unit;
    if constexpr (WEIGHTED) {
        total = tiles * a.ksplit;
    } else {
        const int ex_groups = (a.n + a.ex_per_wg - 1) / a.ex_per_wg;
        total = ex_groups * tiles * a.ksplit;
    }
    const int per_xcd = (total + 7) >> 3;
    const int wg = (int)(bid & 7u) * per_xcd + (int)(bid >> 3);
    if (wg >= total) return;
    int split;
    if constexpr (WEIGHTED) {
        tile = wg / a.ksplit;
        split = wg - tile * a.ksplit;
        unit = 0;
    } else {
        split = wg % a.ksplit;
        const int r = wg / a.ksplit;
        unit = r / tiles;
        tile = r - unit * tiles;
    }
    const int tile_m = tile / a.tiles_n, tile_n = tile - tile_m * a.tiles_n;
    const int m0 = __builtin_amdgcn_readfirstlane(tile_m * MT), n0 = __builtin_amdgcn_readfirstlane(tile_n * NT);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    int i_begin, i_end, c_begin, c_end;
    if constexpr (WEIGHTED) {
        i_begin = split * a.ex_per_split;
        i_end = min(a.n, i_begin + a.ex_per_split);
        c_begin = 0;
        c_end = a.chunks_per_ex;
    } else {
        i_begin = unit * a.ex_per_wg;
        i_end = min(a.n, i_begin + a.ex_per_wg);
        c_begin = split * a.chunks_per_split;
        c_end = min(a.chunks_per_ex, c_begin + a.chunks_per_split);
    }
    i_begin = __builtin_amdgcn_readfirstlane(i_begin);
    c_begin = __builtin_amdgcn_readfirstlane(c_begin);
    c_end = __builtin_amdgcn_readfirstlane(c_end);
    const int cpe = c_end - c_begin;
    const int n_chunks = __builtin_amdgcn_readfirstlane((i_end - i_begin) * cpe);

    const int S = __builtin_amdgcn_readfirstlane(a.S);
    const int cout = __builtin_amdgcn_readfirstlane(a.cout), J = __builtin_amdgcn_readfirstlane(a.J);
    const int n_examples = __builtin_amdgcn_readfirstlane(a.n), chunks_per_ex = __builtin_amdgcn_readfirstlane(a.chunks_per_ex);
    const int ksplit = __builtin_amdgcn_readfirstlane(a.ksplit);
    const size_t x_ex = (size_t)a.cin * S, dy_ex = (size_t)cout * S;
    const E *xg = static_cast<const E *>(a.x), *dyg = static_cast<const E *>(a.dy);
    // the last chunk of an example when the row does not end on a chunk boundary: only some K steps hold data
    const int last_valid = S - (chunks_per_ex - 1) * KC;              // elements of a row in the last chunk: 1 .. 64
    const bool has_tail = last_valid < KC;
    const int tail = S & 7;                                           // elements of a row's partial last piece (0: none)
    const int last_ksteps = (last_valid + 15) >> 4;                   // MFMA steps of 16 that hold data in the last chunk

    // ---- this thread's NLD loads of a chunk: load q of wave w fills rows [(4 q + w) 8, +8) of the stage
    // (loads q < NLA are rows of A, the rest rows of B); lane -> row rb = lane / 8 of those, slot = lane % 8,
    // piece p = slot ^ ((row >> 1) & 7)
    unsigned byte_off[NLD];      // of the row's piece within one example's operand, at chunk 0
    unsigned tail_off[NLD];      // what the last chunk fetches instead, relative to the START OF THE PREVIOUS CHUNK
    unsigned stand_off[NLD];     // the stand-in (last piece of the previous chunk), relative to the same
    unsigned guard_mask = 0;     // bit q: load q is the partial last piece of its operand's last row (its own row, or as
                                 // stand-in for a row beyond the matrix): in the last example it would read past the tensor
    unsigned long long tail_lanes[NLD];   // lanes of load q whose piece starts inside the row in the last chunk (one in eight at least)
    const int rb = lane >> 3, slot = lane & 7;
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const int row = (NWAVES * q + wave) * 8 + rb;
        const int pk = (slot ^ ((row >> 1) & 7)) * EPP;
        int r;                                            // row of the operand; rows beyond the matrix fetch its last row
        bool last_row;
        if (q < NLA) {
            r = min(m0 + row, cout - 1);
            last_row = m0 + row >= cout - 1;
        } else {
            r = min(n0 + row - MT, J - 1);
            last_row = n0 + row - MT >= J - 1;
        }
        const unsigned row_byte = (unsigned)r * (unsigned)S * 2u;
        byte_off[q] = row_byte + (unsigned)pk * 2u;
        // last chunk: pieces that start at or beyond the row's end fetch the last piece of the chunk before
        // (inside the tensor; their K steps are never computed or are masked); all others their own piece
        stand_off[q] = row_byte + 2u * (KC - EPP);
        tail_off[q] = pk < last_valid ? byte_off[q] + 2u * KC : stand_off[q];
        tail_lanes[q] = __ballot(pk < last_valid);
        if (last_row && pk < last_valid && pk + EPP > last_valid) guard_mask |= 1u << q;
    }

    // ---- the stream of chunks to fetch: scalar base addresses advanced by constants
    unsigned long long ga = uniform_bits(dyg + (size_t)i_begin * dy_ex + (size_t)c_begin * KC);
    unsigned long long gb = uniform_bits(xg + (size_t)i_begin * x_ex + (size_t)c_begin * KC);
    const unsigned long long a_jump = (unsigned long long)(dy_ex - (size_t)cpe * KC) * 2ull;      // from an example's last chunk to the next one's first
    const unsigned long long b_jump = (unsigned long long)(x_ex - (size_t)cpe * KC) * 2ull;
    const unsigned lds_wave = __builtin_amdgcn_readfirstlane((unsigned)(size_t)lds + (unsigned)wave * 1024u);
    int f_i = i_begin, f_c = c_begin;                     // next chunk to fetch
    unsigned f_dst = lds_wave;                            // where it goes: its stage, this wave's kilobyte
    auto fetch = [&]() {
        if (!(has_tail && f_c == chunks_per_ex - 1)) {
#pragma unroll
            for (int q = 0; q < NLD; ++q) lds_direct_16(q < NLA ? ga : gb, byte_off[q], f_dst + q * (NWAVES * 1024));
        } else {
            // offsets are unsigned, so those of the last chunk count from the start of the chunk before it.  The partial
            // last piece of the tensor's very last row would read past the tensor: it fetches the stand-in as well.
            const unsigned guard = (tail && f_i == n_examples - 1) ? guard_mask : 0u;
#pragma unroll
            for (int q = 0; q < NLD; ++q)
                lds_direct_16_lanes((q < NLA ? ga : gb) - 2ull * KC, ((guard >> q) & 1u) ? stand_off[q] : tail_off[q], f_dst + q * (NWAVES * 1024),
                                    tail_lanes[q]);
        }
        ga += 2ull * KC;
        gb += 2ull * KC;
        f_dst += STAGE_BYTES;
        if (f_dst >= lds_wave + STAGES * STAGE_BYTES) f_dst = lds_wave;
        if (++f_c == c_end) { f_c = c_begin; ++f_i; ga += a_jump; gb += b_jump; }
    };

    // the tensor's very last row, last example: its partial last piece fetched a stand-in; the valid dwords
    // come through registers (taken by at most two workgroups of a launch), between two barriers
    auto fix_very_last = [&](int stage) {
#pragma unroll
        for (int q = 0; q < NLD; ++q) {
            if ((guard_mask >> q) & 1u) {
                uint32_t *d4 = reinterpret_cast<uint32_t *>(lds + stage * STAGE_BYTES + (NWAVES * q + wave) * 1024 + lane * 16);
                const char *ex = reinterpret_cast<const char *>(q < NLA ? dyg + (size_t)(n_examples - 1) * dy_ex
                                                                        : xg + (size_t)(n_examples - 1) * x_ex);
                const uint32_t *src = reinterpret_cast<const uint32_t *>(ex + byte_off[q] + (size_t)(chunks_per_ex - 1) * KC * 2);
#pragma unroll
                for (int d = 0; d < 3; ++d)
                    if (2 * d < tail) d4[d] = src[d];
            }
        }
    };

    f32x16 acc[NACC];
    f32x16 tot[WEIGHTED ? NACC : 1];
#pragma unroll
    for (int t = 0; t < NACC; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
    if constexpr (WEIGHTED) {
#pragma unroll
        for (int t = 0; t < NACC; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) tot[t][r] = 0.0f;
    }

    // operand reads: lane -> row (lane & 31) of a 32-row block, K step ks -> pieces 2 ks + (lane >> 5), swizzled
    int koff[4];
    {
        const int t16 = (((lane >> 5) ^ ((lane >> 1) & 7)) & 7) * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) koff[ks] = (ks * 32) ^ t16;
    }
    const int a_row = (wm * TM * 32 + (lane & 31)) * 128;
    const int b_row = (MT + wn * TN * 32 + (lane & 31)) * 128;
    // the last K step of an example's last chunk: elements at or beyond the row's end are zeroed in registers
    // (lane holds elements (lane >> 5) * 8 .. +8 of the step); dword d keeps its low / high half or nothing
    uint32_t kmask[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const int e0 = (last_ksteps - 1) * 16 + (lane >> 5) * 8 + 2 * d;
        kmask[d] = (e0 < last_valid ? 0x0000FFFFu : 0u) | (e0 + 1 < last_valid ? 0xFFFF0000u : 0u);
    }

    // MFMAs of one full chunk: the operand reads of two K steps are issued together, ahead of their MFMAs
    auto compute = [&](int stage) {
        const char *base = lds + stage * STAGE_BYTES;
        constexpr int KB = (TM * TN > 1) ? 2 : 4;        // K steps whose operand reads are issued together
#pragma unroll
        for (int k0 = 0; k0 < 4; k0 += KB) {
            uint4 fa[KB][TM], fb[KB][TN];
#pragma unroll
            for (int kk = 0; kk < KB; ++kk) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) fa[kk][tm] = *reinterpret_cast<const uint4 *>(base + a_row + tm * 32 * 128 + koff[k0 + kk]);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) fb[kk][tn] = *reinterpret_cast<const uint4 *>(base + b_row + tn * 32 * 128 + koff[k0 + kk]);
            }
#pragma unroll
            for (int kk = 0; kk < KB; ++kk)
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm * TN + tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, fa[kk][tm]), __builtin_bit_cast(bf16x8, fb[kk][tn]), acc[tm * TN + tn], 0, 0, 0);
        }
    };
    // the same for an example's last chunk when the row ends inside it
    auto compute_tail = [&](int stage) {
        const char *base = lds + stage * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < last_ksteps) {                       // uniform
                uint4 fa[TM], fb[TN];
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) fa[tm] = *reinterpret_cast<const uint4 *>(base + a_row + tm * 32 * 128 + koff[ks]);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) fb[tn] = *reinterpret_cast<const uint4 *>(base + b_row + tn * 32 * 128 + koff[ks]);
                if (ks == last_ksteps - 1) {
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) { fa[tm].x &= kmask[0]; fa[tm].y &= kmask[1]; fa[tm].z &= kmask[2]; fa[tm].w &= kmask[3]; }
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) { fb[tn].x &= kmask[0]; fb[tn].y &= kmask[1]; fb[tn].z &= kmask[2]; fb[tn].w &= kmask[3]; }
                }
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm * TN + tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, fa[tm]), __builtin_bit_cast(bf16x8, fb[tn]), acc[tm * TN + tn], 0, 0, 0);
            }
        }
    };

    // ---- per-example mode, end of an example: norm share of every wave into its own slot (no barrier), optional store.
    // Whole tiles (all of them when the channel counts are multiples of the tile): a value's address is a scalar base
    // (example, 32-row block) + a per-lane offset that is fixed for the kernel (register r's row, the lane's column)
    // + an immediate (32-column block), so a store costs no arithmetic at all.
    const bool whole_tile = WM != 2 || (m0 + MT <= cout && n0 + NT <= J);                   // uniform
    float *const out_w = a.out_w;
    float *const partials = a.partials;
    const bool store_whole = out_w != nullptr && whole_tile;
    unsigned row_off[16];
    {
        const unsigned lane_off = ((unsigned)(wm * TM * 32 + (lane >> 5) * 4) * (unsigned)J + (unsigned)(wn * TN * 32 + (lane & 31))) * 4u;
#pragma unroll
        for (int r = 0; r < 16; ++r) row_off[r] = lane_off + (unsigned)((r >> 2) * 8 + (r & 3)) * (unsigned)J * 4u;
    }
    const unsigned long long block_bytes = (unsigned long long)J * 128ull;                  // 32 rows of the gradient matrix
    const unsigned long long out_ex_bytes = uniform_bits(reinterpret_cast<const void *>(a.out_stride_w * sizeof(float)));
    unsigned long long out_corner = uniform_bits(out_w + (size_t)i_begin * a.out_stride_w + (size_t)m0 * J + n0);
    auto finish = [&](int i) {
        float ss = 0.0f;
        if (whole_tile) {
            float part[NACC];                             // one chain of multiply-adds per block: they run interleaved
#pragma unroll
            for (int t = 0; t < NACC; ++t) {
                part[t] = acc[t][0] * acc[t][0];
#pragma unroll
                for (int r = 1; r < 16; ++r) part[t] += acc[t][r] * acc[t][r];
            }
#pragma unroll
            for (int t = 0; t < NACC; ++t) ss += part[t];
            if (store_whole) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    const unsigned long long base = out_corner + (unsigned long long)tm * block_bytes;
                    static_for<TN>([&](auto tn_c) {
                        constexpr int tn = decltype(tn_c)::value;
#pragma unroll
                        for (int r = 0; r < 16; ++r) store_f32_uniform_base_nt_at<tn * 128>(base, row_off[r], acc[tm * TN + tn][r]);
                    });
                }
            }
        } else {
            ss = tile_epilogue<2, TM, TN, false, false, false>(acc, a, i, m0, n0, wm, wn, lane, false);
        }
        out_corner += out_ex_bytes;
        const float ws = wave_sum_last_lane(ss);
        if (lane == 63) partials[((size_t)i * tiles + tile) * NWAVES + wave] = ws;
    };

    // ---- pipeline: chunks c+1 .. c+STAGES-2 are in flight while chunk c is in the MFMAs.  One loop nest per example
    // (its full chunks, then the partial one) so that the accumulators live in one set of registers.
    int fetched = 0;
#pragma unroll
    for (int s0 = 0; s0 < STAGES - 1; ++s0)
        if (fetched < n_chunks) { fetch(); ++fetched; }
    int stage = 0, c = 0;
    // gradient stores this wave issued in each of the last STAGES - 1 steps ([0]: the step before this one) and since the
    // current step began.  Only epilogues whose store count is certain are entered (whole tiles: one unconditional store
    // per accumulator register).
    int stores_in[STAGES - 1], stores_now = 0;
#pragma unroll
    for (int k = 0; k < STAGES - 1; ++k) stores_in[k] = 0;
    const int stores_per_tile = __builtin_amdgcn_readfirstlane((!WEIGHTED && store_whole) ? NACC * 16 : 0);
    // chunk c becomes current
    auto begin_step = [&]() {
#pragma unroll
        for (int k = STAGES - 2; k > 0; --k) stores_in[k] = stores_in[k - 1];
        stores_in[0] = stores_now;
        stores_now = 0;
        // chunk c has landed when at most the operations issued after its loads are outstanding (the counter covers loads
        // and stores alike, in issue order): the loads of the chunks fetched since, and the stores of the epilogues that
        // ran since -- chunk c was fetched STAGES - 1 steps ago, or before the first step
        int after = (fetched - c - 1) * NLD;
#pragma unroll
        for (int k = 0; k < STAGES - 1; ++k) after += stores_in[k];
        wait_outstanding(after);
        __syncthreads();                                  // everyone's loads of chunk c are in LDS; chunk c-1 has been read
        if (fetched < n_chunks) { fetch(); ++fetched; }   // into the stage chunk c-1 used
    };
    auto end_step = [&]() {
        ++c;
        if (++stage == STAGES) stage = 0;
    };
    const bool tail_here = has_tail && c_end == chunks_per_ex;                  // this range of chunks ends with the partial one
    const int full_here = cpe - (tail_here ? 1 : 0);
    const bool edge_tile = m0 + MT >= cout || n0 + NT >= J;
    const float *const group_sqnorm = a.group_sqnorm;
    const float clip_c = a.clip_c;
    for (int ex = i_begin; ex < i_end; ++ex) {
#pragma unroll
        for (int t = 0; t < NACC; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
        for (int ch = 0; ch < full_here; ++ch) {
            begin_step();
            compute(stage);
            end_step();
        }
        if (tail_here) {
            begin_step();
            if (tail && ex == n_examples - 1 && edge_tile) {                    // uniform, rare
                fix_very_last(stage);
                __syncthreads();
            }
            compute_tail(stage);
            end_step();
        }
        if constexpr (WEIGHTED) {
            const float f = group_sqnorm ? clip_factor(group_sqnorm[ex], clip_c) : 1.0f;
#pragma unroll
            for (int t = 0; t < NACC; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) tot[t][r] += f * acc[t][r];
        } else if (ksplit == 1) {
            finish(ex);
            stores_now = stores_per_tile;
        }
    }

    if constexpr (WEIGHTED) {
        if (ksplit == 1 && !a.unit_major) {
            tile_epilogue<2, TM, TN, true, false>(tot, a, 0, m0, n0, wm, wn, lane, false);
            return;
        }
    } else if (ksplit == 1) {
        return;
    }
    if constexpr (WM != 2) return;                        // never sliced (the host plans it so)
    // slices of one tile meet in the workspace (conv_fixup_kernel adds them in slice order)
    const int group = WEIGHTED ? tile : (unit * tiles + tile);
    size_t part = (size_t)group * ksplit + split;
    if (WEIGHTED && a.unit_major) {                       // (unit, tile, range within the unit)
        const int u = split / a.unit_major;
        part = ((size_t)u * tiles + tile) * a.unit_major + (split - u * a.unit_major);
    }
    float *mine = a.ws_part + part * (NACC * 16 * THREADS);
#pragma unroll
    for (int t = 0; t < NACC; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(t * 16 + r) * THREADS + threadIdx.x] = WEIGHTED ? tot[t][r] : acc[t][r];
}

// Slices of one tile meet here.  The sum over slices is elementwise, so it is spread over many
// small workgroups: one per (tile, 32x32 accumulator block t, four of its sixteen registers).
// Each thread adds its four values over the slices in slice order (same bits every run) with
// eight slices of loads in flight, then does for them what the unsliced epilogue does.
constexpr int FIX_R = 4;                       // accumulator registers per fixup thread
constexpr int FIX_PARTS = 16 / FIX_R;

template <int WAVES_M, int WAVES_N, int TM, int TN, bool WEIGHTED, bool BIAS>
__global__ void __launch_bounds__(THREADS) conv_fixup_kernel(const Grouped<ConvArgs> grp)
{
    constexpr int MT = WAVES_M * TM * 32, NT = WAVES_N * TN * 32;
    constexpr int NACC = TM * TN + (BIAS ? TM : 0);
    __shared__ float red[4];
    unsigned bid;
    const ConvArgs &a = grp.a[group_pick(grp, bid)];
    const int tiles = a.tiles_m * a.tiles_n;
    const int part = bid % FIX_PARTS;
    const int t = (bid / FIX_PARTS) % NACC;
    const int group = bid / (FIX_PARTS * NACC);
    const int i = WEIGHTED ? 0 : group / tiles;
    const int tile = WEIGHTED ? group : group - i * tiles;
    const int tile_m = tile / a.tiles_n, tile_n = tile - tile_m * a.tiles_n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / WAVES_N, wn = wave - wm * WAVES_N;

    const size_t slice = (size_t)NACC * 16 * THREADS;
    const float *base = a.ws_part + (size_t)group * a.ksplit * slice + (size_t)(t * 16 + part * FIX_R) * THREADS + threadIdx.x;
    float v[FIX_R];
#pragma unroll
    for (int r = 0; r < FIX_R; ++r) v[r] = 0.0f;
    int s = 0;
    for (; s + 8 <= a.ksplit; s += 8) {
        float tmp[8][FIX_R];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < FIX_R; ++r) tmp[u][r] = base[(size_t)(s + u) * slice + r * THREADS];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < FIX_R; ++r) v[r] += tmp[u][r];
    }
    for (; s < a.ksplit; ++s) {
        float tmp[FIX_R];
#pragma unroll
        for (int r = 0; r < FIX_R; ++r) tmp[r] = base[(size_t)s * slice + r * THREADS];
#pragma unroll
        for (int r = 0; r < FIX_R; ++r) v[r] += tmp[r];
    }

    const bool is_bias = BIAS && t >= TM * TN;
    const int tm = is_bias ? t - TM * TN : t / TN, tn = is_bias ? 0 : t - tm * TN;
    const int j = tile_n * NT + (wn * TN + tn) * 32 + (lane & 31);
    const bool bias_lane = is_bias && tile_n == 0 && wn == 0 && (lane & 31) == 0;
    float ss = 0.0f;
#pragma unroll
    for (int rr = 0; rr < FIX_R; ++rr) {
        const int r = part * FIX_R + rr;
        const int m = tile_m * MT + (wm * TM + tm) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (!is_bias) {
            const bool ok = m < a.cout && j < a.J;
            if constexpr (WEIGHTED) {
                if (ok) a.out_w[(size_t)m * a.J + j] += v[rr];
            } else {
                ss += ok ? v[rr] * v[rr] : 0.0f;
                if (ok && a.out_w) a.out_w[(size_t)i * a.out_stride_w + (size_t)m * a.J + j] = v[rr];
            }
        } else if (bias_lane) {
            if constexpr (WEIGHTED) {
                if (m < a.cout) a.out_b[m] += v[rr];
            } else {
                ss += v[rr] * v[rr];
                if (m < a.cout && a.out_w) a.out_b[(size_t)i * a.out_stride_b + m] = v[rr];
            }
        }
    }
    if constexpr (!WEIGHTED) {
        const float tot = block_sum<4>(ss, red);
        if (threadIdx.x == 0) a.partials[bid] = tot;
    }
}

// ---------------------------------------------------------------------------------------------
// Row-panel form of the per-example contraction for the LOADER 0 geometry with SHORT rows (S a little under 16 KS
// elements, S = 4 mod 8; the 1x1 layers on 14x14 maps: S = 196).
//
// Cutting such rows into 64-element chunks makes every load instruction fetch eight separate 128-byte pieces that
// straddle cache lines (rows are S * 2 bytes apart); the cache serves that pattern at about a third of the rate of
// contiguous kilobytes.  But 32 whole rows of one example ARE one contiguous span of 64 S bytes.  So the unit that
// travels is a block of 32 whole rows, copied as it lies in memory into a slot of a ring in LDS (each wave an eighth
// of it, 16 bytes per lane), and the workgroup walks a stream of blocks: per example first the eight blocks of its 256
// dY rows -- wave w keeps block w in REGISTERS as MFMA operands (all KS steps of K: 4 KS registers) -- then eight
// blocks of 32 X rows each; every wave multiplies its dY rows with each X block (KS MFMAs 32x32x16, the first one
// onto zero), squares, stores its 32 x 32 piece of the gradient, and forgets it.  The ring is as deep as LDS allows
// (eleven blocks in flight), the stream runs across example boundaries, one barrier per block.
// Rows lie S * 2 bytes apart in LDS: a multiple of 8 but not of 16 bytes, so an operand is read as two 8-byte halves,
// and with S / 2 = 2 mod 4 dwords per row sixteen consecutive rows start in sixteen different pairs of banks.
// The last K step reads past the row's end (into the next row, or the slot's padding): those elements are cleared in
// registers, in both operands.
// Whole tiles only: cout a multiple of 256, J a multiple of 256 (the host plans it so).  Norm partials: one slot per
// (example, 256 x 256 tile, wave).
constexpr int PANEL_RING = 12;               // slots of the ring
constexpr int PANEL_CB = 8;                  // X blocks (32 columns each) per tile

__device__ __forceinline__ uint4 lds_read16_halves(const char *p)         // p: 8-byte aligned
{
    const uint2 lo = *reinterpret_cast<const uint2 *>(p), hi = *reinterpret_cast<const uint2 *>(p + 8);
    return make_uint4(lo.x, lo.y, hi.x, hi.y);
}

template <int KS>
__global__ void __launch_bounds__(512, 1) conv_panel_kernel(const Grouped<ConvArgs> grp)
{
    typedef uint16_t E;
    constexpr int R = PANEL_RING, CB = PANEL_CB, STEPS = 8 + CB;
    constexpr int NL = (KS * 8 + 63) / 64;               // load instructions per wave and block: S / 2 lanes of 16 bytes
    extern __shared__ __attribute__((aligned(16))) char lds[];

    unsigned bid;
    const ConvArgs &a = grp.a[group_pick(grp, bid)];
    const int tiles = a.tiles_m * a.tiles_n;
    const int ex_groups = (a.n + a.ex_per_wg - 1) / a.ex_per_wg;
    const int total = ex_groups * tiles;
    const int per_xcd = (total + 7) >> 3;
    const int wg = (int)(bid & 7u) * per_xcd + (int)(bid >> 3);
    if (wg >= total) return;
    const int unit = wg / tiles, tile = wg - unit * tiles;
    const int tile_m = tile / a.tiles_n, tile_n = tile - tile_m * a.tiles_n;
    const int m0 = __builtin_amdgcn_readfirstlane(tile_m * 256), j0 = __builtin_amdgcn_readfirstlane(tile_n * 256);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int S = __builtin_amdgcn_readfirstlane(a.S), cout = __builtin_amdgcn_readfirstlane(a.cout), J = __builtin_amdgcn_readfirstlane(a.J);
    const int i_begin = __builtin_amdgcn_readfirstlane(unit * a.ex_per_wg);
    const int i_end = __builtin_amdgcn_readfirstlane(min(a.n, i_begin + a.ex_per_wg));
    const int n_blocks = (i_end - i_begin) * STEPS;
    const unsigned row_bytes = 2u * (unsigned)S, block_bytes = 32u * row_bytes, share = block_bytes / 8u;
    const unsigned slot_bytes = block_bytes + 64u;       // padding: the last row's last K step reads 24 bytes past it
    const E *const xg = static_cast<const E *>(a.x), *const dyg = static_cast<const E *>(a.dy);
    float *const out_w = a.out_w;
    float *const partials = a.partials;
    const bool store = out_w != nullptr;

    // ---- the stream of blocks to fetch
    int f_i = i_begin, f_p = 0, fetched = 0;
    unsigned f_slot = 0;
    const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(size_t)lds);
    const unsigned long long lanes_last = __ballot(lane < S / 2 - 64 * (NL - 1));       // never empty (the host checks S)
    auto fetch = [&]() {
        const E *src = f_p < 8 ? dyg + ((size_t)f_i * cout + m0 + 32 * f_p) * S
                               : xg + ((size_t)f_i * J + j0 + 32 * (f_p - 8)) * S;
        const unsigned long long base = uniform_bits(src) + (unsigned long long)((unsigned)wave * share);
        const unsigned dst = lds0 + f_slot * slot_bytes + (unsigned)wave * share;
#pragma unroll
        for (int q = 0; q < NL; ++q) {
            if (q < NL - 1) lds_direct_16(base, (unsigned)lane * 16u + q * 1024u, dst + q * 1024u);
            else lds_direct_16_lanes(base, (unsigned)lane * 16u + q * 1024u, dst + q * 1024u, lanes_last);
        }
        if (++f_slot == R) f_slot = 0;
        if (++f_p == STEPS) { f_p = 0; ++f_i; }
        ++fetched;
    };

    // ---- what a wave keeps
    uint4 afr[KS];                                        // its 32 dY rows as MFMA operands, all of K
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) afr[ks] = make_uint4(0, 0, 0, 0);
    uint32_t kmask[4];                                    // last K step: lane holds elements (KS-1) 16 + (lane >> 5) 8 .. +8
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const int e0 = (KS - 1) * 16 + (lane >> 5) * 8 + 2 * d;
        kmask[d] = (e0 < S ? 0x0000FFFFu : 0u) | (e0 + 1 < S ? 0xFFFF0000u : 0u);
    }
    const unsigned frag_off = (unsigned)(lane & 31) * row_bytes + (unsigned)(lane >> 5) * 16u;     // K step ks: + 32 ks
    unsigned row_off[16];                                 // byte offset of register r's value from the 32-column block's corner
#pragma unroll
    for (int r = 0; r < 16; ++r)
        row_off[r] = ((unsigned)(32 * wave + (lane >> 5) * 4 + (r >> 2) * 8 + (r & 3)) * (unsigned)J + (unsigned)(lane & 31)) * 4u;
    const unsigned long long out_ex_bytes = uniform_bits(reinterpret_cast<const void *>(a.out_stride_w * sizeof(float)));
    unsigned long long out_blk = uniform_bits(out_w + (size_t)i_begin * a.out_stride_w + (size_t)m0 * J + j0);

    // ---- counted waits: `issued` counts this wave's vector memory operations; marks[b mod 16] (a few words of LDS of
    // the wave's own) is its value right after the loads of block b went out; block b has landed when at most
    // issued - marks[b mod 16] operations are outstanding.  c: the next block to be consumed.
    int issued = 0, c = 0;
    int *const marks = reinterpret_cast<int *>(lds + R * slot_bytes) + wave * 16;
    auto issued_after = [&](int b) { return issued - __builtin_amdgcn_readfirstlane(marks[b & 15]); };
    // blocks before c are free: fetch while the ring has room
    auto top_up = [&]() {
#pragma nounroll
        while (fetched < n_blocks && fetched - c < R) {
            const int b = fetched;
            fetch();
            issued += NL;
            marks[b & 15] = issued;
        }
    };
    top_up();

    unsigned c_slot = 0;                                  // slot of block c
    auto slot_after = [&](unsigned k) { const unsigned t = c_slot + k; return t >= (unsigned)R ? t - (unsigned)R : t; };
    const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    for (int i = i_begin; i < i_end; ++i) {
        // ---- the example's eight dY blocks in one step: wave w takes block w into registers
        wait_outstanding(issued_after(c + 7));
        __syncthreads();                                  // all eight are in LDS; everything before them has been read
        top_up();
        {
            const char *mine = lds + slot_after((unsigned)wave) * slot_bytes + frag_off;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) afr[ks] = lds_read16_halves(mine + ks * 32);
            afr[KS - 1].x &= kmask[0]; afr[KS - 1].y &= kmask[1]; afr[KS - 1].z &= kmask[2]; afr[KS - 1].w &= kmask[3];
        }
        c += 8;
        c_slot = slot_after(8);

        // ---- its X blocks two at a time: 32 x 64 values of the gradient per wave and step, four independent chains of MFMAs
        float ss0 = 0.0f, ss1 = 0.0f;
#pragma nounroll
        for (int pair = 0; pair < CB / 2; ++pair) {
            wait_outstanding(issued_after(c + 1));
            __syncthreads();
            top_up();
            const char *b0 = lds + c_slot * slot_bytes + frag_off, *b1 = lds + slot_after(1) * slot_bytes + frag_off;
            f32x16 acc[2][2];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint4 v0 = lds_read16_halves(b0 + ks * 32), v1 = lds_read16_halves(b1 + ks * 32);
                if (ks == KS - 1) {
                    v0.x &= kmask[0]; v0.y &= kmask[1]; v0.z &= kmask[2]; v0.w &= kmask[3];
                    v1.x &= kmask[0]; v1.y &= kmask[1]; v1.z &= kmask[2]; v1.w &= kmask[3];
                }
                acc[0][ks & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, afr[ks]), __builtin_bit_cast(bf16x8, v0),
                                                                        ks < 2 ? zero : acc[0][ks & 1], 0, 0, 0);
                acc[1][ks & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, afr[ks]), __builtin_bit_cast(bf16x8, v1),
                                                                        ks < 2 ? zero : acc[1][ks & 1], 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (KS > 1) { acc[0][0][r] += acc[0][1][r]; acc[1][0][r] += acc[1][1][r]; }
                ss0 += acc[0][0][r] * acc[0][0][r];
                ss1 += acc[1][0][r] * acc[1][0][r];
            }
            if (store) {
#pragma unroll
                for (int r = 0; r < 16; ++r) store_f32_uniform_base_nt_at<0>(out_blk, row_off[r], acc[0][0][r]);
#pragma unroll
                for (int r = 0; r < 16; ++r) store_f32_uniform_base_nt_at<128>(out_blk, row_off[r], acc[1][0][r]);
                issued += 32;
            }
            out_blk += 256ull;
            c += 2;
            c_slot = slot_after(2);
        }
        const float ws = wave_sum_last_lane(ss0 + ss1);
        if (lane == 63) partials[((size_t)i * tiles + tile) * 8 + wave] = ws;
        out_blk += out_ex_bytes - 128ull * CB;
    }
}

// ------------------------------------------------------------------------------------ host

enum TileShape { T64 = 0, T128 = 1, T256x128 = 2, T256rows = 3 };
static const int kTileM[4] = {64, 128, 256, 256};
static const int kTileN[4] = {64, 128, 128, 256};
static const char *kTileName[4] = {"64x64", "128x128", "256x128", "256x256rows"};
constexpr int PANEL_KS = 13;                 // K steps the row-panel kernel is built for: 192 < S <= 208

struct FullPlan {
    int shape, tiles_m, tiles_n;
    int kcolsp, chunks_per_ex;
    int ksplit, chunks_per_split, ex_per_split, ex_per_wg;
    int nacc;               // accumulator tiles per wave
    int groups;             // groups of slices (counters)
    size_t part_floats;     // floats of partial tiles in the workspace
    // geometry as the kernel sees it (1x1 stride-1 convs are flattened to one long row)
    int h, w, oh, ow;
};

// Whether plans are made for a launch shared with many other workgroups (a batch call): then a layer
// need not fill the chip by itself, so K is sliced only when a workgroup's walk would get very long and
// example ranges of the weighted form are as long as they can be.  Workspace sizes cover both cases.
static thread_local int tl_forced_crowd = -1;
static int plan_crowd() { return tl_forced_crowd >= 0 ? tl_forced_crowd : crowd_hint(); }

// geometry of the LDS-direct kernel: bf16, one aligned row of S >= 64 (even) elements per channel, no bias
static bool flat_direct(const Geo &g)
{
    const bool flat = (g.kh == 1 && g.kw == 1 && g.stride == 1 && g.pad == 0);
    return g.bf16 && flat && !g.has_bias && (g.oh * g.ow) % 2 == 0 && g.oh * g.ow >= 64;
}

static FullPlan full_plan(const Geo &g, int mode)
{
    FullPlan p;
    const int crowd = plan_crowd();                  // 0, or the 128x128x64 chunks of work a workgroup should get
    const int J = g.cin * g.kh * g.kw;
    const int S = g.oh * g.ow;
    const bool flat = (g.kh == 1 && g.kw == 1 && g.stride == 1 && g.pad == 0);
    p.h = flat ? 1 : g.h; p.w = flat ? S : g.w; p.oh = flat ? 1 : g.oh; p.ow = flat ? S : g.ow;
    const int epp = g.bf16 ? 8 : 4, kc = g.bf16 ? 64 : 32;
    p.kcolsp = (p.ow + epp - 1) / epp * epp;
    p.chunks_per_ex = (int)(((long long)p.oh * p.kcolsp + kc - 1) / kc);

    p.shape = (g.cout > 64 && J > 64) ? T128 : T64;
    if (p.shape == T128 && mode != MODE_WEIGHTED && p.chunks_per_ex >= 8 && !crowd) {
        // long K and few 128x128 tiles: 64x64 tiles give four times the (example, tile) units, so K
        // needs no (or less) slicing and far fewer partial tiles travel through the workspace
        const long long t128 = (long long)((g.cout + 127) / 128) * ((J + 127) / 128);
        if ((long long)g.n * t128 < 512) p.shape = T64;
    }
    // 256 x 128 tiles, eight waves, three stages, one workgroup per compute unit: the per-example form of aligned 1x1
    // layers with short K (at most 7 chunks: never sliced below) whose tiles are all whole, when the layer still has
    // a few hundred (example, tile) units
    if (p.shape == T128 && mode != MODE_WEIGHTED && flat_direct(g) && g.cout % 256 == 0 && J % 128 == 0 && p.chunks_per_ex <= 7 &&
        (long long)g.n * (g.cout / 256) * (J / 128) >= 128)
        p.shape = T256x128;
    // whole rows travelling in blocks of 32 (conv_panel_kernel): the same layers when their rows are short and of the
    // length that kernel's LDS layout wants, and output tiles of 256 x 256 are all whole
    const bool panel = mode != MODE_WEIGHTED && flat_direct(g) && S % 8 == 4 && S > 16 * (PANEL_KS - 1) && S <= 16 * PANEL_KS &&
                       g.cout % 256 == 0 && J % 256 == 0 && (long long)g.n * (g.cout / 256) * (J / 256) >= 128;
    if (panel) p.shape = T256rows;
    p.tiles_m = (g.cout + kTileM[p.shape] - 1) / kTileM[p.shape];
    p.tiles_n = (J + kTileN[p.shape] - 1) / kTileN[p.shape];
    const int tiles = p.tiles_m * p.tiles_n;
    const int per_wave_tiles = (p.shape == T64) ? 1 : 4;
    p.nacc = per_wave_tiles + (g.has_bias ? (p.shape == T64 ? 1 : 2) : 0);
    const size_t tile_floats = (size_t)p.nacc * 16 * THREADS;

    p.ksplit = 1; p.chunks_per_split = p.chunks_per_ex; p.ex_per_split = g.n; p.ex_per_wg = 1;
    if (mode == MODE_WEIGHTED) {
        // example ranges: enough workgroups to fill the chip, with the partial tiles that are
        // written and read back (cache-resident in practice) kept below ~100 MB
        long long want = (512 + tiles - 1) / tiles;
        if (crowd) {                                     // example ranges of about twice the target
            const long long per = (long long)2 * crowd * (p.shape == T64 ? 4 : 1);
            want = ((long long)g.n * p.chunks_per_ex + per - 1) / per;
        }
        const long long cap = (long long)(96.0e6 / (4.0 * (double)tiles * (double)tile_floats));
        if (want > cap) want = cap;
        if (want > g.n) want = g.n;
        if (want < 1) want = 1;
        p.ex_per_split = (int)((g.n + want - 1) / want);
        p.ksplit = (g.n + p.ex_per_split - 1) / p.ex_per_split;
        p.groups = tiles;
    } else {
        const long long units = (long long)g.n * tiles;
        if (p.shape == T256rows) {
            // a unit (example, tile) is sixteen blocks; several in a row hide the filling of the ring (measured: 1, 2, 4 within 4 %)
            long long e = crowd ? 4 : (units + 511) / 512;
            if (e > 4) e = 4;
            if (e > g.n) e = g.n;
            p.ex_per_wg = (int)(e < 1 ? 1 : e);
        } else if (crowd) {
            // chunks of this tile shape per workgroup (a 256 x 128 chunk is two units of work; at least 8 of them, so
            // that K is not sliced)
            const int tgt = p.shape == T256x128 ? (crowd / 2 > 8 ? crowd / 2 : 8) : crowd * (p.shape == T64 ? 4 : 1);
            if (p.chunks_per_ex > tgt + tgt / 2) {
                const long long want = (p.chunks_per_ex + tgt - 1) / tgt;
                p.chunks_per_split = (int)((p.chunks_per_ex + want - 1) / want);
                p.ksplit = (p.chunks_per_ex + p.chunks_per_split - 1) / p.chunks_per_split;
            } else {
                // short K: a workgroup takes several examples in a row (its loads stream across the boundaries)
                long long e = (tgt + p.chunks_per_ex / 2) / p.chunks_per_ex;
                if (e > 16) e = 16;
                if (e > g.n) e = g.n;
                p.ex_per_wg = (int)(e < 1 ? 1 : e);
            }
        } else if (units < 512 && p.chunks_per_ex >= 8) {
            // few tiles, long K: slice K so that about 256 workgroups run (one per CU: measured best when several
            // layers share the chip; more slices mean more partial tiles through the workspace)
            long long want = 256 / units;
            const long long by_length = (p.chunks_per_ex + 23) / 24;      // and no workgroup walks more than ~24 chunks
            if (want < by_length) want = by_length;
            if (want > p.chunks_per_ex / 4) want = p.chunks_per_ex / 4;
            if (want < 1) want = 1;
            p.chunks_per_split = (int)((p.chunks_per_ex + want - 1) / want);
            p.ksplit = (p.chunks_per_ex + p.chunks_per_split - 1) / p.chunks_per_split;
        } else if (units > 768 && p.chunks_per_ex <= 4) {
            // short K, many tiles: one round of ~512 workgroups that each stream several examples
            // (loads run ahead across example boundaries) beats several rounds of short ones
            long long e = (units + 511) / 512;
            if (e > 8) e = 8;
            if (e > g.n) e = g.n;
            p.ex_per_wg = (int)(e < 1 ? 1 : e);
        }
        p.groups = g.n * tiles;
    }
    p.part_floats = (p.ksplit > 1) ? (size_t)p.groups * p.ksplit * tile_floats : 0;
    return p;
}

// Clip-weighted contraction of a bf16 layer whose packed operands are small: rewrite the
// operands first (pack.hip) and run the aligned one-long-row variant on `g2`, the geometry of
// the packed tensors (example ranges as its "examples", im2col rows as its input channels).
static bool packed_weighted(const Geo &g, int mode, PackPlan &pp, Geo &g2)
{
    if (mode != MODE_WEIGHTED || !g.bf16) return false;
    // a 1x1 stride-1 layer with even S is already K-contiguous and dword aligned: the aligned loader reads it
    // in place and scales dY while staging, which beats packing it first (measured)
    if (g.kh == 1 && g.kw == 1 && g.stride == 1 && g.pad == 0 && (g.oh * g.ow) % 2 == 0) return false;
    const long long J = (long long)g.cin * g.kh * g.kw;
    const int shape = (g.cout > 64 && J > 64) ? T128 : T64;
    const long long tiles = (long long)((g.cout + kTileM[shape] - 1) / kTileM[shape]) * ((J + kTileN[shape] - 1) / kTileN[shape]);
    long long groups = (256 + tiles - 1) / tiles;
    if (plan_crowd()) {
        // sharing the launch with other layers: example ranges of about twice the target number of chunks
        const long long sp = ((long long)g.oh * g.ow + 7) / 8 * 8;
        const long long per = (long long)2 * plan_crowd() * (shape == T64 ? 4 : 1) * 64;
        groups = ((long long)g.n * sp + per - 1) / per;
    }
    if (groups > g.n) groups = g.n;
    if (groups < 1) groups = 1;
    pp = pack_plan(g, (int)groups);
    if (pp.x_bytes + pp.dy_bytes > ((size_t)64 << 20)) return false;
    if ((long long)J * pp.kg >= (1ll << 31) || (long long)g.cout * pp.kg >= (1ll << 31)) return false;
    g2 = g;
    g2.n = pp.groups;
    g2.cin = (int)J;
    g2.h = 1; g2.w = pp.kg; g2.oh = 1; g2.ow = pp.kg;
    g2.kh = 1; g2.kw = 1; g2.stride = 1; g2.pad = 0;
    g2.x_elems = (size_t)J * pp.kg;
    g2.dy_elems = (size_t)g.cout * pp.kg;
    return true;
}

// Per-example calls of strided 1x1 bf16 convolutions (projection shortcuts): contract on a compact
// copy of the sampled positions of X (pack.hip) with the stride-1 loaders.
static bool subsampled(const Geo &g, int mode, Geo &g2)
{
    if (mode == MODE_WEIGHTED || !g.bf16) return false;
    if (g.kh != 1 || g.kw != 1 || g.stride < 2 || g.pad != 0) return false;
    const size_t s = (size_t)g.oh * g.ow;
    if ((size_t)g.n * g.cin * s * 2 > ((size_t)96 << 20) || g.cin * s < 512) return false;
    g2 = g;
    g2.h = g.oh; g2.w = g.ow; g2.stride = 1;
    g2.x_elems = (size_t)g.cin * s;
    // odd rows would go through the gather loader anyway (no gain) unless the norm-only call can then take
    // the Gram route
    if (s % 2 && !gram_norm_applicable(g2, mode)) return false;
    return true;
}

// workspace: [partial squared norms (per-example mode)] [partial tiles]
static size_t align16(size_t b) { return (b + 15) & ~(size_t)15; }

// partial squared norms per example: one per tile, or one per fixup workgroup when K is sliced
static size_t norm_partials_per_example(const FullPlan &f)
{
    const size_t tiles = (size_t)f.tiles_m * f.tiles_n;
    return f.ksplit > 1 ? tiles * f.nacc * FIX_PARTS : tiles * ((f.shape == T256x128 || f.shape == T256rows) ? 8 : 4);     // unsliced: a slot per wave
}
static size_t norm_partials(const Geo &g, const FullPlan &f) { return (size_t)g.n * norm_partials_per_example(f); }

// Exact workspace need of the kernels that (g, mode) is dispatched to.
static size_t conv_ws_bytes_mode(const Geo &g, int mode);

// One per-example workspace serves norm-only and materialising calls (they may take different routes).
size_t conv_ws_bytes(const Geo &g, int mode)
{
    size_t need = 0;
    const int saved = tl_forced_crowd;
    for (int crowd = 0; crowd <= 4; crowd += 4) {   // a call alone and a call inside a batch (smallest target: most slices)
        tl_forced_crowd = crowd;
        size_t b = conv_ws_bytes_mode(g, mode == MODE_WEIGHTED ? MODE_WEIGHTED : MODE_NORM);
        if (mode != MODE_WEIGHTED) {
            const size_t m = conv_ws_bytes_mode(g, MODE_MATERIALISE);
            if (m > b) b = m;
        }
        if (b > need) need = b;
    }
    tl_forced_crowd = saved;
    return need;
}

static size_t conv_ws_bytes_mode(const Geo &g, int mode)
{
    if (stem_applicable(g, mode)) return stem_ws_bytes(g);
    if (gram_norm_applicable(g, mode)) return gram_ws_bytes(g);
    if (conv3x3_applicable(g, mode)) return conv3x3_ws_bytes(g, mode);
    PackPlan pp;
    Geo g2;
    if (packed_weighted(g, mode, pp, g2)) {
        const FullPlan f = full_plan(g2, mode);
        return align16(pp.x_bytes) + align16(pp.dy_bytes) + (f.ksplit > 1 ? f.part_floats * sizeof(float) : 0);
    }
    if (subsampled(g, mode, g2)) return conv_ws_bytes_mode(g2, mode) + align16(g2.x_elems * g.n * 2);
    const FullPlan f = full_plan(g, mode);
    size_t b = 0;
    if (mode != MODE_WEIGHTED) b += align16(norm_partials(g, f) * sizeof(float));
    if (f.ksplit > 1) b += f.part_floats * sizeof(float);
    return b;
}

size_t conv_norm_partial_count(const Geo &g, int mode)
{
    if (stem_applicable(g, mode)) return stem_norm_partial_count();
    if (gram_norm_applicable(g, mode)) return gram_norm_partial_count();
    if (conv3x3_applicable(g, mode)) return conv3x3_norm_partial_count(g);
    Geo g2;
    if (subsampled(g, mode, g2)) return conv_norm_partial_count(g2, mode);
    return norm_partials_per_example(full_plan(g, mode));
}

// loader of the contraction kernel for a geometry as the kernel sees it
static int loader_of(const Geo &g)
{
    const bool flat = (g.kh == 1 && g.kw == 1 && g.stride == 1 && g.pad == 0);
    return (flat && (!g.bf16 || (g.oh * g.ow) % 2 == 0)) ? 0 : (g.stride == 2 ? 2 : 1);
}

// `shared` = as planned inside a batch call (the launch is shared with other layers).  Two layers with the
// same name run the same kernel instantiation, so a batch call puts them into one launch.
const char *conv_variant_name(const Geo &g, int mode, bool shared)
{
    const int saved = tl_forced_crowd;
    tl_forced_crowd = shared ? 32 : 0;
    struct Restore { int v; ~Restore() { tl_forced_crowd = v; } } restore{saved};
    c3_set_forced_crowd(shared ? 32 : 0);
    struct Restore3 { ~Restore3() { c3_set_forced_crowd(-1); } } restore3;
    if (stem_applicable(g, mode)) return "conv_stem7x7<bf16,per_example>";
    if (gram_norm_applicable(g, mode)) return "conv_gram_norm<bf16>";
    if (conv3x3_applicable(g, mode)) return conv3x3_variant_name(g, mode);
    struct Names {
        char v[2][4][2][2][3][72];
        Names()
        {
            static const char *const ld[3] = {"", ",gather", ",gather2"};
            for (int b = 0; b < 2; ++b)
                for (int s = 0; s < 4; ++s)
                    for (int w = 0; w < 2; ++w)
                        for (int bi = 0; bi < 2; ++bi)
                            for (int l = 0; l < 3; ++l)
                                snprintf(v[b][s][w][bi][l], 72, "conv_contract<%s,%s,%s%s%s>", b ? "bf16" : "f32", kTileName[s],
                                         w ? "weighted" : "per_example", bi ? ",bias" : "", ld[l]);
        }
    };
    static const Names names;               // initialised once, thread-safe
    // the geometry the contraction kernel really sees (packed or subsampled operands are one long aligned row)
    Geo ge = g, g2;
    PackPlan pp;
    if (packed_weighted(g, mode, pp, g2)) ge = g2;
    else if (subsampled(g, mode, g2)) ge = g2;
    const FullPlan f = full_plan(ge, mode);
    return names.v[g.bf16 ? 1 : 0][f.shape][mode == MODE_WEIGHTED ? 1 : 0][g.has_bias ? 1 : 0][loader_of(ge)];
}

template <int WM, int WN, int TM, int TN>
static const void *fixup_of(bool weighted, bool bias)
{
    if (weighted) {
        if (bias) return reinterpret_cast<const void *>(&conv_fixup_kernel<WM, WN, TM, TN, true, true>);
        return reinterpret_cast<const void *>(&conv_fixup_kernel<WM, WN, TM, TN, true, false>);
    }
    if (bias) return reinterpret_cast<const void *>(&conv_fixup_kernel<WM, WN, TM, TN, false, true>);
    return reinterpret_cast<const void *>(&conv_fixup_kernel<WM, WN, TM, TN, false, false>);
}

template <bool BF16, int WM, int WN, int TM, int TN, int SIMPLE>
static const void *kernel_of2(bool weighted, bool bias)
{
    if (weighted) {
        if (bias) return reinterpret_cast<const void *>(&conv_contract_kernel<BF16, WM, WN, TM, TN, true, true, SIMPLE>);
        return reinterpret_cast<const void *>(&conv_contract_kernel<BF16, WM, WN, TM, TN, true, false, SIMPLE>);
    }
    if (bias) return reinterpret_cast<const void *>(&conv_contract_kernel<BF16, WM, WN, TM, TN, false, true, SIMPLE>);
    return reinterpret_cast<const void *>(&conv_contract_kernel<BF16, WM, WN, TM, TN, false, false, SIMPLE>);
}

template <bool BF16, int WM, int WN, int TM, int TN>
static const void *kernel_of(int loader, bool weighted, bool bias)
{
    if (loader == 0) return kernel_of2<BF16, WM, WN, TM, TN, 0>(weighted, bias);
    if (loader == 1) return kernel_of2<BF16, WM, WN, TM, TN, 1>(weighted, bias);
    return kernel_of2<BF16, WM, WN, TM, TN, 2>(weighted, bias);
}

static dp_status launch_conv_impl(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                                  size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c,
                                  void *ws, hipStream_t s, int unit = 0);

// The plan of the clip-weighted kernel with one example range per clipping unit.
static FullPlan unit_plan(const Geo &g, int unit)
{
    FullPlan f = full_plan(g, MODE_WEIGHTED);
    const int tiles = f.tiles_m * f.tiles_n;
    // a range is a whole unit, unless that leaves too few workgroups walking too long: then the largest divisor
    // of the unit that gives about 256 of them (down to one example per range)
    int e = unit;
    while (e > 1 && (long long)tiles * (g.n / e) < 256 && (long long)e * f.chunks_per_ex > 32) {
        int d = e - 1;
        while (unit % d) --d;
        e = d;
    }
    f.ex_per_split = e;
    f.ksplit = g.n / e;
    f.groups = tiles;
    f.part_floats = (size_t)tiles * f.ksplit * f.nacc * 16 * THREADS;
    return f;
}

size_t conv_unit_ws_bytes(const Geo &g, int unit)
{
    if (conv3x3_applicable(g, MODE_WEIGHTED)) return conv3x3_unit_ws_bytes(g, unit);
    const FullPlan f = unit_plan(g, unit);
    const size_t units = (size_t)(g.n / unit), tiles = (size_t)f.tiles_m * f.tiles_n;
    return align16(units * tiles * f.nacc * FIX_PARTS * sizeof(float)) + f.part_floats * sizeof(float);
}

// partial squared norms per unit left at the start of the workspace by a call with clipping units
size_t conv_unit_norm_partial_count(const Geo &g, int unit)
{
    if (conv3x3_applicable(g, MODE_WEIGHTED)) return conv3x3_unit_norm_partial_count(g);
    const FullPlan f = unit_plan(g, unit);
    return (size_t)f.tiles_m * f.tiles_n * f.nacc * FIX_PARTS;
}

// Sums of the per-example gradients over clipping units of `unit` consecutive examples, and their squared norms:
// the clip-weighted kernel with factor 1 and one example range per unit (K runs over the unit's examples and
// positions), whose slices the per-example slice-sum kernel then treats as "examples".
dp_status launch_conv_units(const Geo &g, int unit, const void *x, const void *dy, float *out_w, float *out_b,
                            size_t out_stride, float *sqnorm, void *ws, hipStream_t s)
{
    const int mode = out_w ? MODE_MATERIALISE : MODE_NORM;
    if (conv3x3_applicable(g, MODE_WEIGHTED))
        return launch_conv3x3(g, mode, x, dy, out_w, out_stride, sqnorm, nullptr, 0.0f, ws, s, unit);
    return launch_conv_impl(g, mode, x, dy, out_w, out_b, out_stride, sqnorm, nullptr, 0.0f, ws, s, unit);
}

dp_status launch_conv(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                      size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c, void *ws,
                      hipStream_t s)
{
    if (stem_applicable(g, mode)) return launch_stem(g, x, dy, out_w, out_stride, sqnorm, ws, s);
    if (gram_norm_applicable(g, mode)) return launch_gram_norm(g, x, dy, sqnorm, ws, s);
    if (conv3x3_applicable(g, mode))
        return launch_conv3x3(g, mode, x, dy, out_w, out_stride, sqnorm, group_sqnorm, clip_c, ws, s);
    PackPlan pp;
    Geo g2;
    if (packed_weighted(g, mode, pp, g2)) {
        char *w = static_cast<char *>(ws);
        void *xp = w;
        w += align16(pp.x_bytes);
        void *dyp = w;
        w += align16(pp.dy_bytes);
        const dp_status st = launch_pack_weighted(g, pp, x, dy, group_sqnorm, clip_c, xp, dyp, s);
        if (st != DP_OK) return st;
        // the factors are already in dYp: an infinite bound makes the kernel's own factor 1
        return launch_conv_impl(g2, mode, xp, dyp, out_w, out_b, out_stride, nullptr, group_sqnorm,
                                __builtin_inff(), w, s);
    }
    if (subsampled(g, mode, g2)) {
        // the sub-problem's own workspace comes first (its partial norms stay at the start), the copy of X after it
        void *xs = static_cast<char *>(ws) + conv_ws_bytes_mode(g2, mode);
        const dp_status st = launch_subsample(g, x, xs, s);
        if (st != DP_OK) return st;
        if (gram_norm_applicable(g2, mode)) return launch_gram_norm(g2, xs, dy, sqnorm, ws, s);
        return launch_conv_impl(g2, mode, xs, dy, out_w, out_b, out_stride, sqnorm, group_sqnorm, clip_c, ws, s);
    }
    return launch_conv_impl(g, mode, x, dy, out_w, out_b, out_stride, sqnorm, group_sqnorm, clip_c, ws, s);
}

static dp_status launch_conv_impl(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                                  size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c,
                                  void *ws, hipStream_t s, int unit)
{
    // unit > 0: `mode` says whether the unit sums are stored; the kernel that runs is the weighted one
    const FullPlan f = unit ? unit_plan(g, unit) : full_plan(g, mode);
    const bool weighted = mode == MODE_WEIGHTED || unit > 0;
    ConvArgs a;
    a.unit_major = unit ? unit / f.ex_per_split : 0;
    a.x = x; a.dy = dy;
    a.n = g.n; a.cin = g.cin; a.cout = g.cout; a.h = f.h; a.w = f.w; a.kh = g.kh; a.kw = g.kw;
    a.stride = g.stride; a.pad = g.pad; a.oh = f.oh; a.ow = f.ow;
    a.J = g.cin * g.kh * g.kw;
    a.S = g.oh * g.ow;
    a.tiles_m = f.tiles_m; a.tiles_n = f.tiles_n;
    a.kcolsp = f.kcolsp; a.chunks_per_ex = f.chunks_per_ex;
    a.ksplit = f.ksplit; a.chunks_per_split = f.chunks_per_split;
    a.ex_per_split = f.ex_per_split; a.ex_per_wg = f.ex_per_wg;
    a.group_sqnorm = group_sqnorm; a.clip_c = clip_c;
    a.out_w = out_w; a.out_b = out_b;
    a.out_stride_w = out_stride ? out_stride : g.pw;
    a.out_stride_b = out_stride ? out_stride : g.pb;
    const int tiles = f.tiles_m * f.tiles_n;
    char *w = static_cast<char *>(ws);
    a.partials = nullptr;
    const size_t unit_partials = (size_t)tiles * f.nacc * FIX_PARTS;      // per unit, from the slice-sum kernel
    if (!weighted) {
        a.partials = reinterpret_cast<float *>(w);
        w += align16(norm_partials(g, f) * sizeof(float));
    } else if (unit) {
        a.partials = reinterpret_cast<float *>(w);
        w += align16((size_t)(g.n / unit) * unit_partials * sizeof(float));
    }
    a.ws_part = (f.ksplit > 1 || unit) ? reinterpret_cast<float *>(w) : nullptr;
    long long total;
    if (weighted) total = (long long)tiles * f.ksplit;
    else total = (long long)((g.n + f.ex_per_wg - 1) / f.ex_per_wg) * tiles * f.ksplit;
    const unsigned blocks = (unsigned)(((total + 7) / 8) * 8);
    const bool bias = g.has_bias != 0;
    const int loader = loader_of(g);
    a.force_slow = (g.stride > 2) ? 1 : 0;
    const void *fn;
    unsigned lds_bytes = 0;
    if (g.bf16 && loader == 0 && !bias && a.S >= 64) {
        // aligned one-row-per-channel geometry: operands go global -> LDS directly.  Two workgroups per compute unit
        // (64 KB of LDS each): 64x64 tiles four stages deep, 128x128 tiles two stages deep (measured: a second
        // resident workgroup hides more than two more stages do).
        if (f.shape == T256rows) {                         // per-example form only (full_plan)
            fn = reinterpret_cast<const void *>(&conv_panel_kernel<PANEL_KS>);
            lds_bytes = (unsigned)PANEL_RING * (64u * (unsigned)a.S + 64u) + 8u * 64u;      // ring + each wave's marks
        } else if (f.shape == T256x128) {                  // per-example form only (full_plan)
            fn = reinterpret_cast<const void *>(&conv_flat_kernel<4, 2, 2, false, 3>);
            lds_bytes = 3 * 384 * 128;
        } else if (f.shape == T64) {
            fn = weighted ? reinterpret_cast<const void *>(&conv_flat_kernel<2, 1, 1, true, 4>) : reinterpret_cast<const void *>(&conv_flat_kernel<2, 1, 1, false, 4>);
            lds_bytes = 4 * 128 * 128;
        } else {
            fn = weighted ? reinterpret_cast<const void *>(&conv_flat_kernel<2, 2, 2, true, 2>) : reinterpret_cast<const void *>(&conv_flat_kernel<2, 2, 2, false, 2>);
            lds_bytes = 2 * 256 * 128;
        }
        static std::atomic<bool> attr_done[4][2];        // zero-initialised; setting the attribute twice is harmless
        if (!attr_done[f.shape][weighted ? 1 : 0].load()) {
            // the row-panel kernel's ring grows with S: reserve for the longest row it takes
            const unsigned reserve = f.shape == T256rows ? (unsigned)PANEL_RING * (64u * 16u * PANEL_KS + 64u) + 8u * 64u : lds_bytes;
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)reserve) != hipSuccess)
                return fail(DP_ERR_DEVICE, "conv_flat: cannot reserve %u bytes of LDS", lds_bytes);
            attr_done[f.shape][weighted ? 1 : 0].store(true);
        }
    } else if (g.bf16) fn = (f.shape == T64) ? kernel_of<true, 2, 2, 1, 1>(loader, weighted, bias) : kernel_of<true, 2, 2, 2, 2>(loader, weighted, bias);
    else fn = (f.shape == T64) ? kernel_of<false, 2, 2, 1, 1>(loader, weighted, bias) : kernel_of<false, 2, 2, 2, 2>(loader, weighted, bias);
    dp_status st = submit_main<ConvArgs>(fn, a, blocks, (f.shape == T256x128 || f.shape == T256rows) ? 512 : THREADS, lds_bytes, s, "conv_contract");
    if (st != DP_OK) return st;
    // what follows the main kernel: at once, or after the grouped launches of a batch call
    if (unit) {
        // every unit's slice is finished like an unsliced example: stored (if wanted) and squared
        ConvArgs u = a;
        u.n = g.n / unit; u.ksplit = a.unit_major;
        const unsigned fix_blocks = (unsigned)((size_t)u.n * unit_partials);
        const void *fix = (f.shape == T64) ? fixup_of<2, 2, 1, 1>(false, bias) : fixup_of<2, 2, 2, 2>(false, bias);
        st = submit_kernel<ConvArgs>(TIER_POST, fix, u, fix_blocks, THREADS, 0, s, "conv_fixup");
        if (st != DP_OK || !sqnorm) return st;
        const float *partials = a.partials;
        const int units = u.n, per = (int)unit_partials;
        return submit_post([=]() -> dp_status { return launch_sum_partials(partials, units, per, sqnorm, s); });
    }
    if (f.ksplit > 1) {
        const unsigned fix_blocks = (unsigned)(f.groups * f.nacc * FIX_PARTS);
        const void *fix = (f.shape == T64) ? fixup_of<2, 2, 1, 1>(weighted, bias) : fixup_of<2, 2, 2, 2>(weighted, bias);
        st = submit_kernel<ConvArgs>(TIER_POST, fix, a, fix_blocks, THREADS, 0, s, "conv_fixup");
        if (st != DP_OK) return st;
    }
    if (weighted || !sqnorm) return DP_OK;
    const int per_example = (int)norm_partials_per_example(f), n = g.n;
    const float *partials = a.partials;
    return submit_post([=]() -> dp_status { return launch_sum_partials(partials, n, per_example, sqnorm, s); });
}

}  // namespace dp

