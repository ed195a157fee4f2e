// Register-level helpers shared by the contraction kernels (gfx950): operand vector types, the
// two-step "piece" loader (whole-dword loads, then funnel shift / de-interleave / edge mask in
// registers) and the clip-factor scaling of staged values.
#pragma once

#include "internal.h"

namespace dp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));   // 16 bytes, dword aligned

template <bool BF16> struct ElemTraits;
template <> struct ElemTraits<true> {
    typedef uint16_t type;
    static constexpr int KC = 64;      // elements per K-chunk (128 bytes)
    static constexpr int EPP = 8;      // elements per 16-byte piece
};
template <> struct ElemTraits<false> {
    typedef float type;
    static constexpr int KC = 32;
    static constexpr int EPP = 4;
};

__device__ __forceinline__ uint32_t funnel(uint32_t hi, uint32_t lo, uint32_t bits)
{
    // v_alignbit_b32: the low 32 bits of {hi, lo} >> bits (bits < 32).  The builtin keeps the two
    // dwords separate values; written as a 64-bit shift, the compiler merges their loads from a
    // register array into overlapping 8-byte accesses and the array ends up in scratch.
    return __builtin_amdgcn_alignbit(hi, lo, bits);
}

// Keep elements lo <= i < hi of a piece, zero the rest (an empty range zeroes everything).
template <bool BF16>
__device__ __forceinline__ void mask_piece(uint32_t (&v)[4], int lo, int hi)
{
    constexpr int EPP = ElemTraits<BF16>::EPP;
    if (lo <= 0 && hi >= EPP) return;
    const int l = min(max(lo, 0), EPP), h = min(max(hi, l), EPP);
    const uint32_t bits = ((1u << h) - 1u) & ~((1u << l) - 1u);
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        if constexpr (BF16) {
            const uint32_t m = ((bits >> (2 * d)) & 1u ? 0x0000FFFFu : 0u) | ((bits >> (2 * d + 1)) & 1u ? 0xFFFF0000u : 0u);
            v[d] &= m;
        } else {
            if (!((bits >> d) & 1u)) v[d] = 0u;
        }
    }
}

// One 16-byte piece = elements src[i * STRIDE], i in [lo, hi) (others zero), packed K-contiguous.
// It is produced in two steps so that every load of a chunk is in flight before any is used:
//   piece_load : whole dwords around the run -- one dword-aligned 16-byte load plus the next
//                dword for stride 1 (the run may start on an odd bf16), two 16-byte loads for
//                stride 2.  No branches.  Up to 32 bytes from the run's start are touched: the
//                caller only uses this where that stays inside the tensor, and passes a harmless
//                address when the piece is empty.
//   piece_finish : funnel shift / de-interleave and the edge mask, in registers.
template <bool BF16, int STRIDE> constexpr int raw_n() { return (STRIDE == 1) ? (BF16 ? 5 : 4) : 8; }
template <int N> struct Raw { uint32_t d[N]; };

template <bool BF16, int STRIDE>
__device__ __forceinline__ Raw<raw_n<BF16, STRIDE>()> piece_load(const typename ElemTraits<BF16>::type *src)
{
    Raw<raw_n<BF16, STRIDE>()> out;
    uint32_t *raw = out.d;
    uintptr_t addr = reinterpret_cast<uintptr_t>(src);
    if constexpr (BF16) addr &= ~(uintptr_t)3;                      // dword aligned; bit 1 of src is the shift
    const uint32_t *pw = reinterpret_cast<const uint32_t *>(addr);
    const u32x4_a4 a = *reinterpret_cast<const u32x4_a4 *>(pw);
    raw[0] = a.x; raw[1] = a.y; raw[2] = a.z; raw[3] = a.w;
    if constexpr (STRIDE == 1) {
        if constexpr (BF16) raw[4] = pw[4];
    } else {
        const u32x4_a4 b = *reinterpret_cast<const u32x4_a4 *>(pw + 4);
        raw[4] = b.x; raw[5] = b.y; raw[6] = b.z; raw[7] = b.w;
    }
    return out;
}

// The stride-1 bf16 load from a dword pointer (element index of the run's start rounded down
// to even, halved): 16 bytes + the next dword, as plain global loads.
__device__ __forceinline__ Raw<5> piece_load_words(const uint32_t *pw)
{
    Raw<5> out;
    const u32x4_a4 a = *reinterpret_cast<const u32x4_a4 *>(pw);
    out.d[0] = a.x; out.d[1] = a.y; out.d[2] = a.z; out.d[3] = a.w;
    out.d[4] = pw[4];
    return out;
}

template <bool BF16, int STRIDE>
__device__ __forceinline__ void piece_finish(uint32_t (&v)[4], const Raw<raw_n<BF16, STRIDE>()> &in, uint32_t odd,
                                             int lo, int hi)
{
    const uint32_t *raw = in.d;
    if constexpr (BF16) {
        const uint32_t bits = odd * 16u;
        if constexpr (STRIDE == 1) {
            v[0] = funnel(raw[1], raw[0], bits);
            v[1] = funnel(raw[2], raw[1], bits);
            v[2] = funnel(raw[3], raw[2], bits);
            v[3] = funnel(raw[4], raw[3], bits);
        } else {                                                    // low or high halves of 8 dwords
            v[0] = ((raw[0] >> bits) & 0xFFFFu) | ((raw[1] >> bits) << 16);
            v[1] = ((raw[2] >> bits) & 0xFFFFu) | ((raw[3] >> bits) << 16);
            v[2] = ((raw[4] >> bits) & 0xFFFFu) | ((raw[5] >> bits) << 16);
            v[3] = ((raw[6] >> bits) & 0xFFFFu) | ((raw[7] >> bits) << 16);
        }
    } else {
        if constexpr (STRIDE == 1) { v[0] = raw[0]; v[1] = raw[1]; v[2] = raw[2]; v[3] = raw[3]; }
        else { v[0] = raw[0]; v[1] = raw[2]; v[2] = raw[4]; v[3] = raw[6]; }
    }
    mask_piece<BF16>(v, lo, hi);
}

template <bool BF16, int N>
__device__ __forceinline__ void scale_regs(uint32_t (&st)[N], float f)
{
#pragma unroll
    for (int d = 0; d < N; ++d) {
        if constexpr (BF16) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            const f32x2 p = {__uint_as_float(st[d] << 16) * f, __uint_as_float(st[d] & 0xFFFF0000u) * f};
            st[d] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));   // nearest-even, one instruction
        } else {
            st[d] = __float_as_uint(__uint_as_float(st[d]) * f);
        }
    }
}

}  // namespace dp
