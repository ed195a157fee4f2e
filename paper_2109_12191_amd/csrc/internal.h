// Internal declarations shared by the translation units of libdp_privatise (gfx950 only).
#pragma once

#include <type_traits>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/dp_privatise.h"

namespace dp {

// ---- error reporting (api.hip) ---------------------------------------------------------
dp_status fail(dp_status code, const char *fmt, ...);
dp_status check_launch(const char *what);

// ---- benchmark timing aid (api.hip): events armed by dp_profile_next_contraction.  A contraction
// launcher calls profile_begin(s) right before and profile_end(s) right after its main kernel.
void profile_begin(hipStream_t s);
void profile_end(hipStream_t s);

// ---- geometry of a validated descriptor ------------------------------------------------
struct Geo {
    int kind, bf16, n;
    int cin, cout, h, w, kh, kw, stride, pad, oh, ow;
    int has_bias, gn_groups;
    float gn_eps;
    int nhwc;               // conv / GroupNorm inputs arrive channels-last; the kernels read a transposed copy
    size_t pw, pb;          // weight / bias parameter counts
    size_t x_elems, dy_elems;   // per example
};

// Contraction modes of the conv / dense kernels.
enum Mode { MODE_NORM = 0, MODE_MATERIALISE = 1, MODE_WEIGHTED = 2 };

size_t conv_ws_bytes(const Geo &g, int mode);
const char *conv_variant_name(const Geo &g, int mode, bool shared);
void c3_set_forced_crowd(int v);      // conv3x3.hip: plan as alone (0), as in a shared launch (1), or by the open batch (-1)
dp_status launch_conv(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                      size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c, void *ws,
                      hipStream_t s);

// 3x3 stride-1 pad-1 bf16 convolutions staged from raw image rows (conv3x3.hip); launch_conv,
// conv_ws_bytes and conv_variant_name route to these when conv3x3_applicable() says so.
bool conv3x3_applicable(const Geo &g, int mode);
size_t conv3x3_ws_bytes(const Geo &g, int mode);
const char *conv3x3_variant_name(const Geo &g, int mode);
dp_status launch_conv3x3(const Geo &g, int mode, const void *x, const void *dy, float *out_w, size_t out_stride,
                         float *sqnorm, const float *group_sqnorm, float clip_c, void *ws, hipStream_t s, int unit = 0);
size_t conv3x3_unit_ws_bytes(const Geo &g, int unit);

// Sums of the per-example gradients over clipping units of `unit` consecutive examples (n a multiple of unit), and
// their squared norms [n / unit]; out_w / out_b rows are units.
size_t conv_unit_ws_bytes(const Geo &g, int unit);
dp_status launch_conv_units(const Geo &g, int unit, const void *x, const void *dy, float *out_w, float *out_b,
                            size_t out_stride, float *sqnorm, void *ws, hipStream_t s);
size_t conv_unit_norm_partial_count(const Geo &g, int unit);
size_t conv3x3_unit_norm_partial_count(const Geo &g);
const float *gn_unit_partials(const Geo &g, const void *ws);
size_t gn_unit_norm_partial_count(const Geo &g);
size_t gn_unit_ws_bytes(const Geo &g, int unit);
dp_status launch_gn_units(const Geo &g, int unit, const void *x, const void *dy, float *out_w, float *out_b,
                          size_t out_stride, float *sqnorm, void *ws, hipStream_t s);

// Packed operands of the clip-weighted contraction (pack.hip): K-contiguous, aligned, dY
// pre-scaled by the clip factors; `groups` example ranges of `eg` examples, rows of `kg` elements.
struct PackPlan {
    int S, SP, J, groups, eg, kg;
    size_t x_bytes, dy_bytes;
};
PackPlan pack_plan(const Geo &g, int groups);
dp_status launch_pack_weighted(const Geo &g, const PackPlan &p, const void *x, const void *dy,
                               const float *group_sqnorm, float clip_c, void *xp, void *dyp, hipStream_t s);

// Partial squared norms per example that a per-example call leaves at the start of its workspace
// ([n, count] floats) when it is told not to reduce them (sqnorm == nullptr).
size_t conv_norm_partial_count(const Geo &g, int mode);
size_t conv3x3_norm_partial_count(const Geo &g);
size_t dense_norm_partial_count(const Geo &g, int mode);
size_t gn_norm_partial_count(const Geo &g);

// [n][positions][channels] -> [n][channels][positions], elements of 2 or 4 bytes (pack.hip): channels-last inputs
dp_status launch_to_channels_first(const void *in, void *out, int n, int positions, int channels, int elem_bytes, hipStream_t s);

// compact copy of the rows / columns a strided 1x1 convolution reads: out[n*cin][OH*OW] (pack.hip)
dp_status launch_subsample(const Geo &g, const void *x, void *out, hipStream_t s);

// Norm-only calls of 1x1 convolutions on small feature maps through two Gram matrices (gram.hip).
// the network's first convolution (7x7, stride 2, pad 3, few input channels): stem.hip
bool stem_applicable(const Geo &g, int mode);
size_t stem_ws_bytes(const Geo &g);
size_t stem_norm_partial_count(void);
dp_status launch_stem(const Geo &g, const void *x, const void *dy, float *out_w, size_t out_stride, float *sqnorm, void *ws,
                      hipStream_t s);
bool gram_norm_applicable(const Geo &g, int mode);
size_t gram_ws_bytes(const Geo &g);
size_t gram_norm_partial_count(void);
dp_status launch_gram_norm(const Geo &g, const void *x, const void *dy, float *sqnorm, void *ws, hipStream_t s);

size_t dense_ws_bytes(const Geo &g, int mode);
dp_status launch_dense(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                       size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c, void *ws,
                       hipStream_t s);

size_t gn_ws_bytes(const Geo &g, int mode);
dp_status launch_gn(const Geo &g, int mode, const void *x, const void *dy, float *out_w, float *out_b,
                    size_t out_stride, float *sqnorm, const float *group_sqnorm, float clip_c, void *ws,
                    hipStream_t s);

// streaming kernels (stream_kernels.hip)
dp_status launch_sum_partials(const float *partials, int n, int per_example, float *sqnorm, hipStream_t s);
dp_status launch_norms(const float *layer_sqnorm, const int32_t *group_of_layer, int n_layers, int n,
                       int n_groups, float *group_sqnorm, hipStream_t s);
dp_status launch_norms_from_partials(const float *const *partials, const int32_t *counts, const int32_t *group_of_layer,
                                     int n_layers, int n, int n_groups, float *group_sqnorm, hipStream_t s);
dp_status launch_layer_norms(const float *const *partials, const int32_t *counts, float *const *out, int n_layers, int n,
                             hipStream_t s);
dp_status launch_clip_factors(const float *sqnorm, float clip_c, int n, float *f, hipStream_t s);
dp_status launch_clip_accumulate(const float *g, size_t stride, const float *sqnorm, float clip_c, int n,
                                 size_t p, float *acc, hipStream_t s);
dp_status launch_clip_accumulate_segments(const float *g, size_t stride, const float *group_sqnorm, const size_t *seg_begin,
                                          const int32_t *seg_group, const float *seg_clip, int n_seg, int n, size_t p,
                                          float *acc, hipStream_t s);
dp_status launch_noise_finalize(const float *acc, float *out, size_t p, float sigma, float clip_total,
                                uint64_t total_batch, uint64_t seed, uint64_t step, uint32_t tensor_id,
                                hipStream_t s);
dp_status launch_example_noise(float *acc, size_t p, float sigma, float clip_total, uint64_t total_batch, uint64_t seed,
                               uint64_t step, uint32_t tensor_id, uint64_t first_example, int count,
                               const uint64_t *step_dev, hipStream_t s);
dp_status launch_noise_finalize_update(const float *acc, float *theta, float *vbuf, float *out, size_t p, float sigma,
                                       float clip_total, uint64_t total_batch, uint64_t seed, uint64_t step,
                                       uint32_t tensor_id, float lr, float momentum, hipStream_t s);
dp_status launch_noise_finalize_flat(const float *acc, float *out, float *theta, float *vbuf, const uint64_t *seg_begin,
                                     const uint64_t *seg_size, const uint32_t *seg_tensor_id, int n_seg, float sigma,
                                     float clip_total, uint64_t total_batch, uint64_t seed, uint64_t step,
                                     const uint64_t *step_dev, float lr, float momentum, hipStream_t s);
dp_status launch_philox_raw(uint32_t *raw, size_t p, uint64_t seed, uint64_t step, uint32_t tensor_id,
                            hipStream_t s);

// ---- device helpers --------------------------------------------------------------------
#if defined(__HIP_DEVICE_COMPILE__) || defined(__HIPCC__)

// min(1, C / sqrt(n2)); 1 for a zero gradient or an infinite bound; 0 for a squared norm that is
// NaN or negative (a broken example contributes nothing instead of passing unclipped).
__device__ __forceinline__ float clip_factor(float n2, float clip_c)
{
    if (n2 == 0.0f) return 1.0f;
    const float r = clip_c / sqrtf(n2);     // +inf / x = +inf -> 1
    return r < 1.0f ? r : (r >= 1.0f ? 1.0f : 0.0f);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// The same sum by data-parallel-primitive moves (no trip through LDS), valid in lane 63 only: an inclusive scan inside
// each row of 16 lanes (shifts by 1, 2, 4, 8 with zeros shifted in), then lane 15 of rows 0 and 2 added into rows 1 and 3,
// then lane 31 into rows 2 and 3.  Fixed order: the same bits every run.
__device__ __forceinline__ float wave_sum_last_lane(float v)
{
    auto moved = [](float x, auto ctrl, auto rows) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                                                     decltype(rows)::value, 0xf, true));
    };
    typedef std::integral_constant<int, 0xf> all_rows;
    v += moved(v, std::integral_constant<int, 0x111>{}, all_rows{});         // row_shr:1
    v += moved(v, std::integral_constant<int, 0x112>{}, all_rows{});         // row_shr:2
    v += moved(v, std::integral_constant<int, 0x114>{}, all_rows{});         // row_shr:4
    v += moved(v, std::integral_constant<int, 0x118>{}, all_rows{});         // row_shr:8
    v += moved(v, std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});   // row_bcast:15 into rows 1, 3
    v += moved(v, std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});   // row_bcast:31 into rows 2, 3
    return v;
}

// Sum over a workgroup of `NW` waves; result valid in every thread.  `red` holds NW floats.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float *red)
{
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[wave] = v;
    __syncthreads();
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < NW; ++i) t += red[i];
    return t;
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b)
{
    return __uint_as_float(((uint32_t)b) << 16);
}

// round to nearest, ties to even (finite inputs)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    const uint32_t u = __float_as_uint(f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

#endif

}  // namespace dp
