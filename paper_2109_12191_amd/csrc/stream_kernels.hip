// Streaming kernels of the privatisation path: norm bookkeeping, clip-scale-accumulate,
// and Philox noise + finalize.  All are HBM-bound by design: 16-byte accesses, one pass.
#include "internal.h"

namespace dp {

// ------------------------------------------------------------------------------------------
// sqnorm[i] = sum_t partials[i, t].  One wavefront per example: lane l adds tiles l, l+64, ...
// in order, then a fixed xor-shuffle tree combines the lanes (same bits on every run).
__global__ void __launch_bounds__(256) sum_partials_kernel(const float *__restrict__ partials, int n,
                                                            int per_example, float *__restrict__ sqnorm)
{
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (i >= n) return;
    const float *p = partials + (size_t)i * per_example;
    float s = 0.0f;
    for (int t = lane; t < per_example; t += 64) s += p[t];
    s = wave_sum(s);
    if (lane == 0) sqnorm[i] = s;
}

dp_status launch_sum_partials(const float *partials, int n, int per_example, float *sqnorm, hipStream_t s)
{
    hipLaunchKernelGGL(sum_partials_kernel, dim3((n + 3) / 4), dim3(256), 0, s, partials, n, per_example, sqnorm);
    return check_launch("sum_partials");
}

// ------------------------------------------------------------------------------------------
// H2: group_sqnorm[g, i] = sum_{l : group_of_layer[l] == g} layer_sqnorm[l, i].  One wavefront
// per (group, example): lane l takes layers l, l+64, ... in order, then the fixed shuffle tree.
__global__ void __launch_bounds__(256) norms_kernel(const float *__restrict__ layer_sqnorm,
                                                     const int32_t *__restrict__ group_of_layer, int n_layers,
                                                     int n, int n_groups, float *__restrict__ group_sqnorm)
{
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.y;
    if (i >= n) return;
    float s = 0.0f;
    for (int l = lane; l < n_layers; l += 64)
        if (group_of_layer[l] == g) s += layer_sqnorm[(size_t)l * n + i];
    s = wave_sum(s);
    if (lane == 0) group_sqnorm[(size_t)g * n + i] = s;
}

dp_status launch_norms(const float *layer_sqnorm, const int32_t *group_of_layer, int n_layers, int n,
                       int n_groups, float *group_sqnorm, hipStream_t s)
{
    hipLaunchKernelGGL(norms_kernel, dim3((n + 3) / 4, n_groups), dim3(256), 0, s, layer_sqnorm, group_of_layer,
                       n_layers, n, n_groups, group_sqnorm);
    return check_launch("norms");
}

// Group norms straight from the per-layer partial sums the contraction kernels leave in their
// workspaces (so that no per-layer reduction launch is needed): one wavefront per (group, example)
// walks the layers of the group in order and, inside a layer, that example's partials 64 at a
// time; fixed order, same bits on every run.
constexpr int NP_MAX = 64;                 // layers per launch
struct NormPartialArgs {
    const float *ptr[NP_MAX];
    int count[NP_MAX];
    int group[NP_MAX];
    int n_layers, n, accumulate;
    float *group_sqnorm;
};

__global__ void __launch_bounds__(256) norms_from_partials_kernel(const NormPartialArgs a)
{
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.y;
    if (i >= a.n) return;
    float s = 0.0f;
    for (int l = 0; l < a.n_layers; ++l) {
        if (a.group[l] != g) continue;
        const int cnt = a.count[l];
        const float *p = a.ptr[l] + (size_t)i * cnt;
        for (int c = lane; c < cnt; c += 64) s += p[c];
    }
    s = wave_sum(s);
    if (lane == 0) {
        float *dst = a.group_sqnorm + (size_t)g * a.n + i;
        *dst = a.accumulate ? *dst + s : s;
    }
}

dp_status launch_norms_from_partials(const float *const *partials, const int32_t *counts, const int32_t *group_of_layer,
                                     int n_layers, int n, int n_groups, float *group_sqnorm, hipStream_t s)
{
    for (int l0 = 0; l0 < n_layers; l0 += NP_MAX) {
        NormPartialArgs a;
        a.n_layers = n_layers - l0 < NP_MAX ? n_layers - l0 : NP_MAX;
        for (int l = 0; l < NP_MAX; ++l) {
            const bool live = l < a.n_layers;
            a.ptr[l] = live ? partials[l0 + l] : nullptr;
            a.count[l] = live ? counts[l0 + l] : 0;
            a.group[l] = live ? group_of_layer[l0 + l] : -1;
        }
        a.n = n; a.accumulate = l0 > 0; a.group_sqnorm = group_sqnorm;
        hipLaunchKernelGGL(norms_from_partials_kernel, dim3((n + 3) / 4, n_groups), dim3(256), 0, s, a);
        const dp_status st = check_launch("norms_from_partials");
        if (st != DP_OK) return st;
    }
    return DP_OK;
}

// Per-layer squared norms of several layers from the partial sums their contraction kernels left in
// their workspaces: out[l][i] = sum_c partials[l][i * count[l] + c].  One wavefront per (layer,
// example), fixed order.  Used by the batch calls: one launch for all their layers.
struct LayerNormArgs {
    const float *ptr[NP_MAX];
    float *out[NP_MAX];
    int count[NP_MAX];
    int n;
};

__global__ void __launch_bounds__(256) layer_norms_kernel(const LayerNormArgs a)
{
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int l = blockIdx.y;
    if (i >= a.n) return;
    const int cnt = a.count[l];
    const float *p = a.ptr[l] + (size_t)i * cnt;
    float s = 0.0f;
    for (int c = lane; c < cnt; c += 64) s += p[c];
    s = wave_sum(s);
    if (lane == 0) a.out[l][i] = s;
}

dp_status launch_layer_norms(const float *const *partials, const int32_t *counts, float *const *out, int n_layers, int n,
                             hipStream_t s)
{
    for (int l0 = 0; l0 < n_layers; l0 += NP_MAX) {
        LayerNormArgs a;
        const int cnt = n_layers - l0 < NP_MAX ? n_layers - l0 : NP_MAX;
        for (int l = 0; l < NP_MAX; ++l) {
            const bool live = l < cnt;
            a.ptr[l] = live ? partials[l0 + l] : nullptr;
            a.out[l] = live ? out[l0 + l] : nullptr;
            a.count[l] = live ? counts[l0 + l] : 0;
        }
        a.n = n;
        hipLaunchKernelGGL(layer_norms_kernel, dim3((n + 3) / 4, cnt), dim3(256), 0, s, a);
        const dp_status st = check_launch("layer_norms");
        if (st != DP_OK) return st;
    }
    return DP_OK;
}

// ------------------------------------------------------------------------------------------
// H3
__global__ void __launch_bounds__(256) clip_factors_kernel(const float *__restrict__ sqnorm, float clip_c, int n,
                                                            float *__restrict__ f)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) f[i] = clip_factor(sqnorm[i], clip_c);
}

dp_status launch_clip_factors(const float *sqnorm, float clip_c, int n, float *f, hipStream_t s)
{
    hipLaunchKernelGGL(clip_factors_kernel, dim3((n + 255) / 256), dim3(256), 0, s, sqnorm, clip_c, n, f);
    return check_launch("clip_factors");
}

// ------------------------------------------------------------------------------------------
// H4 (materialised form): acc[e] += sum_i f_i g[i, e].
// Each thread owns VEC consecutive parameters and walks the examples in order (fixed order =>
// reproducible bits); consecutive threads touch consecutive 16-byte pieces of one example's
// row, so every wave load is a full 1 KiB run.  `stride` is the distance between rows.
constexpr int CA_FMAX = 1024;   // clip factors staged in LDS per pass over the examples

// 16-byte load of data that is read exactly once (the per-example gradient matrix): non-temporal, so the
// stream does not push the accumulator and the clip factors out of the caches (measured: 5.5 -> 6.0 TB/s)
__device__ __forceinline__ float4 load_once(const float *p)
{
    const float4 *q = reinterpret_cast<const float4 *>(p);
    float4 v;
    v.x = __builtin_nontemporal_load(&q->x);
    v.y = __builtin_nontemporal_load(&q->y);
    v.z = __builtin_nontemporal_load(&q->z);
    v.w = __builtin_nontemporal_load(&q->w);
    return v;
}

template <int VEC>
__global__ void __launch_bounds__(256) clip_accumulate_kernel(const float *__restrict__ g, size_t stride,
                                                               const float *__restrict__ sqnorm, float clip_c,
                                                               int n, size_t p, float *__restrict__ acc)
{
    __shared__ float fs[CA_FMAX];
    const size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    float s[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) s[v] = 0.0f;

    for (int base = 0; base < n; base += CA_FMAX) {
        const int cnt = min(CA_FMAX, n - base);
        __syncthreads();
        for (int j = threadIdx.x; j < cnt; j += 256) fs[j] = clip_factor(sqnorm[base + j], clip_c);
        __syncthreads();
        if (e < p) {
            const float *row = g + (size_t)base * stride + e;
            int j = 0;
            if constexpr (VEC == 4) {
                for (; j + 8 <= cnt; j += 8) {        // eight rows' loads in flight per thread
                    float4 v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = load_once(row + (size_t)(j + u) * stride);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {    // example order: same bits on every run
                        const float fu = fs[j + u];
                        s[0] += fu * v[u].x; s[1] += fu * v[u].y; s[2] += fu * v[u].z; s[3] += fu * v[u].w;
                    }
                }
                for (; j < cnt; ++j) {
                    const float4 a = load_once(row + (size_t)j * stride);
                    const float f0 = fs[j];
                    s[0] += f0 * a.x; s[1] += f0 * a.y; s[2] += f0 * a.z; s[3] += f0 * a.w;
                }
            } else {
                for (; j < cnt; ++j) s[0] += fs[j] * row[(size_t)j * stride];
            }
        }
    }
    if (e >= p) return;
    if constexpr (VEC == 4) {
        float4 a = *reinterpret_cast<float4 *>(acc + e);
        a.x += s[0]; a.y += s[1]; a.z += s[2]; a.w += s[3];
        *reinterpret_cast<float4 *>(acc + e) = a;
    } else {
        acc[e] += s[0];
    }
}

// The same sum for several clipping groups in one launch: the columns [0, p) of the gradient matrix are cut
// into segments (one per tensor or per group), each with its own bound and its own row of squared norms.
// A thread finds the segment of its four columns by bisection of the (at most SEG_MAX + 1) boundaries it
// gets as kernel arguments; boundaries are multiples of 4, so a thread never straddles two segments.
constexpr int SEG_MAX = 64;
struct SegArgs {
    unsigned long long begin[SEG_MAX + 1];         // column where each segment starts; begin[n_seg] = p
    float clip[SEG_MAX];
    int group[SEG_MAX];
    int n_seg;
};

__global__ void __launch_bounds__(256) clip_accumulate_segments_kernel(const float *__restrict__ g, size_t stride,
                                                                       const float *__restrict__ group_sqnorm,
                                                                       const SegArgs sa, int n, size_t p,
                                                                       float *__restrict__ acc)
{
    const size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= p) return;
    int lo = 0, hi = sa.n_seg - 1;                 // last segment with begin <= e
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (sa.begin[mid] <= e) lo = mid; else hi = mid - 1;
    }
    const float *sq = group_sqnorm + (size_t)sa.group[lo] * n;
    const float c = sa.clip[lo];
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    const float *row = g + e;
#pragma unroll 8
    for (int i = 0; i < n; ++i) {                  // example order: same bits on every run
        const float f = clip_factor(sq[i], c);
        const float4 v = load_once(row + (size_t)i * stride);
        s0 += f * v.x; s1 += f * v.y; s2 += f * v.z; s3 += f * v.w;
    }
    float4 a = *reinterpret_cast<float4 *>(acc + e);
    a.x += s0; a.y += s1; a.z += s2; a.w += s3;
    *reinterpret_cast<float4 *>(acc + e) = a;
}

dp_status launch_clip_accumulate_segments(const float *g, size_t stride, const float *group_sqnorm, const size_t *seg_begin,
                                          const int32_t *seg_group, const float *seg_clip, int n_seg, int n, size_t p,
                                          float *acc, hipStream_t s)
{
    for (int s0 = 0; s0 < n_seg; s0 += SEG_MAX) {
        SegArgs sa;
        sa.n_seg = n_seg - s0 < SEG_MAX ? n_seg - s0 : SEG_MAX;
        const size_t first = seg_begin[s0], last = (s0 + sa.n_seg == n_seg) ? p : seg_begin[s0 + sa.n_seg];
        for (int k = 0; k < SEG_MAX; ++k) {
            const bool live = k < sa.n_seg;
            sa.begin[k] = live ? seg_begin[s0 + k] - first : last - first;
            sa.clip[k] = live ? seg_clip[s0 + k] : 1.0f;
            sa.group[k] = live ? seg_group[s0 + k] : 0;
        }
        sa.begin[SEG_MAX] = last - first;
        const size_t span = last - first;
        hipLaunchKernelGGL(clip_accumulate_segments_kernel, dim3((unsigned)((span / 4 + 255) / 256)), dim3(256), 0, s,
                           g + first, stride, group_sqnorm, sa, n, span, acc + first);
        const dp_status st = check_launch("clip_accumulate_segments");
        if (st != DP_OK) return st;
    }
    return DP_OK;
}

dp_status launch_clip_accumulate(const float *g, size_t stride, const float *sqnorm, float clip_c, int n, size_t p,
                                 float *acc, hipStream_t s)
{
    const bool vec4 = (p % 4 == 0) && (stride % 4 == 0);
    const size_t threads = vec4 ? p / 4 : p;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    if (vec4)
        hipLaunchKernelGGL(clip_accumulate_kernel<4>, dim3(blocks), dim3(256), 0, s, g, stride, sqnorm, clip_c, n, p,
                           acc);
    else
        hipLaunchKernelGGL(clip_accumulate_kernel<1>, dim3(blocks), dim3(256), 0, s, g, stride, sqnorm, clip_c, n, p,
                           acc);
    return check_launch("clip_accumulate");
}

// ------------------------------------------------------------------------------------------
// H5: Philox4x32-10 (Salmon et al., SC'11) + Box-Muller + finalize.
struct Philox4 { uint32_t x, y, z, w; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1)
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += W0;               // the bump after the last round is unused
        k1 += W1;
    }
    return Philox4{c0, c1, c2, c3};
}

__device__ __forceinline__ float uniform_open(uint32_t r)
{
    return ((float)(r >> 9) + 0.5f) * 1.1920928955078125e-07f;     // 2^-23; exact in fp32, in (0,1)
}

__device__ __forceinline__ void box_muller(uint32_t ra, uint32_t rb, float &z0, float &z1)
{
    const float radius = sqrtf(-2.0f * logf(uniform_open(ra)));
    float sn, cs;
    sincospif(2.0f * uniform_open(rb), &sn, &cs);                   // 2u is exact; argument in (0,2)
    z0 = radius * cs;
    z1 = radius * sn;
}

// One thread per Philox call = 4 consecutive parameters (one 16-byte load, one 16-byte store).
template <bool NOISE>
__global__ void __launch_bounds__(256) noise_finalize_kernel(const float *__restrict__ acc, float *__restrict__ out,
                                                              size_t p, float scale, float inv_batch, uint32_t k0,
                                                              uint32_t k1, uint32_t step_lo, uint32_t tensor_id)
{
    const uint64_t q = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const size_t e = (size_t)q * 4;
    if (e >= p) return;
    float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (NOISE) {
        const Philox4 r = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), tensor_id, step_lo, k0, k1);
        box_muller(r.x, r.y, z[0], z[1]);
        box_muller(r.z, r.w, z[2], z[3]);
    }
    if (e + 4 <= p) {
        const float4 a = *reinterpret_cast<const float4 *>(acc + e);
        float4 o;
        o.x = (a.x + scale * z[0]) * inv_batch;
        o.y = (a.y + scale * z[1]) * inv_batch;
        o.z = (a.z + scale * z[2]) * inv_batch;
        o.w = (a.w + scale * z[3]) * inv_batch;
        *reinterpret_cast<float4 *>(out + e) = o;
    } else {
        for (int j = 0; e + j < p; ++j) out[e + j] = (acc[e + j] + scale * z[j]) * inv_batch;
    }
}

dp_status launch_noise_finalize(const float *acc, float *out, size_t p, float sigma, float clip_total,
                                uint64_t total_batch, uint64_t seed, uint64_t step, uint32_t tensor_id,
                                hipStream_t s)
{
    const size_t calls = (p + 3) / 4;
    const unsigned blocks = (unsigned)((calls + 255) / 256);
    const float scale = sigma * clip_total;
    const float inv_batch = 1.0f / (float)total_batch;
    if (sigma > 0.0f)
        hipLaunchKernelGGL(noise_finalize_kernel<true>, dim3(blocks), dim3(256), 0, s, acc, out, p, scale, inv_batch,
                           (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, tensor_id);
    else
        hipLaunchKernelGGL(noise_finalize_kernel<false>, dim3(blocks), dim3(256), 0, s, acc, out, p, 0.0f, inv_batch,
                           0u, 0u, 0u, 0u);
    return check_launch("noise_finalize");
}

// Per-example form of the noise (second equation of the Algorithm section): acc[e] += scale * sum_j z(j, e)
// over `count` examples starting at `first`; example j's draws use the counter (q, j, tensor_id, step) and the
// key (seed lo, seed hi ^ 0x50455245).  One thread per four parameters; the examples are summed in order.
__global__ void __launch_bounds__(256) example_noise_kernel(float *__restrict__ acc, size_t p, float scale, uint32_t k0,
                                                             uint32_t k1, uint32_t step_arg, uint32_t tensor_id,
                                                             uint32_t first, int count,
                                                             const unsigned long long *__restrict__ step_dev)
{
    const uint64_t q = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const size_t e = (size_t)q * 4;
    if (e >= p) return;
    const uint32_t step_lo = step_dev ? (uint32_t)*step_dev : step_arg;
    float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int j = 0; j < count; ++j) {
        const Philox4 r = philox4x32_10((uint32_t)q, first + (uint32_t)j, tensor_id, step_lo, k0, k1);
        float z[4];
        box_muller(r.x, r.y, z[0], z[1]);
        box_muller(r.z, r.w, z[2], z[3]);
#pragma unroll
        for (int u = 0; u < 4; ++u) sum[u] += z[u];
    }
    if (e + 4 <= p) {
        float4 a = *reinterpret_cast<float4 *>(acc + e);
        a.x += scale * sum[0]; a.y += scale * sum[1]; a.z += scale * sum[2]; a.w += scale * sum[3];
        *reinterpret_cast<float4 *>(acc + e) = a;
    } else {
        for (int u = 0; e + u < p; ++u) acc[e + u] += scale * sum[u];
    }
}

dp_status launch_example_noise(float *acc, size_t p, float sigma, float clip_total, uint64_t total_batch, uint64_t seed,
                               uint64_t step, uint32_t tensor_id, uint64_t first_example, int count,
                               const uint64_t *step_dev, hipStream_t s)
{
    if (sigma == 0.0f) return DP_OK;
    const size_t calls = (p + 3) / 4;
    const float scale = sigma * clip_total / sqrtf((float)total_batch);
    hipLaunchKernelGGL(example_noise_kernel, dim3((unsigned)((calls + 255) / 256)), dim3(256), 0, s, acc, p, scale,
                       (uint32_t)seed, (uint32_t)(seed >> 32) ^ 0x50455245u, (uint32_t)step, tensor_id,
                       (uint32_t)first_example, count, reinterpret_cast<const unsigned long long *>(step_dev));
    return check_launch("example_noise");
}

// H5 fused with the optimiser step that follows it: g = (acc + scale z) / |B| is formed in registers
// and applied at once -- v <- mu v + g, theta <- theta - lr v (v == nullptr: theta <- theta - lr g);
// g is written only if the caller asks for it.  20 bytes per parameter instead of 8 + 20.
template <bool NOISE>
__global__ void __launch_bounds__(256) noise_finalize_update_kernel(const float *__restrict__ acc, float *__restrict__ theta,
                                                                     float *__restrict__ vbuf, float *__restrict__ out,
                                                                     size_t p, float scale, float inv_batch, float lr,
                                                                     float momentum, uint32_t k0, uint32_t k1,
                                                                     uint32_t step_lo, uint32_t tensor_id)
{
    const uint64_t q = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const size_t e = (size_t)q * 4;
    if (e >= p) return;
    float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (NOISE) {
        const Philox4 r = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), tensor_id, step_lo, k0, k1);
        box_muller(r.x, r.y, z[0], z[1]);
        box_muller(r.z, r.w, z[2], z[3]);
    }
    const bool full = e + 4 <= p;
    float a[4], t[4], v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (full) {
        const float4 av = *reinterpret_cast<const float4 *>(acc + e), tv = *reinterpret_cast<const float4 *>(theta + e);
        a[0] = av.x; a[1] = av.y; a[2] = av.z; a[3] = av.w;
        t[0] = tv.x; t[1] = tv.y; t[2] = tv.z; t[3] = tv.w;
        if (vbuf) { const float4 vv = *reinterpret_cast<const float4 *>(vbuf + e); v[0] = vv.x; v[1] = vv.y; v[2] = vv.z; v[3] = vv.w; }
    } else {
        for (int j = 0; j < 4; ++j) {
            const bool ok = e + j < p;
            a[j] = ok ? acc[e + j] : 0.0f;
            t[j] = ok ? theta[e + j] : 0.0f;
            v[j] = (ok && vbuf) ? vbuf[e + j] : 0.0f;
        }
    }
    float g[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        g[j] = (a[j] + scale * z[j]) * inv_batch;
        if (vbuf) { v[j] = momentum * v[j] + g[j]; t[j] -= lr * v[j]; }
        else t[j] -= lr * g[j];
    }
    if (full) {
        *reinterpret_cast<float4 *>(theta + e) = make_float4(t[0], t[1], t[2], t[3]);
        if (vbuf) *reinterpret_cast<float4 *>(vbuf + e) = make_float4(v[0], v[1], v[2], v[3]);
        if (out) *reinterpret_cast<float4 *>(out + e) = make_float4(g[0], g[1], g[2], g[3]);
    } else {
        for (int j = 0; e + j < p; ++j) {
            theta[e + j] = t[j];
            if (vbuf) vbuf[e + j] = v[j];
            if (out) out[e + j] = g[j];
        }
    }
}

dp_status launch_noise_finalize_update(const float *acc, float *theta, float *vbuf, float *out, size_t p, float sigma,
                                       float clip_total, uint64_t total_batch, uint64_t seed, uint64_t step,
                                       uint32_t tensor_id, float lr, float momentum, hipStream_t s)
{
    const size_t calls = (p + 3) / 4;
    const unsigned blocks = (unsigned)((calls + 255) / 256);
    const float inv_batch = 1.0f / (float)total_batch;
    if (sigma > 0.0f)
        hipLaunchKernelGGL(noise_finalize_update_kernel<true>, dim3(blocks), dim3(256), 0, s, acc, theta, vbuf, out, p,
                           sigma * clip_total, inv_batch, lr, momentum, (uint32_t)seed, (uint32_t)(seed >> 32),
                           (uint32_t)step, tensor_id);
    else
        hipLaunchKernelGGL(noise_finalize_update_kernel<false>, dim3(blocks), dim3(256), 0, s, acc, theta, vbuf, out, p,
                           0.0f, inv_batch, lr, momentum, 0u, 0u, 0u, 0u);
    return check_launch("noise_finalize_update");
}

// H5 over a whole flat parameter vector in one launch.  The vector holds several tensors (each starting
// at a multiple of 4 floats, padding after a tensor is left untouched); every tensor keeps its own
// Philox counters (tensor id, element index within the tensor), so the bits are those of one
// dp_add_noise_finalize call per tensor.  A workgroup covers FLAT_BLOCK consecutive elements of ONE
// tensor: it finds its tensor by bisection over the tensors' first-workgroup numbers (uniform, scalar
// loads), so no thread straddles two tensors.  The step may come from a device word, which lets a
// captured graph draw fresh noise on every replay.
constexpr int FLAT_SEG_MAX = 128;
constexpr int FLAT_BLOCK = 1024;                // elements per workgroup: 256 threads x 4
struct FlatArgs {
    unsigned long long begin[FLAT_SEG_MAX];     // first element of tensor k in the flat vector
    unsigned int size[FLAT_SEG_MAX];            // elements of tensor k
    unsigned int first_block[FLAT_SEG_MAX + 1]; // workgroup where tensor k starts; [n_seg] = grid size
    unsigned int tensor_id[FLAT_SEG_MAX];
    int n_seg;
};

template <bool NOISE, bool UPDATE>
__global__ void __launch_bounds__(256) noise_finalize_flat_kernel(const float *__restrict__ acc, float *__restrict__ out,
                                                                   float *__restrict__ theta, float *__restrict__ vbuf,
                                                                   const FlatArgs fa, float scale, float inv_batch, float lr,
                                                                   float momentum, uint32_t k0, uint32_t k1, uint32_t step_lo,
                                                                   const unsigned long long *__restrict__ step_dev)
{
    int lo = 0, hi = fa.n_seg - 1;              // last tensor whose first workgroup is <= blockIdx.x
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (fa.first_block[mid] <= blockIdx.x) lo = mid; else hi = mid - 1;
    }
    const uint32_t size = fa.size[lo];
    const uint32_t q = (blockIdx.x - fa.first_block[lo]) * 256u + threadIdx.x;       // Philox call within the tensor
    const uint32_t e = q * 4u;
    if (e >= size) return;
    const size_t at = (size_t)fa.begin[lo] + e;
    const bool full = e + 4u <= size;
    // the loads go out first; the integer and transcendental work below hides their latency
    float a[4] = {0.0f, 0.0f, 0.0f, 0.0f}, t[4] = {0.0f, 0.0f, 0.0f, 0.0f}, v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (full) {
        const float4 av = load_once(acc + at);            // read once, written once: keep the stream out of the caches
        a[0] = av.x; a[1] = av.y; a[2] = av.z; a[3] = av.w;
        if constexpr (UPDATE) {
            const float4 tv = *reinterpret_cast<const float4 *>(theta + at);
            t[0] = tv.x; t[1] = tv.y; t[2] = tv.z; t[3] = tv.w;
            if (vbuf) { const float4 vv = *reinterpret_cast<const float4 *>(vbuf + at); v[0] = vv.x; v[1] = vv.y; v[2] = vv.z; v[3] = vv.w; }
        }
    } else {
        for (int j = 0; e + j < size; ++j) {
            a[j] = acc[at + j];
            if constexpr (UPDATE) { t[j] = theta[at + j]; if (vbuf) v[j] = vbuf[at + j]; }
        }
    }
    float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (NOISE) {
        const uint32_t step_word = step_dev ? (uint32_t)*step_dev : step_lo;
        const Philox4 r = philox4x32_10(q, 0u, fa.tensor_id[lo], step_word, k0, k1);
        box_muller(r.x, r.y, z[0], z[1]);
        box_muller(r.z, r.w, z[2], z[3]);
    }
    float g[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        g[j] = (a[j] + scale * z[j]) * inv_batch;
        if constexpr (UPDATE) {
            if (vbuf) { v[j] = momentum * v[j] + g[j]; t[j] -= lr * v[j]; }
            else t[j] -= lr * g[j];
        }
    }
    if (full) {
        if (out) {
            float4 *o = reinterpret_cast<float4 *>(out + at);
            __builtin_nontemporal_store(g[0], &o->x);
            __builtin_nontemporal_store(g[1], &o->y);
            __builtin_nontemporal_store(g[2], &o->z);
            __builtin_nontemporal_store(g[3], &o->w);
        }
        if constexpr (UPDATE) {
            *reinterpret_cast<float4 *>(theta + at) = make_float4(t[0], t[1], t[2], t[3]);
            if (vbuf) *reinterpret_cast<float4 *>(vbuf + at) = make_float4(v[0], v[1], v[2], v[3]);
        }
    } else {
        for (int j = 0; e + j < size; ++j) {
            if (out) out[at + j] = g[j];
            if constexpr (UPDATE) { theta[at + j] = t[j]; if (vbuf) vbuf[at + j] = v[j]; }
        }
    }
}

dp_status launch_noise_finalize_flat(const float *acc, float *out, float *theta, float *vbuf, const uint64_t *seg_begin,
                                     const uint64_t *seg_size, const uint32_t *seg_tensor_id, int n_seg, float sigma,
                                     float clip_total, uint64_t total_batch, uint64_t seed, uint64_t step,
                                     const uint64_t *step_dev, float lr, float momentum, hipStream_t s)
{
    const float inv_batch = 1.0f / (float)total_batch;
    const float scale = sigma > 0.0f ? sigma * clip_total : 0.0f;
    for (int s0 = 0; s0 < n_seg; s0 += FLAT_SEG_MAX) {
        FlatArgs fa;
        fa.n_seg = n_seg - s0 < FLAT_SEG_MAX ? n_seg - s0 : FLAT_SEG_MAX;
        unsigned int blocks = 0;
        for (int k = 0; k < FLAT_SEG_MAX; ++k) {
            const bool live = k < fa.n_seg;
            fa.begin[k] = live ? seg_begin[s0 + k] : 0;
            fa.size[k] = live ? (unsigned int)seg_size[s0 + k] : 0;
            fa.tensor_id[k] = live ? seg_tensor_id[s0 + k] : 0;
            fa.first_block[k] = blocks;
            if (live) blocks += (unsigned int)((seg_size[s0 + k] + FLAT_BLOCK - 1) / FLAT_BLOCK);
        }
        fa.first_block[FLAT_SEG_MAX] = blocks;
        const unsigned long long *sd = reinterpret_cast<const unsigned long long *>(step_dev);
        const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32), st = (uint32_t)step;
        const bool noise = sigma > 0.0f;
        if (theta) {
            if (noise) hipLaunchKernelGGL((noise_finalize_flat_kernel<true, true>), dim3(blocks), dim3(256), 0, s, acc, out, theta, vbuf, fa, scale, inv_batch, lr, momentum, k0, k1, st, sd);
            else hipLaunchKernelGGL((noise_finalize_flat_kernel<false, true>), dim3(blocks), dim3(256), 0, s, acc, out, theta, vbuf, fa, scale, inv_batch, lr, momentum, k0, k1, st, sd);
        } else {
            if (noise) hipLaunchKernelGGL((noise_finalize_flat_kernel<true, false>), dim3(blocks), dim3(256), 0, s, acc, out, theta, vbuf, fa, scale, inv_batch, lr, momentum, k0, k1, st, sd);
            else hipLaunchKernelGGL((noise_finalize_flat_kernel<false, false>), dim3(blocks), dim3(256), 0, s, acc, out, theta, vbuf, fa, scale, inv_batch, lr, momentum, k0, k1, st, sd);
        }
        const dp_status stt = check_launch("noise_finalize_flat");
        if (stt != DP_OK) return stt;
    }
    return DP_OK;
}

__global__ void __launch_bounds__(256) philox_raw_kernel(uint32_t *__restrict__ raw, size_t p, uint32_t k0,
                                                          uint32_t k1, uint32_t step_lo, uint32_t tensor_id)
{
    const uint64_t q = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    const size_t e = (size_t)q * 4;
    if (e >= p) return;
    const Philox4 r = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), tensor_id, step_lo, k0, k1);
    const uint32_t v[4] = {r.x, r.y, r.z, r.w};
    for (int j = 0; j < 4 && e + j < p; ++j) raw[e + j] = v[j];
}

dp_status launch_philox_raw(uint32_t *raw, size_t p, uint64_t seed, uint64_t step, uint32_t tensor_id, hipStream_t s)
{
    const size_t calls = (p + 3) / 4;
    hipLaunchKernelGGL(philox_raw_kernel, dim3((unsigned)((calls + 255) / 256)), dim3(256), 0, s, raw, p,
                       (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step, tensor_id);
    return check_launch("philox_raw");
}

}  // namespace dp
