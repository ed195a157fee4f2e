// Grouped launches: several layers that run the same kernel instantiation share ONE launch.
//
// A kernel takes a Grouped<Args> by value (kernel arguments, at most GROUP_MAX layers): the argument
// block of every layer and the number of the first workgroup of each.  A workgroup finds its layer
// with a short uniform scan and then behaves exactly as in a single-layer launch with the workgroup
// number `bid` counted from its layer's first workgroup.  A layer's workgroup count is a multiple of
// 8, so the XCD a workgroup lands on depends on `bid` alone.
//
// Why: a micro-step of a deep network is ~100 small launches, most of them far too small to fill
// 256 compute units, and inside one launch all workgroups start, stream and finish together.  With
// the layers of one kernel variant in one launch there are several rounds of workgroups, so loads,
// MFMAs and epilogues of different workgroups overlap, and a one-example micro-step is a handful of
// launches instead of a hundred.
//
// On the host, launchers hand their kernels to submit_kernel() with a tier: layout changes of the
// inputs (TIER_LAYOUT), operand pre-passes (TIER_PRE), the contraction itself (TIER_MAIN, also
// submit_main()), the sums over K slices (TIER_POST).  With no queue open a kernel is launched at once (a group of one); inside a batch call
// (LaunchQueue open on this thread) it is held back until flush(), which launches tier after tier,
// the held launches of a tier grouped by kernel, and then runs the deferred follow-up calls
// (partial-norm reductions) in the order they were registered.
#pragma once

#include <hip/hip_runtime.h>

#include <cstring>
#include <functional>
#include <vector>

#include "internal.h"

namespace dp {

constexpr int GROUP_MAX = 16;

template <typename Args>
struct Grouped {
    Args a[GROUP_MAX];
    unsigned first_block[GROUP_MAX + 1];
    int count;
};

#if defined(__HIPCC__)
// Layer of this workgroup; `bid` = workgroup number within the layer.  Uniform across the workgroup.
template <typename Args>
__device__ __forceinline__ int group_pick(const Grouped<Args> &g, unsigned &bid)
{
    int l = 0;
#pragma unroll
    for (int k = 1; k < GROUP_MAX; ++k)
        if (k < g.count && blockIdx.x >= g.first_block[k]) l = k;
    bid = blockIdx.x - g.first_block[l];
    return l;
}
#endif

enum { TIER_LAYOUT = 0, TIER_PRE = 1, TIER_MAIN = 2, TIER_POST = 3, TIER_COUNT = 4 };

struct LaunchQueue {
    struct Item {
        const void *fn;                 // kernel
        unsigned blocks, threads, lds;
        std::vector<char> args;         // one Args
        dp_status (*go)(const void *fn, const char *args, const unsigned *blocks, int count, unsigned threads,
                        unsigned lds, hipStream_t s);
        const char *what;
    };
    std::vector<Item> tier[TIER_COUNT];
    std::vector<std::function<dp_status()>> post;
    hipStream_t stream = nullptr;
    int crowd = 0;                      // > 0: launches are shared with other layers; the work a workgroup should
                                        // get, in units of one 128x128x64 chunk (about a million multiply-adds)
    int fuse = 0;                       // > 0: launchers hand in the kernels that dispatch on the variant INSIDE the kernel
                                        // (one launch for all row widths of the 3x3 kernel): only four kernels run at a
                                        // time, and a narrow launch inside a wide one costs none of them.  2: micro-steps
                                        // of one or two examples (a launch costs more than the work in it; finely sliced
                                        // variants), 1: larger ones (unsliced and clip-weighted variants)
};

// The queue open on this thread (nullptr: launches are issued at once).
LaunchQueue *open_queue();
void set_open_queue(LaunchQueue *q);
// 0, or inside a batch call of several layers the work per workgroup to plan for (see LaunchQueue::crowd)
int crowd_hint();
// which variant-dispatching kernels the open batch wants (see LaunchQueue::fuse); 0: none
int fuse_hint();
// Launch the held main kernels grouped by kernel, then the deferred follow-ups.
dp_status flush_queue(LaunchQueue &q);

template <typename Args>
dp_status launch_grouped(const void *fn, const char *args, const unsigned *blocks, int count, unsigned threads,
                         unsigned lds, hipStream_t s)
{
    static_assert(sizeof(Grouped<Args>) <= 4000, "kernel arguments are limited to 4 KB");
    Grouped<Args> g;
    std::memset(&g, 0, sizeof(g));
    unsigned total = 0;
    for (int k = 0; k < GROUP_MAX; ++k) {
        g.first_block[k] = total;
        if (k < count) {
            std::memcpy(&g.a[k], args + (size_t)k * sizeof(Args), sizeof(Args));
            total += blocks[k];
        }
    }
    g.first_block[GROUP_MAX] = total;
    g.count = count;
    void *kargs[] = {&g};
    const hipError_t e = hipLaunchKernel(fn, dim3(total), dim3(threads), kargs, lds, s);
    if (e != hipSuccess) return fail(DP_ERR_DEVICE, "grouped launch failed: %s", hipGetErrorString(e));
    return DP_OK;
}

// A kernel of a launcher: at once, or held back for the batch call's grouped launch of its tier.
// A TIER_MAIN kernel is bracketed by the benchmark timing aid when armed.
template <typename Args>
dp_status submit_kernel(int tier, const void *fn, const Args &a, unsigned blocks, unsigned threads, unsigned lds,
                        hipStream_t s, const char *what)
{
    LaunchQueue *q = open_queue();
    if (!q) {
        if (tier == TIER_MAIN) profile_begin(s);
        const dp_status st = launch_grouped<Args>(fn, reinterpret_cast<const char *>(&a), &blocks, 1, threads, lds, s);
        if (tier == TIER_MAIN) profile_end(s);
        return st != DP_OK ? st : check_launch(what);
    }
    LaunchQueue::Item it;
    it.fn = fn; it.blocks = blocks; it.threads = threads; it.lds = lds;
    it.args.assign(reinterpret_cast<const char *>(&a), reinterpret_cast<const char *>(&a) + sizeof(Args));
    it.go = &launch_grouped<Args>;
    it.what = what;
    q->tier[tier].push_back(std::move(it));
    return DP_OK;
}

// The contraction kernel of a launcher.  `blocks` must be a multiple of 8 (the XCD remap relies on it).
template <typename Args>
dp_status submit_main(const void *fn, const Args &a, unsigned blocks, unsigned threads, unsigned lds, hipStream_t s,
                      const char *what)
{
    return submit_kernel<Args>(TIER_MAIN, fn, a, blocks, threads, lds, s, what);
}

// A follow-up call that must come after every kernel of the layer: at once, or after the batch's grouped launches.
inline dp_status submit_post(std::function<dp_status()> fn)
{
    LaunchQueue *q = open_queue();
    if (!q) return fn();
    q->post.push_back(std::move(fn));
    return DP_OK;
}

}  // namespace dp
