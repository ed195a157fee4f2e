// dp_per_example_grad_static: dp_per_example_grad for callers that cannot hand over (or allocate) a
// workspace -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
// The workspace is a file-scope device array of a fixed, modest size; every GPU the library runs on
// holds its own copy until the process ends.  In host code the array's name is only a stand-in: its
// device address is asked for once per device (hipGetSymbolAddress, with that device current) and
// that pointer, never the name, is what the kernels get.
#include "internal.h"

#include <mutex>

namespace {

constexpr size_t SCRATCH_BYTES = (size_t)32 << 20;
__device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES];       // device address of `scratch` on each device, once resolved
std::mutex g_scratch_mutex;

// Address of this device's copy of the array (resolved on the first call on that device).
dp_status scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return dp::fail(DP_ERR_DEVICE, "hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) return dp::fail(DP_ERR_UNSUPPORTED, "device %d beyond the %d this build tracks", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return dp::fail(DP_ERR_DEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DP_OK;
}

}  // namespace

extern "C" {

size_t dp_static_scratch_bytes(void) { return SCRATCH_BYTES; }

dp_status dp_per_example_grad_static(const dp_layer_desc *desc, const void *x, const void *dy, float *g_w, float *g_b,
                                     size_t g_stride, float *sqnorm, dp_stream stream)
{
    const size_t need = dp_workspace_bytes(desc, DP_WS_PER_EXAMPLE_GRAD);     // 0 on a bad descriptor: reported below
    if (need > SCRATCH_BYTES)
        return dp::fail(DP_ERR_WORKSPACE, "this layer needs %zu bytes of workspace, the built-in scratch holds %zu; "
                        "use dp_per_example_grad with a caller-owned workspace", need, SCRATCH_BYTES);
    void *ws = nullptr;
    const dp_status st = scratch_of_current_device(&ws);
    if (st != DP_OK) return st;
    return dp_per_example_grad(desc, x, dy, g_w, g_b, g_stride, sqnorm, ws, SCRATCH_BYTES, stream);
}

}  // extern "C"
