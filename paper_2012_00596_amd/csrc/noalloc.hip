// npas_run_stack_static: npas_run_stack for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  The intermediate tensors of the stack, which
// npas_run_stack places in a caller-provided workspace, live in a file-scope device array instead.
#include <hip/hip_runtime.h>

#include <mutex>

#include "npas_internal.h"

namespace {

// One copy of this array exists on every GPU the library is loaded on, for the life of the process.
static __device__ __align__(256) unsigned char scratch[NPAS_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices] = {}; // device address of `scratch` per device (the array's name is no device address on the host)

// The device address of this GPU's copy of the array; looked up once per device, with that device current.
int scratch_address(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        npas::set_error("no current HIP device (%s)", e == hipSuccess ? "device index out of range" : hipGetErrorString(e));
        return NPAS_E_HIP;
    }
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            npas::set_error("hipGetSymbolAddress(static workspace) failed: %s", hipGetErrorString(e));
            return NPAS_E_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return NPAS_OK;
}

} // namespace

extern "C" int npas_run_stack_static(const npas_stack *s, const void *x_dev, void *y_dev, int N, void *hip_stream)
{
    if (!s || !x_dev || !y_dev) {
        npas::set_error("NULL argument");
        return NPAS_E_NULL;
    }
    if (N <= 0) {
        npas::set_error("bad batch %d", N);
        return NPAS_E_SHAPE;
    }
    const size_t need = npas_stack_workspace_bytes(s, N);
    if (need > (size_t)NPAS_STATIC_WORKSPACE_BYTES) {
        npas::set_error("the stack needs %zu bytes of workspace at batch %d, the static workspace holds %zu: use a smaller "
                        "batch, or npas_run_stack with a workspace of the caller's",
                        need, N, (size_t)NPAS_STATIC_WORKSPACE_BYTES);
        return NPAS_E_WORKSPACE;
    }
    void *ws = nullptr;
    if (int rc = scratch_address(&ws)) return rc;
    // Every intermediate tensor is written in full by the launch that produces it before any launch reads it, so
    // nothing in the array has to start at zero; what the previous call left there is simply overwritten.
    return npas::run_stack_impl(s, x_dev, y_dev, N, ws, (size_t)NPAS_STATIC_WORKSPACE_BYTES, hip_stream);
}
