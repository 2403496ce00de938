// xl_run_static: the entry point for callers that cannot allocate device memory (see include/xl.h).
// The workspace that xl_prepare / xl_run take from the caller lives here in a file-scope device array.
#include <mutex>
#include <string>

#include "plan.h"

// One copy per GPU the library is loaded on, held until the process ends.
static __device__ __align__(256) unsigned char scratch[XL_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
void *g_scratch_ptr[MAX_DEVICES] = {};                 // device address of `scratch` on each GPU
unsigned long long g_scratch_owner[MAX_DEVICES] = {};  // serial of the plan whose filters the array holds

// Device address of this GPU's copy of the array.  `scratch` itself is only a host-side handle:
// the address has to be asked for, once per device, with that device current.
xl_status scratch_address(int dev, void **out, std::string &err)
{
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            err = std::string("cannot resolve the static scratch array: ") + hipGetErrorString(e);
            return XL_E_DEVICE;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return XL_OK;
}

}  // namespace

extern "C" xl_status xl_run_static(xl_plan *plan, const void *const *weights, int nweights, const void *const *tensors,
                                   int ntensors, void *stream, int fused, int relayout)
{
    if (!plan || !tensors) return XL_E_NULL;
    if (plan->workspace_bytes > (size_t)XL_STATIC_SCRATCH_BYTES) {
        plan->error = "the plan needs " + std::to_string(plan->workspace_bytes) + " bytes of workspace, the static scratch holds " +
                      std::to_string((size_t)XL_STATIC_SCRATCH_BYTES);
        return XL_E_SCRATCH;
    }
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        plan->error = "no current HIP device";
        return XL_E_DEVICE;
    }
    void *ws = nullptr;
    xl_status st = scratch_address(dev, &ws, plan->error);
    if (st != XL_OK) return st;
    bool holds_this_plan;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        holds_this_plan = g_scratch_owner[dev] == plan->serial;
    }
    if (relayout || !holds_this_plan) {
        if (!weights) {
            plan->error = "the static scratch does not hold this plan's filters and no weights were passed";
            return relayout ? XL_E_NULL : XL_E_STATE;
        }
        // everything the kernels read from the array is written here or by an earlier kernel of the
        // same run: nothing has to start at zero, whatever the previous call left behind
        st = xl_prepare(plan, weights, nweights, ws, stream);
        if (st != XL_OK) return st;
        std::lock_guard<std::mutex> lock(g_mu);
        g_scratch_owner[dev] = plan->serial;
    }
    return xl_run(plan, tensors, ntensors, ws, stream, fused);
}
