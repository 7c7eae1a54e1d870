// rl_plan_run_static: rl_plan_run for callers that cannot provide (or allocate) a workspace -- code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc.  The plan's intermediates (and the partial sums of
// contractions whose K is split over workgroups) then live in one array that is part of the library's code object:
// every GPU the library runs on holds its own copy until the process ends.
#include <mutex>

#include "handles.h"

namespace {

// Workspace of the allocation-free entry point.  In host code this name is only a handle for
// hipGetSymbolAddress; the address kernels may use is the one that call returns, per device.
static __device__ __align__(256) unsigned char scratch[RL_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices];        // device address of `scratch` on device i, once looked up

// Address of the current device's copy of the array (looked up once per device, with that device current).
hipError_t scratch_address(void **out)
{
    int dev = -1;
    hipError_t er = hipGetDevice(&dev);
    if (er != hipSuccess) return er;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        er = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (er != hipSuccess) return er;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" rl_status rl_plan_run_static(const rl_plan *plan, const rl_binding *bindings, int32_t n_bindings, void *hip_stream)
{
    if (!plan) return RL_ERR_NULL;
    const std::shared_ptr<rl::ErrBox> &err = plan->p.err;
    if (plan->p.workspace_bytes > (size_t)RL_STATIC_WORKSPACE_BYTES) {
        if (err) err->set("plan needs a workspace of " + std::to_string(plan->p.workspace_bytes) + " bytes, the built-in one holds " +
                          std::to_string((size_t)RL_STATIC_WORKSPACE_BYTES) + ": use rl_plan_run with a workspace of the caller's");
        return RL_ERR_WORKSPACE;
    }
    void *ws = nullptr;
    if (plan->p.workspace_bytes > 0) {
        const hipError_t er = scratch_address(&ws);
        if (er != hipSuccess) {
            if (err) err->set(std::string("address of the built-in workspace: ") + hipGetErrorString(er));
            return RL_ERR_HIP;
        }
    }
    // every byte of the workspace a step reads was written by an earlier step of the same run: nothing to clear
    return rl_plan_run(plan, bindings, n_bindings, ws, ws ? (size_t)RL_STATIC_WORKSPACE_BYTES : 0, hip_stream);
}
