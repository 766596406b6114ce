// dft3d_exec for callers that cannot allocate device memory: the ping-pong intermediate of the
// transform lives in a file-scope device array of the library instead of a caller-provided workspace.
#include <mutex>

#include "dft3d_internal.h"

namespace {

// One copy of this array exists on every GPU the library's code object is loaded on, at an address of
// its own, from the first use of the library on that GPU until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress; kernels get the resolved device pointer.
static __device__ __align__(256) unsigned char scratch[DFT3D_NOALLOC_MAX_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

}  // namespace

namespace dft3d {

// Resolves the address of the scratch array on the current device (once per device).  Returns
// nullptr and sets the error text on failure.
void* noalloc_scratch_for_current_device()
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        set_error("exec_noalloc: no current device (%s)", e == hipSuccess ? "index out of range" : hipGetErrorString(e));
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            set_error("exec_noalloc: hipGetSymbolAddress of the scratch array failed on device %d: %s", dev,
                      hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace dft3d

extern "C" dft3d_status dft3d_exec_noalloc(dft3d_plan plan, const void* in, void* out, int direction, void* stream)
{
    if (!plan) {
        dft3d::set_error("exec_noalloc: plan is NULL");
        return DFT3D_ERR_INVALID_ARG;
    }
    const size_t need = dft3d_plan_workspace_bytes(plan);
    if (need > (size_t)DFT3D_NOALLOC_MAX_BYTES) {
        dft3d::set_error("exec_noalloc: this plan needs %zu bytes of intermediate storage, the static scratch array "
                         "holds %zu; use dft3d_exec with a workspace", need, (size_t)DFT3D_NOALLOC_MAX_BYTES);
        return DFT3D_ERR_UNSUPPORTED;
    }
    // resolved at plan creation on the plan's device; this only looks the pointer up (or resolves it
    // when the plan was created with another device current)
    void* ws = dft3d::noalloc_scratch_for_current_device();
    if (!ws) return DFT3D_ERR_HIP;
    return dft3d::exec_with_workspace(plan, in, out, direction, stream, ws, (size_t)DFT3D_NOALLOC_MAX_BYTES,
                                      "exec_noalloc");
}
