// Execution of a compiled plan without a caller-supplied workspace: the
// intermediate tensors and the split-K partial sums of the plan's kernels live
// in a fixed device array that is part of the library's code object.  For
// callers that cannot allocate device memory: code under HIP graph capture,
// serving loops, harnesses that forbid it.
//
// Each GPU the library is loaded on holds its own copy of the array until the
// process ends.  In host code the array's name is only a stand-in for the
// symbol; the device address is looked up once per device and that address is
// what the kernels receive.
#include <hip/hip_runtime.h>

#include "core.h"

namespace clg {

namespace {

constexpr size_t kStaticBytes = CLG_STATIC_WORKSPACE_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

void *g_scratch_ptr[kMaxDevices];        // device address of `scratch` on each device, null until looked up

}  // namespace

// Looks up this device's address of the array (once).  Called from clg_create
// for a device context; leaves the current device as it found it.
int32_t static_workspace_init(int32_t device) {
    if (device < 0 || device >= kMaxDevices)
        return fail(CLG_INVALID_ARG, "device %d: the static workspace serves devices 0..%d", device, kMaxDevices - 1);
    if (g_scratch_ptr[device]) return CLG_OK;
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e == hipSuccess && cur != device) e = hipSetDevice(device);
    void *p = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (cur >= 0 && cur != device) (void)hipSetDevice(cur);
    if (e != hipSuccess || !p)
        return fail(CLG_HIP_ERROR, "address of the static workspace on device %d: %s", device, hipGetErrorString(e));
    g_scratch_ptr[device] = p;
    return CLG_OK;
}

int32_t execute_plan_static(Plan &p, const void *const *inputs, void *const *outputs, void *stream) {
    const int32_t device = p.ctx->device;
    if (device < 0) return fail(CLG_HIP_ERROR, "host-only context: no device to execute on");
    if (p.workspace_bytes > kStaticBytes)
        return fail(CLG_WORKSPACE_TOO_SMALL, "the plan needs a workspace of %zu bytes, the static one holds %zu: use clg_execute",
                    p.workspace_bytes, kStaticBytes);
    if (device >= kMaxDevices || !g_scratch_ptr[device])
        return fail(CLG_HIP_ERROR, "the static workspace of device %d was not set up", device);
    if (p.n_lanes > 1 && p.side_streams.empty())
        return fail(CLG_INVALID_ARG, "the plan's lanes are created at its first clg_execute: run that once, or use one lane");
    return execute_plan(p, inputs, outputs, g_scratch_ptr[device], kStaticBytes, stream, nullptr);
}

}  // namespace clg
