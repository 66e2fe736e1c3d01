// sl_compress_noalloc: sl_compress for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The scratch that
// sl_compress takes from its `workspace` argument (selected values, partial sums of the
// quantizer statistics, per-tensor mean / variance) lives here in one file-scope device array
// of a fixed size; the kernels are the ones sl_compress launches and receive the array's
// device address as they receive a caller's workspace.
//
// In host code the array's name is only a stand-in for the symbol: its device address - one
// per GPU, since every GPU holds its own copy of the array - is looked up once per device with
// hipGetSymbolAddress while that device is current, kept in a table, and only that looked-up
// pointer is ever handed to a kernel or a runtime call.
#include <mutex>

#include "sl_internal.h"

namespace {

constexpr int MAX_DEVICES = 64;

// The scratch of every call made through this entry point on one GPU.  Nothing in it has to be
// zero when a call starts: every section is written by the kernel that precedes its reader.
static __device__ __align__(256) unsigned char scratch[SL_NOALLOC_SCRATCH_BYTES];

std::mutex g_lock;
void *g_scratch_ptr[MAX_DEVICES];        // device address of `scratch` on each device, once resolved

}  // namespace

// Device address of this file's scratch array on `device`, which must be the current device.
// Resolved on first use (sl_plan_create calls it, so a plan's device is normally resolved
// before any compress call and before any stream capture begins).
int sl_noalloc_scratch(int device, void **out)
{
    if (device < 0 || device >= MAX_DEVICES) return SL_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[device]) {
        void *ptr = nullptr;
        const hipError_t err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess || !ptr) {
            sl_note_hip_error(err);
            return SL_ERR_HIP;
        }
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return SL_OK;
}

extern "C" int sl_compress_noalloc(sl_plan *p, float *e, const float *delta, float beta, int flags,
                                   const void *pending, void *payload, void *stream)
{
    if (!p) return SL_ERR_INVALID_ARG;
    if (p->ws_bytes > (size_t)SL_NOALLOC_SCRATCH_BYTES) return SL_ERR_TOO_LARGE;
    int dev = -1;
    const hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) {
        sl_note_hip_error(err);
        return SL_ERR_HIP;
    }
    if (dev != p->device) return SL_ERR_DEVICE;
    void *ws = nullptr;
    const int rc = sl_noalloc_scratch(dev, &ws);
    if (rc) return rc;
    return sl_compress_impl(p, e, delta, nullptr, beta, flags, pending, payload, ws, stream);
}
