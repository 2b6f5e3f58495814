// floe_moe_layer_decode_static: the layer decode for callers that cannot allocate (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc).  It is floe_moe_layer_decode run on a scratch array that
// lives in the library's own device image instead of a caller-supplied workspace.
//
// One array per GPU, held from the moment the library is loaded on that GPU until the process ends.  In host code
// the array's name is only a handle: its device address is asked for once per device (with that device current) and
// every use goes through that pointer.  No kernel of the layer relies on the previous contents of its workspace
// (task table, counts, masks, v, lists and partial sums are all written before they are read), so nothing has to be
// cleared between calls; calls that overlap on one GPU share the array and race.
#include "../../include/floe.h"

#include <hip/hip_runtime.h>

#include <mutex>

namespace {

__device__ __align__(256) unsigned char g_static_scratch[FLOE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void* g_ptr[kMaxDevices];  // per device: each GPU holds its own copy of the array at its own address

// FLOE_OK and the current device's address of the array, or an error code
int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return FLOE_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return FLOE_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) return FLOE_EHIP;
        if (reinterpret_cast<uintptr_t>(p) % 256 != 0) return FLOE_EHIP;
        g_ptr[dev] = p;
    }
    *out = g_ptr[dev];
    return FLOE_OK;
}

}  // namespace

extern "C" int floe_moe_layer_decode_static(const floe_layer* L, const floe_half* x, int T, floe_half* y,
                                            floe_slot_stat* stats, void* stream) {
    if (!L || T < 0) return FLOE_EINVAL;
    if (T == 0) return FLOE_OK;
    const size_t need = floe_layer_workspace_bytes(L, T);  // 0: the layer description itself is invalid
    if (need > FLOE_STATIC_SCRATCH_BYTES) return FLOE_EWORKSPACE;  // decided before anything is touched or enqueued
    void* scratch = nullptr;
    const int rc = static_scratch(&scratch);
    if (rc != FLOE_OK) return rc;
    // (an invalid layer comes back from here with its proper error code)
    return floe_moe_layer_decode(L, x, T, y, stats, scratch, FLOE_STATIC_SCRATCH_BYTES, stream);
}
