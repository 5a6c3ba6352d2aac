// td_decode_step_static: the decode step for callers that cannot allocate (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  Its workspace - split partials,
// ticket counters, group scores, top-k state - is a device array with static storage: it exists on
// a GPU from the moment this code object is loaded there until the process ends, so the call
// neither allocates nor frees.
//
// In host code the array's name is a host-side stand-in, not a device address.  The address on the
// current device comes from hipGetSymbolAddress, once per device with that device current (each
// GPU holds its own copy at its own address), and only that pointer is handed to kernels.
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "common.h"

namespace {

constexpr size_t kStaticScratchBytes = TD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mutex;
char *g_scratch_ptr[kMaxDevices];  // per device; nullptr until resolved
thread_local char g_error[256] = "context is NULL";

hipError_t scratch_of_current_device(char **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<char *>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

namespace tidal {

// Set-up for the current device; td_create calls it so that the first td_decode_step_static on a
// device that already has a context finds the pointer resolved.
hipError_t static_scratch_setup() {
    char *unused = nullptr;
    return scratch_of_current_device(&unused);
}

const char *static_last_error() { return g_error; }

}  // namespace tidal

extern "C" td_status td_decode_step_static(const td_shape *shape, int32_t num_layers, const int32_t *schedule,
                                           const void *const *q_layers, const void *const *K_layers,
                                           const void *const *V_layers, int32_t k, void *const *out_layers,
                                           int32_t *positions, void *hip_stream) {
    // sizes beyond the array are refused here, before anything is enqueued (0: the shape itself is
    // unusable, which the layer loop below reports with its reason)
    const size_t need = td_workspace_bytes(shape, k);
    if (need > kStaticScratchBytes) {
        snprintf(g_error, sizeof g_error,
                 "td_workspace_bytes(shape, k) = %zu is above TD_STATIC_SCRATCH_BYTES = %zu: use td_create and "
                 "td_decode_step", need, kStaticScratchBytes);
        return TD_ERR_WORKSPACE;
    }
    char *ptr = nullptr;
    const hipError_t e = scratch_of_current_device(&ptr);
    if (e != hipSuccess) {
        snprintf(g_error, sizeof g_error, "static scratch of the current device is unavailable: %s", hipGetErrorString(e));
        return TD_ERR_HIP;
    }
    char error[256];
    const td_status st = tidal::decode_step_on_workspace(ptr, kStaticScratchBytes, shape, num_layers, schedule, q_layers,
                                                         K_layers, V_layers, k, out_layers, positions, hip_stream, error);
    if (st != TD_OK) memcpy(g_error, error, sizeof g_error);
    return st;
}
