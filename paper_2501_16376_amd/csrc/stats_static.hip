// swiftprune_layer_stats for callers that cannot allocate device memory: the
// partial sums of the statistics kernels live in a device array owned by the
// library instead of a caller-provided workspace.  Same kernels, same results.
#include "../../include/swiftprune.h"

#include "kernels.hpp"

#include <mutex>

namespace {

constexpr size_t kScratchBytes = SP_STATIC_WORKSPACE_BYTES;
constexpr int kMaxDevices = 64;

// One copy of this array exists on every GPU the library's code object is loaded on, each at its own
// address.  Host code never uses this name as a pointer: it asks the runtime for the device address.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on device i, null until first use

// Device address of the array on the current device (looked up once per device).
hipError_t scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(g_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

inline int64_t elem_size(int dt) { return dt == SP_F32 ? 4 : 2; }

}  // namespace

extern "C" int swiftprune_layer_stats_static(const void* X, int64_t tokens, int64_t in, int64_t ldx,
                                             sp_dtype dt, float* xsq, float* S, float* hr, int accumulate,
                                             int finalize, void* hip_stream) {
    if (X == nullptr || xsq == nullptr || S == nullptr || (finalize && hr == nullptr)) return SP_EINVAL;
    if (tokens <= 0 || in <= 0 || ldx < in) return SP_EINVAL;
    if (dt != SP_F32 && dt != SP_BF16 && dt != SP_F16) return SP_EINVAL;
    if (reinterpret_cast<uintptr_t>(X) % elem_size((int)dt) != 0) return SP_EINVAL;
    if (swiftprune_stats_workspace_bytes(tokens, in) > kScratchBytes) return SP_ENOSPC;
    void* ws = nullptr;
    if (scratch_address(&ws) != hipSuccess) return SP_EHIP;
    const int64_t epu = 16 / elem_size((int)dt);
    const bool vec = (reinterpret_cast<uintptr_t>(X) & 15u) == 0 && in % epu == 0 && ldx % epu == 0;
    // the statistics kernels overwrite every partial sum they later read, so nothing has to be cleared
    const hipError_t e = sp::launch_layer_stats(X, tokens, in, ldx, (int)dt, vec, xsq, S, hr, accumulate, finalize,
                                                ws, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SP_OK : SP_EHIP;
}
