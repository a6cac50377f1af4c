// Host-side process state of the library: the once-per-(kernel, device) raising of the dynamic-LDS limit and
// the explicit set-up call behind meteora_init.
#include <mutex>

#include "common.hpp"
#include "kernels.hpp"

namespace meteora {

namespace {
constexpr int kMaxDevices = 64;
constexpr int kMaxKernels = 64;
struct LdsEntry { const void* kernel; uint64_t done; };   // bit d: the limit is set on device d
LdsEntry g_lds[kMaxKernels];
int g_lds_count = 0;
std::mutex g_lds_mutex;
}  // namespace

// Kernels with more than 64 KB of dynamic LDS need the limit raised by a host-side attribute, which HIP keeps
// per device.  The first launch of a kernel on a device does it (or init_kernels below, ahead of time); the
// table is guarded by a mutex so that threads launching on different streams do not race on it.
hipError_t ensure_lds_limit(const void* kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_lds_mutex);
    LdsEntry* ent = nullptr;
    for (int i = 0; i < g_lds_count; ++i)
        if (g_lds[i].kernel == kernel) ent = &g_lds[i];
    if (ent == nullptr) {
        if (g_lds_count >= kMaxKernels) return hipErrorOutOfMemory;
        ent = &g_lds[g_lds_count++];
        *ent = LdsEntry{kernel, 0};
    }
    if (ent->done >> dev & 1) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) ent->done |= 1ull << dev;
    return e;
}

// Everything a first launch would set up lazily, for the current device.
hipError_t init_kernels() {
    hipError_t e = gemm_init_kernels();
    if (e != hipSuccess) return e;
    e = gate_init_kernels();
    if (e != hipSuccess) return e;
    e = shrink_init_kernels();
    if (e != hipSuccess) return e;
    return bucket_init_scratch();
}

}  // namespace meteora
