// Host-side launch helpers: the one-time kernel attribute set-up, kept per kernel variant and per
// device in atomics (two host threads may make their first call together, and a process may
// drive several GPUs).
#ifndef ATOM_LAUNCH_H
#define ATOM_LAUNCH_H

#include <hip/hip_runtime.h>

#include <atomic>

namespace atom_launch {

constexpr int kMaxDevices = 64;

inline int current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) dev = 0;
    return dev;
}

// Largest dynamic LDS size a kernel variant has been allowed so far, per device (zero-initialised
// static storage: one instance per kernel variant).
struct LdsOptIn {
    std::atomic<unsigned> bytes[kMaxDevices];
};

// Raise the kernel's dynamic-LDS limit to `lds` bytes if it is not there yet.  Calling
// hipFuncSetAttribute twice for the same size is harmless; it is only kept off the launch path.
inline hipError_t ensure_dynamic_lds(LdsOptIn &state, const void *kernel, size_t lds)
{
    std::atomic<unsigned> &slot = state.bytes[current_device()];
    if (slot.load(std::memory_order_acquire) >= lds) return hipSuccess;
    hipError_t err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return err;
    unsigned seen = slot.load(std::memory_order_relaxed);
    while (seen < lds && !slot.compare_exchange_weak(seen, (unsigned)lds, std::memory_order_release)) {}
    return hipSuccess;
}

// Compute units of the current device (256 when the query fails).
inline int compute_units()
{
    static std::atomic<int> cus[kMaxDevices];
    const int dev = current_device();
    int n = cus[dev].load(std::memory_order_relaxed);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cus[dev].store(n, std::memory_order_relaxed);
    return n;
}

}  // namespace atom_launch
#endif
