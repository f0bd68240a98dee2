// Host-side launch helpers shared by the kernel sources of the potq library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace potq {

constexpr size_t kLdsDefaultLimit = 64 * 1024;    // dynamic LDS a kernel may ask for without further ado
constexpr size_t kLdsPerWorkgroup = 160 * 1024;   // what a gfx950 workgroup can be given

// A kernel that wants more dynamic LDS than the default limit has that limit raised, once per
// device and process.  `raised` is the caller's flag word for this kernel (bit d: done on device d;
// devices past 63 repeat the call).  The call is not stream work, so it is legal while a stream is
// being captured into a graph.
inline hipError_t allow_large_lds(const void *kernel, size_t lds_bytes, std::atomic<uint64_t> &raised)
{
    if (lds_bytes <= kLdsDefaultLimit) return hipSuccess;
    if (lds_bytes > kLdsPerWorkgroup) return hipErrorInvalidValue;
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 64 && ((raised.load(std::memory_order_acquire) >> device) & 1u)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerWorkgroup);
    if (e == hipSuccess && device < 64) raised.fetch_or(uint64_t{1} << device, std::memory_order_release);
    return e;
}

// The same for a kernel given as a template argument: one flag word per kernel.
template <auto Kernel>
inline hipError_t allow_large_lds(size_t lds_bytes)
{
    static std::atomic<uint64_t> raised{0};
    return allow_large_lds((const void *)Kernel, lds_bytes, raised);
}

}  // namespace potq
