// attn_launch.h -- host-side launch helpers shared by the entry points.
#pragma once
#include <stdint.h>

#include <hip/hip_runtime.h>

#include <mutex>
#include <unordered_map>

namespace attn {

// Opt in to more than 64 KB of dynamic LDS when a kernel needs it (gfx950 has 160 KB per CU).  The
// attribute belongs to the kernel on a device: it is set on the first launch of that kernel on that
// device and remembered, so later launches pay a lock and a lookup instead of a runtime call.
inline bool allow_lds(const void *kern, int bytes)
{
    if (bytes <= 64 * 1024)
        return true;
    constexpr int kMaxDev = 64;
    static std::mutex mu;
    static std::unordered_map<const void *, uint64_t> done;  // kernel -> devices that have the attribute
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev)
        return false;
    std::lock_guard<std::mutex> lock(mu);
    uint64_t &mask = done[kern];
    if (mask >> dev & 1)
        return true;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    mask |= 1ull << dev;
    return true;
}

// Compute units of the current device (asked once per device), rounded down to a multiple of `multiple`;
// 0 when the runtime cannot tell.
inline int cu_count(int multiple)
{
    constexpr int kMaxDev = 64;
    static std::mutex mu;
    static int cached[kMaxDev] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev)
        return 0;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            return 0;
        }
        cached[dev] = n;
    }
    return cached[dev] / multiple * multiple;
}

// Slots of a persistent launch of `kern` (threads per workgroup, dynamic LDS bytes as launched): compute units
// of the current device, rounded down to a multiple of `multiple`, times the workgroups of this kernel that a CU
// holds at once (asked from the runtime once per kernel and device).  0 when the runtime cannot tell.
inline int persistent_slots(const void *kern, int threads, int lds_bytes, int multiple)
{
    constexpr int kMaxDev = 64;
    static std::mutex mu;
    static std::unordered_map<const void *, std::unordered_map<int, int>> cached;  // kernel -> device -> per CU
    const int cus = cu_count(multiple);
    int dev = 0;
    if (cus < 1 || hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev)
        return 0;
    std::lock_guard<std::mutex> lock(mu);
    int &per_cu = cached[kern][dev];
    if (per_cu == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, (size_t)lds_bytes) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            return 0;
        }
        per_cu = n;
    }
    return cus * per_cu;
}

}  // namespace attn
