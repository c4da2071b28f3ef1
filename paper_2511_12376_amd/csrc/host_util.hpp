// Host-side helpers shared by the entry points: cached device facts, pointer checks, launch status.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/bitsnap.h"

namespace bitsnap {

struct DeviceInfo {
    int cu_count = 0;
};

constexpr int kMaxDevices = 64;

inline const DeviceInfo &device_info()
{
    static DeviceInfo info[kMaxDevices];
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        dev = 0;
    std::lock_guard<std::mutex> lock(mu);
    if (info[dev].cu_count == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        info[dev].cu_count = cus;
    }
    return info[dev];
}

// Resident workgroups per CU for `kernel` at `block` threads (no dynamic LDS); cached per kernel.
inline int occupancy_blocks_per_cu(const void *kernel, int block)
{
    struct Entry {
        const void *k;
        int v;
    };
    static Entry cache[64];
    static int used = 0;
    static std::mutex mu;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i)
        if (cache[i].k == kernel)
            return cache[i].v;
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, block, 0) != hipSuccess || per_cu < 1)
        per_cu = 1;
    if (used < 64)
        cache[used++] = Entry{kernel, per_cu};
    return per_cu;
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

inline int launch_status() { return hipGetLastError() == hipSuccess ? BITSNAP_OK : BITSNAP_E_LAUNCH; }

}  // namespace bitsnap
