// Internal helpers shared by the translation units of libdsa_hip.so.  The host-side launchers of
// each unit are declared in its own *_api.h, so that a change to one unit rebuilds that unit and
// the ABI layer only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "dsa.h"

namespace dsa {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kXcds = 8;           // accelerator complex dies of an MI355X, each with its own L2

// Workgroups are handed to the XCDs round-robin by launch index.  This maps launch index b of
// `total` to a virtual index such that each XCD receives one contiguous range of virtual
// indices: neighbouring work (same head, same K / V rows) then shares one L2.  Bijective.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned b, unsigned total)
{
    const unsigned q = total / kXcds, r = total % kXcds;
    const unsigned x = b % kXcds, s = b / kXcds;
    return x * q + (x < r ? x : r) + s;
}

// A kernel that wants more than the default 48 KB of dynamic LDS needs its limit raised first.  That
// is done once per (kernel, device) and raises the limit to everything the device offers, so later
// launches of the same kernel with any plan cost no runtime call.  (If the small table is full the
// attribute is simply set again on every launch.)
inline hipError_t allow_dynamic_lds(const void *kern, size_t bytes)
{
    if (bytes <= 48 * 1024) return hipSuccess;
    struct Entry { const void *kern; int dev; };
    static Entry done[128];
    static int used = 0;
    static std::mutex mu;
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev)) return e;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < used; ++i)
        if (done[i].kern == kern && done[i].dev == dev) return hipSuccess;
    int limit = 0;
    if (hipError_t e = hipDeviceGetAttribute(&limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev)) return e;
    if ((size_t)limit < bytes) return hipErrorInvalidValue;
    if (hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, limit)) return e;
    if (used < 128) done[used++] = Entry{kern, dev};
    return hipSuccess;
}

}  // namespace dsa
