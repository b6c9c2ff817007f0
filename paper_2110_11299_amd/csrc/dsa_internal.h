// Internal declarations shared by the translation units of libdsa_hip.so.
// Host-side launchers: each validates nothing (the ABI layer did) and enqueues kernels.
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

hipError_t launch_predict(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx,
                          void *ws, hipStream_t st);
size_t predict_workspace_bytes(const dsa_shape &sh);
// The streaming form of the fine-grained predictor and the shapes it serves (launch_predict picks it).
bool stream_predict_fits(const dsa_shape &sh);
hipError_t launch_predict_stream(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx,
                                 hipStream_t st);

enum AttnMode { kFused = 0, kSddmm = 1, kSpmm = 2 };
hipError_t launch_attention(AttnMode mode, const dsa_shape &sh, const void *Q, const void *K,
                            const void *V, const int32_t *idx, const float *Pin, float *S, float *O,
                            hipStream_t st);
hipError_t launch_attention_csr(const dsa_shape &sh, const void *Q, const void *K, const void *V,
                                const int32_t *row_ptr, const int32_t *col, float *O, hipStream_t st);
// Threshold masks in CSR form: which shapes, how much scratch, the launch.
bool threshold_supported(const dsa_shape &sh);
size_t threshold_workspace_bytes(const dsa_shape &sh);
hipError_t launch_predict_threshold(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int theta,
                                    int32_t *row_ptr, int32_t *col, long long col_capacity, void *ws, hipStream_t st);
hipError_t launch_gather_probe(const dsa_shape &sh, const void *K, const void *V, const int32_t *idx, unsigned *sink,
                               hipStream_t st);
hipError_t launch_softmax(const dsa_shape &sh, const float *S, float *P, hipStream_t st);
hipError_t launch_rowmax(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *rowmax,
                         hipStream_t st);

hipError_t launch_project_quantize(const dsa_shape &sh, int bits, const void *X, const float *R, void *Xt,
                                   float *amax_out, void *ws, hipStream_t st);
hipError_t launch_unpack_codes(int bits, const void *packed, int8_t *codes, size_t n_codes, hipStream_t st);
size_t project_workspace_bytes(const dsa_shape &sh);

hipError_t launch_mfma_i8_stream(int blocks, int iters, int32_t *sink, hipStream_t st);

// Largest `keep` the attention kernels accept (scores of one row are staged in LDS).
int attention_max_keep();
// Largest L the attention kernels accept.
int attention_max_L();
// Largest L the predict kernel accepts.
int predict_max_L();

}  // namespace dsa
