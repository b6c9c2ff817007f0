// Internal declarations shared by the translation units of libdsa_hip.so.
// Host-side launchers: each validates nothing (the ABI layer did) and enqueues kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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

hipError_t launch_predict(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx,
                          void *ws, hipStream_t st);
size_t predict_workspace_bytes(const dsa_shape &sh);

enum AttnMode { kFused = 0, kSddmm = 1, kSpmm = 2 };
hipError_t launch_attention(AttnMode mode, const dsa_shape &sh, const void *Q, const void *K,
                            const void *V, const int32_t *idx, const float *Pin, float *S, float *O,
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
// Largest L the predict kernel accepts.
int predict_max_L();

}  // namespace dsa
