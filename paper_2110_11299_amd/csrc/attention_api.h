// Host-side launchers of attention.hip (SDDMM, softmax, SpMM: ELL and CSR masks, gather probe): each validates nothing (the ABI layer did) and enqueues kernels.
#pragma once

#include "dsa_internal.h"

namespace dsa {

enum AttnMode { kFused = 0, kSddmm = 1, kSpmm = 2 };
hipError_t launch_attention(AttnMode mode, const dsa_shape &sh, const void *Q, const void *K,
                            const void *V, const int32_t *idx, const float *Pin, float *S, float *O,
                            hipStream_t st);
hipError_t launch_attention_csr(const dsa_shape &sh, const void *Q, const void *K, const void *V,
                                const int32_t *row_ptr, const int32_t *col, float *O, hipStream_t st);
hipError_t launch_gather_probe(const dsa_shape &sh, const void *K, const void *V, const int32_t *idx, unsigned *sink,
                               hipStream_t st);
hipError_t launch_softmax(const dsa_shape &sh, const float *S, float *P, hipStream_t st);
// Largest `keep` the attention kernels accept (scores of one row are staged in LDS).
int attention_max_keep();
// Largest L the attention kernels accept.
int attention_max_L();

}  // namespace dsa
