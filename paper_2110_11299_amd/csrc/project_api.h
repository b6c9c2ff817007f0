// Host-side launchers of project.hip (projection + quantiser, code unpacking): each validates nothing (the ABI layer did) and enqueues kernels.
#pragma once

#include "dsa_internal.h"

namespace dsa {

// R: float [d,k] projection, or (R == nullptr) P3: int8 [d,k] with entries in {-1, 0, 1}.
hipError_t launch_project_quantize(const dsa_shape &sh, int bits, const void *X, const float *R, const int8_t *P3,
                                   void *Xt, float *amax_out, void *ws, hipStream_t st);
hipError_t launch_unpack_codes(int bits, const void *packed, int8_t *codes, size_t n_codes, hipStream_t st);
size_t project_workspace_bytes(const dsa_shape &sh);

}  // namespace dsa
