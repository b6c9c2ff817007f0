// Host-side launchers of threshold.hip (threshold masks in CSR form): each validates nothing (the ABI layer did) and enqueues kernels.
#pragma once

#include "dsa_internal.h"

namespace dsa {

bool threshold_supported(const dsa_shape &sh);
size_t threshold_workspace_bytes(const dsa_shape &sh);
hipError_t launch_predict_threshold(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int theta,
                                    int32_t *row_ptr, int32_t *col, long long col_capacity, void *ws, hipStream_t st);

}  // namespace dsa
