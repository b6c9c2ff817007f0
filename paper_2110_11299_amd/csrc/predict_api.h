// Host-side launchers of predict.hip (tiled predictor, row-max contraction, MFMA yardstick): each validates nothing (the ABI layer did) and enqueues kernels.
#pragma once

#include "dsa_internal.h"

namespace dsa {

hipError_t launch_predict(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx,
                          void *ws, hipStream_t st);
size_t predict_workspace_bytes(const dsa_shape &sh);
hipError_t launch_rowmax(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *rowmax,
                         hipStream_t st);
hipError_t launch_mfma_i8_stream(int blocks, int iters, int32_t *sink, hipStream_t st);
// Largest L the predict kernels accept.
int predict_max_L();

}  // namespace dsa
