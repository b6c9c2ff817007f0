// Host-side launchers of predict_stream.hip (streaming form of the fine-grained predictor): each validates nothing (the ABI layer did) and enqueues kernels.
#pragma once

#include "dsa_internal.h"

namespace dsa {

// The shapes the streaming kernel serves (launch_predict picks it for them) and its launch.
bool stream_predict_fits(const dsa_shape &sh);
hipError_t launch_predict_stream(const dsa_shape &sh, const int8_t *Qt, const int8_t *Kt, int32_t *idx,
                                 hipStream_t st);

}  // namespace dsa
