// Tuned MFMA path (placeholder while the generic path is brought up).
#pragma once
#include "../../include/gla_decode.h"
#include "common.hpp"
namespace gla {
inline bool tuned_supported(const gla_decode_params*, int) { return false; }
inline size_t tuned_workspace(const gla_decode_params*, int) { return 0; }
inline int tuned_launch(const gla_decode_params*, int, DevParams&, hipStream_t, hipEvent_t*) {
  return GLA_ERR_UNSUPPORTED_SHAPE;
}
}  // namespace gla
