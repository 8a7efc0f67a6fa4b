// MFMA (bf16) fast path -- placeholder until the matrix-core kernels land.
#include "ssd_internal.h"

namespace ssdk {
bool mfma_path_supported(const ssd_shape_t&) { return false; }
hipError_t mfma_forward_segment(const SegParams&, bool, hipStream_t) { return hipErrorNotSupported; }
hipError_t mfma_backward_segment(const SegParams&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace ssdk
