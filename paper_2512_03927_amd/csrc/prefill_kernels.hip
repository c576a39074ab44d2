// Prefill path (paper Section 3.3): tokens grouped by expert, one grouped GEMM per expert on
// the matrix cores.  (Placeholder until the MFMA kernels land: reports "not supported".)
#include "kernels.h"

namespace odmoe {

size_t prefill_workspace_bytes(const Shape&, int32_t) { return 256; }

hipError_t launch_prefill(hipStream_t, const Shape&, const void* const*, int32_t, const int32_t*,
                          const float*, const void*, int32_t, void*, void*, size_t) {
  return hipErrorNotSupported;
}

}  // namespace odmoe
