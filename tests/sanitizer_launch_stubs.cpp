// Stand-ins for the kernel launchers of libmosaic, used ONLY by tests/test_sanitized_host_code.py: that test builds
// the host side of the library (argument validation, the chunk-size selector, the graph planner, the VMM object)
// with AddressSanitizer and UndefinedBehaviorSanitizer and runs the CPU tests against it.  No kernel is launched in
// those tests (there is no GPU), so the launchers only have to exist.
#include "mosaic_internal.h"

namespace mosaic {
int launch_compact(const uint8_t*, int64_t, int32_t*, int32_t*, int32_t*, hipStream_t) { return -1; }
int launch_masked_logits(const LogitsArgs&, const mosaic_plan&, hipStream_t) { return -1; }
int launch_unmask_topn(const float*, const int32_t*, const int32_t*, const int32_t*, int64_t, const int32_t*, int32_t,
                       const int32_t*, int32_t*, uint8_t*, int64_t, hipStream_t) { return -1; }
int launch_shift_indices(const int32_t*, const int32_t*, int64_t, const int32_t*, int32_t, int32_t*, hipStream_t) {
  return -1;
}
int launch_mfma_probe(const void*, float*, int32_t, int32_t, hipStream_t) { return -1; }
}  // namespace mosaic
