// Matrix-core kernel family (fp32).  No shape is served yet.
#include "sig_internal.h"

namespace sig {

const char *mfma_kernel_name(const Shape &) { return nullptr; }

hipError_t launch_mfma_f32(const Shape &, const float *, float *, hipStream_t) { return hipErrorNotSupported; }

}  // namespace sig
