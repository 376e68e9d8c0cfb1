// CSC (sparse) design: placeholders until the sparse kernels are in.
#include "strads_internal.h"

namespace strads {
size_t csc_scratch_bytes(int64_t, int32_t) { return 0; }
hipError_t launch_gram_csc(strads_lasso *) { return hipErrorNotSupported; }
hipError_t launch_dots_csc(strads_lasso *) { return hipErrorNotSupported; }
hipError_t launch_residual_csc(strads_lasso *) { return hipErrorNotSupported; }
hipError_t launch_kkt_csc(strads_lasso *, float *) { return hipErrorNotSupported; }
} // namespace strads
