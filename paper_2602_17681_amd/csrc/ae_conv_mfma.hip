// ae_conv_mfma.hip — implicit-GEMM convolution on the matrix cores (placeholder:
// every shape is routed to the direct kernels until the MFMA kernels land).
#include "ae_device.h"
#include "ae_internal.h"

namespace ae {

bool conv_mfma_supported(const ConvArgs&) { return false; }
int conv_partial_rows(const ConvArgs&, bool) { return kReduceRows; }
int launch_conv_mfma(const ConvArgs&, hipStream_t) { return fail(AE_EINVAL, "conv_mfma: shape not supported"); }

}  // namespace ae
