// Implicit-GEMM convolution on the matrix cores (placeholder: no shape is taken yet).
#include "common.hpp"

namespace wmdec {

bool conv_mfma_supported(const ConvArgs&) { return false; }

int launch_conv_mfma(const ConvArgs&, hipStream_t) {
  set_error("conv_mfma: not available");
  return WMDEC_ERR_UNSUPPORTED;
}

}  // namespace wmdec
