// Sparse incremental convolution on the matrix cores (fp32 MFMA) - placeholder until built.
#include "evconv_kernels.h"

namespace evk {
bool conv_mfma_f32_supported(const ConvParams&) { return false; }
void launch_conv_mfma_f32(const ConvParams& p, hipStream_t s) { launch_conv_valu(p, s); }
}  // namespace evk
