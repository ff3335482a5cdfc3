// Matrix-core convolution, bf16 operands with fp32 accumulation (v_mfma_f32_32x32x16_bf16);
// weights are [tap][c_in/8][c_out][8] bf16.  The kernel itself is in conv_mfma_impl.h.
#include "conv_mfma_impl.h"

namespace evk {

bool conv_mfma_bf16_supported(const ConvParams& p) { return conv_mfma_f32_supported(p); }
void launch_conv_mfma_bf16(const ConvParams& p, hipStream_t s) { launch_any<kOpBf16>(p, s); }
int conv_mfma_bf16_phase_stamps(unsigned long long* host, int max_records, bool reset) {
  return phase_stamps_read(host, max_records, reset);
}

}  // namespace evk
