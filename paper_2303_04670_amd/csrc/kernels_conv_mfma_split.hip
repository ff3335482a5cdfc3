// Matrix-core convolution, fp32 weights and increments each split into bf16 high + low parts:
// three bf16 MFMAs per product with fp32 accumulation; weights are [2 planes][tap][c_in/8][c_out][8]
// bf16.  The kernel itself is in conv_mfma_impl.h.
#include "conv_mfma_impl.h"

namespace evk {

bool conv_mfma_split_supported(const ConvParams& p) { return conv_mfma_f32_supported(p); }
void launch_conv_mfma_split(const ConvParams& p, hipStream_t s) { launch_any<kOpSplit>(p, s); }
int conv_mfma_split_phase_stamps(unsigned long long* host, int max_records, bool reset) {
  return phase_stamps_read(host, max_records, reset);
}

}  // namespace evk
