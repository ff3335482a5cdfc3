// Matrix-core convolution, fp32 operands (v_mfma_f32_32x32x2_f32), and the shape predicates
// shared by all operand modes.  The kernel itself is in conv_mfma_impl.h.
#include "conv_mfma_impl.h"

namespace evk {

bool conv_mfma_f32_supported(const ConvParams& p) {
  return p.gi.c >= 9 && p.go.c >= 16 && p.c_out_pad == (p.go.c + 31) / 32 * 32 &&  // (fewer input channels: the narrow-input kernel)
         (long long)p.gi.h * p.gi.w * p.gi.c * 4 < (1ll << 31) &&  // byte offsets of the gather fit 31 bits
         (long long)(p.go.h + 8) * p.go.w * p.go.c * 4 < (1ll << 31) &&  // those of the epilogue too
         (long long)p.k * p.k * ((p.gi.c + 127) / 128 * 128) * p.c_out_pad * 8 < (1ll << 31);  // and those of both weight planes
}
// a bilinear x2 up-sampling in front of this conv can be folded into its gather
bool conv_mfma_upsample_supported(const ConvParams& p) {
  return conv_mfma_f32_supported(p) && chunk_for(p) == 32 && p.stride == 1 && p.k <= 7;
}
// input channels of the re-laid weights: c_in rounded up to whole chunks of the variant that runs
int conv_mfma_padded_cin(const ConvParams& p) {
  const int chunk = chunk_for(p);
  return (p.gi.c + chunk - 1) / chunk * chunk;
}
void launch_conv_mfma_f32(const ConvParams& p, hipStream_t s) { launch_any<kOpF32>(p, s); }
int conv_mfma_f32_phase_stamps(unsigned long long* host, int max_records, bool reset) {
  return phase_stamps_read(host, max_records, reset);
}

}  // namespace evk
