// The builds of the pointwise tile family (see q8_conv_pw_kernel.h) and their table.  A build
// asked for a layer it cannot take hands the layer to the generic kernel.
#include "q8_conv_pw_kernel.h"

namespace q8 {
namespace {

template <int TC, int KS>
int launch_pw_or_generic(ConvParams& p, hipStream_t stream) {
  if (pw_applicable<TC, KS>(p)) return launch_pw<TC, KS>(p, stream);
  return launch_ring<2, 2, 2, 2, 64, 3, 0>(p, stream);
}

struct PwVariant {
  const char* name;
  int (*launch)(ConvParams&, hipStream_t);
};
#define Q8_PW_ROW(TC, KS) { "conv_i8_pw_kernel<" #TC "," #KS ">", &launch_pw_or_generic<TC, KS> },
const PwVariant kPwVariants[] = {
    Q8_PW_ROW(1, 1)    // 0: 128 pixels x 64 channels, C = 64
    Q8_PW_ROW(2, 1)    // 1: 128 x 128, C = 64
    Q8_PW_ROW(1, 2)    // 2: 128 x 64, C = 128
    Q8_PW_ROW(2, 2)    // 3: 128 x 128, C = 128
    Q8_PW_ROW(1, 4)    // 4: 128 x 64, C = 256
    Q8_PW_ROW(2, 4)    // 5: 128 x 128, C = 256
};
#undef Q8_PW_ROW
constexpr int kNumPwVariants = sizeof(kPwVariants) / sizeof(kPwVariants[0]);

}  // namespace

int num_pw_variants() { return kNumPwVariants; }
int launch_pw_variant(int variant, ConvParams& p, hipStream_t stream) {
  if (variant < 0 || variant >= kNumPwVariants) return Q8_EINVAL;
  return kPwVariants[variant].launch(p, stream);
}
const char* pw_variant_name(int variant) {
  return variant >= 0 && variant < kNumPwVariants ? kPwVariants[variant].name : "unsupported";
}

}  // namespace q8
