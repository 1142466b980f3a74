// The build of the image-row tile family (see q8_conv_stem_kernel.h) and its table.  A layer
// the build cannot take goes to the generic kernel.
#include "q8_conv_stem_kernel.h"

namespace q8 {
namespace {

int launch_stem_or_generic(ConvParams& p, hipStream_t stream) {
  if (stem_applicable(p)) return launch_stem(p, stream);
  return launch_ring<2, 2, 2, 1, 64, 2, 0>(p, stream);
}

struct StemVariant {
  const char* name;
  int (*launch)(ConvParams&, hipStream_t);
};
const StemVariant kStemVariants[] = {
    {"conv_i8_stem_kernel", &launch_stem_or_generic},
};
constexpr int kNumStemVariants = sizeof(kStemVariants) / sizeof(kStemVariants[0]);

}  // namespace

int num_stem_variants() { return kNumStemVariants; }
int launch_stem_variant(int variant, ConvParams& p, hipStream_t stream) {
  if (variant < 0 || variant >= kNumStemVariants) return Q8_EINVAL;
  return kStemVariants[variant].launch(p, stream);
}
const char* stem_variant_name(int variant) {
  return variant >= 0 && variant < kNumStemVariants ? kStemVariants[variant].name : "unsupported";
}

}  // namespace q8
