// The builds of the persistent 3x3 tile family (see q8_conv_p3_kernel.h, q8_conv_p3b_kernel.h)
// and their table.  A
// build asked for a layer it cannot take hands the layer to the generic kernel.
#include "q8_conv_p3_kernel.h"
#include "q8_conv_p3b_kernel.h"

namespace q8 {
namespace {

template <int PL>
int launch_p3_or_generic(ConvParams& p, hipStream_t stream) {
  if (p3_applicable<PL>(p)) return launch_p3<PL>(p, stream);
  return launch_ring<2, 2, 2, 2, 64, 3, 0>(p, stream);
}

int launch_p3b_or_generic(ConvParams& p, hipStream_t stream) {
  if (p3b_applicable(p)) return launch_p3b(p, stream);
  return launch_ring<2, 2, 2, 2, 64, 3, 0>(p, stream);
}

struct P3Variant {
  const char* name;
  int (*launch)(ConvParams&, hipStream_t);
};
const P3Variant kP3Variants[] = {
    {"conv_i8_p3_kernel<4>", &launch_p3_or_generic<4>},     // maps up to 63 pixels wide
    {"conv_i8_p3_kernel<6>", &launch_p3_or_generic<6>},     // up to 127
    {"conv_i8_p3b_kernel", &launch_p3b_or_generic},         // 8 x 16 blocks: maps of any width
};
constexpr int kNumP3Variants = sizeof(kP3Variants) / sizeof(kP3Variants[0]);

}  // namespace

int num_p3_variants() { return kNumP3Variants; }
int launch_p3_variant(int variant, ConvParams& p, hipStream_t stream) {
  if (variant < 0 || variant >= kNumP3Variants) return Q8_EINVAL;
  return kP3Variants[variant].launch(p, stream);
}
const char* p3_variant_name(int variant) {
  return variant >= 0 && variant < kNumP3Variants ? kP3Variants[variant].name : "unsupported";
}

}  // namespace q8
