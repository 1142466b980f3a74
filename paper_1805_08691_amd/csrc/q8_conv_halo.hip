// The builds of the 3x3 tile family (see q8_conv_halo_kernel.h) and their table.  A variant
// asked for a layer it cannot take (not 3x3 / stride 1 / padding 1, C % 64 != 0, a map wider
// than its patch buffer holds) hands the layer to the generic kernel.
#include "q8_conv_halo_kernel.h"

namespace q8 {
namespace {

template <int WP, int WC, int TP, int TC, int PL, int KW = 1, int ST = 3>
int launch_halo3_or_generic(ConvParams& p, hipStream_t stream) {
  if (halo3_applicable<WP, WC, TP, TC, PL, KW>(p))
    return launch_halo3<WP, WC, TP, TC, PL, KW, ST>(p, stream);
  if (KW > 1 && halo3_applicable<WP, WC, TP, TC, PL>(p))      // an odd number of chunks
    return launch_halo3<WP, WC, TP, TC, PL, 1, ST>(p, stream);
  return launch_ring<2, 2, 2, 2, 64, 3, 0>(p, stream);
}

struct HaloVariant {
  const char* name;
  int (*launch)(ConvParams&, hipStream_t);
  int bp, bc, max_w;
};
#define Q8_HALO_ROW(WP, WC, TP, TC, PL)                                        \
  { "conv_i8_halo3_kernel<" #WP "," #WC "," #TP "," #TC "," #PL ">",            \
    &launch_halo3_or_generic<WP, WC, TP, TC, PL>, WP * TP * 32, WC * TC * 32,   \
    HaloShape<WP, WC, TP, TC, PL>::max_w() },
const HaloVariant kHaloVariants[] = {
    Q8_HALO_ROW(2, 2, 2, 1, 4)     // 0: 128 pixels x 64 channels, maps up to 63 wide
    Q8_HALO_ROW(2, 2, 2, 2, 4)     // 1: 128 x 128
    Q8_HALO_ROW(4, 2, 2, 2, 4)     // 2: 256 x 128, eight wavefronts, maps up to 127 wide
    Q8_HALO_ROW(4, 2, 2, 2, 8)     // 3: 256 x 128, maps up to 383 wide
    Q8_HALO_ROW(2, 2, 2, 1, 8)     // 4: 128 x 64, maps up to 191 wide
    Q8_HALO_ROW(4, 1, 2, 2, 14)    // 5: 256 x 64, maps up to 319 wide
    Q8_HALO_ROW(2, 2, 1, 1, 2)     // 6: 64 x 64, maps up to 31 wide
    Q8_HALO_ROW(2, 2, 1, 2, 2)     // 7: 64 x 128, maps up to 31 wide
    // the reduction split over two groups of four wavefronts
    { "conv_i8_halo3_kernel<2,2,1,1,2,2>", &launch_halo3_or_generic<2, 2, 1, 1, 2, 2>, 64, 64,
      HaloShape<2, 2, 1, 1, 2, 2>::max_w() },                   // 8: 64 x 64
    { "conv_i8_halo3_kernel<2,2,1,2,2,2>", &launch_halo3_or_generic<2, 2, 1, 2, 2, 2>, 64, 128,
      HaloShape<2, 2, 1, 2, 2, 2>::max_w() },                   // 9: 64 x 128
    { "conv_i8_halo3_kernel<2,2,2,1,4,2>", &launch_halo3_or_generic<2, 2, 2, 1, 4, 2>, 128, 64,
      HaloShape<2, 2, 2, 1, 4, 2>::max_w() },                   // 10: 128 x 64
    // a filter ring of nine slabs (eight in flight)
    { "conv_i8_halo3_kernel<2,2,1,1,2,1,9>", &launch_halo3_or_generic<2, 2, 1, 1, 2, 1, 9>, 64, 64,
      HaloShape<2, 2, 1, 1, 2>::max_w() },                      // 11: 64 x 64
    { "conv_i8_halo3_kernel<2,2,1,1,2,2,9>", &launch_halo3_or_generic<2, 2, 1, 1, 2, 2, 9>, 64, 64,
      HaloShape<2, 2, 1, 1, 2>::max_w() },                      // 12: 64 x 64, two groups
    { "conv_i8_halo3_kernel<2,2,1,2,2,1,9>", &launch_halo3_or_generic<2, 2, 1, 2, 2, 1, 9>, 64, 128,
      HaloShape<2, 2, 1, 2, 2>::max_w() },                      // 13: 64 x 128
};
#undef Q8_HALO_ROW
constexpr int kNumHaloVariants = sizeof(kHaloVariants) / sizeof(kHaloVariants[0]);

}  // namespace

int num_halo_variants() { return kNumHaloVariants; }
int launch_halo_variant(int variant, ConvParams& p, hipStream_t stream) {
  if (variant < 0 || variant >= kNumHaloVariants) return Q8_EINVAL;
  return kHaloVariants[variant].launch(p, stream);
}
const char* halo_variant_name(int variant) {
  return variant >= 0 && variant < kNumHaloVariants ? kHaloVariants[variant].name : "unsupported";
}
int halo_variant_max_w(int variant) {
  return variant >= 0 && variant < kNumHaloVariants ? kHaloVariants[variant].max_w : 0;
}

}  // namespace q8
