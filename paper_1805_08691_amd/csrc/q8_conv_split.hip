// The split-reduction builds of the main convolution kernel (see SPLIT in
// q8_conv_ring_kernel.h) and their table.  A layer the builds cannot take, or a call without
// a split factor, goes to the generic kernel.
#include "q8_conv_ring_kernel.h"

namespace q8 {
namespace {

template <int WP, int WC, int TP, int TC, int BK, int ST>
int launch_split_or_generic(ConvParams& p, hipStream_t stream) {
  if (p.n_split >= 2 && split_applicable(p) && p.C % BK == 0)
    return launch_ring_split<WP, WC, TP, TC, BK, ST>(p, stream);
  p.n_split = 1;
  return launch_ring<2, 2, 2, 2, 64, 3, 0>(p, stream);
}

struct SplitVariant {
  const char* name;
  int bp, bc;       // tile: pixels x channels
  int (*launch)(ConvParams&, hipStream_t);
};
#define Q8_SPLIT_ROW(WP, WC, TP, TC, BK, ST)                                      \
  { "conv_i8_ring_split_kernel<" #WP "," #WC "," #TP "," #TC "," #BK "," #ST ">", \
    WP * TP * 32, WC * TC * 32, &launch_split_or_generic<WP, WC, TP, TC, BK, ST> },
const SplitVariant kSplitVariants[] = {
    Q8_SPLIT_ROW(2, 2, 2, 2, 64, 3)    // 0: 128 x 128
    Q8_SPLIT_ROW(2, 2, 2, 2, 64, 4)    // 1
    Q8_SPLIT_ROW(2, 2, 2, 1, 64, 4)    // 2: 128 x 64
    Q8_SPLIT_ROW(2, 2, 1, 2, 64, 4)    // 3: 64 x 128
    Q8_SPLIT_ROW(2, 2, 1, 1, 64, 4)    // 4: 64 x 64
    Q8_SPLIT_ROW(2, 4, 2, 1, 64, 4)    // 5: 128 x 128, eight wavefronts
};
#undef Q8_SPLIT_ROW
constexpr int kNumSplitVariants = sizeof(kSplitVariants) / sizeof(kSplitVariants[0]);

}  // namespace

int num_split_variants() { return kNumSplitVariants; }
void split_variant_tile(int variant, int* bp, int* bc) {
  *bp = kSplitVariants[variant].bp;
  *bc = kSplitVariants[variant].bc;
}
int launch_split_variant(int variant, ConvParams& p, hipStream_t stream) {
  if (variant < 0 || variant >= kNumSplitVariants) return Q8_EINVAL;
  return kSplitVariants[variant].launch(p, stream);
}
const char* split_variant_name(int variant) {
  return variant >= 0 && variant < kNumSplitVariants ? kSplitVariants[variant].name : "unsupported";
}

}  // namespace q8
