// The plain builds of the main convolution kernel (see q8_conv_ring_kernel.h) and the table
// of tile / ring variants.  The extended builds (unsigned codes, per-channel scales) and the
// pair builds are compiled in files of their own, so the three compile side by side.
#include "q8_conv_ring_kernel.h"

namespace q8 {
namespace {

struct RingVariant {
  const char* name;
  int (*launch)(ConvParams&, hipStream_t);
};
#define Q8_RING_ROW(I, WP, WC, TP, TC, BK, ST) \
  { "conv_i8_ring_kernel<" #WP "," #WC "," #TP "," #TC "," #BK "," #ST ">", \
    &launch_ring<WP, WC, TP, TC, BK, ST, 0> },
const RingVariant kRingVariants[] = {
    Q8_RING_EXT_LIST(Q8_RING_ROW)          //  0 .. 11: also in the extended build
    Q8_RING_ROW(12, 4, 2, 1, 2, 64, 3)     // 12: 128 x 128, eight wavefronts of 32 x 64
    Q8_RING_ROW(13, 4, 2, 2, 2, 64, 3)     // 13: 256 x 128, eight wavefronts of 64 x 64
    Q8_RING_ROW(14, 2, 4, 2, 2, 64, 3)     // 14: 128 x 256, eight wavefronts of 64 x 64
    Q8_RING_ROW(15, 2, 2, 2, 2, 64, 6)     // 15: 128 x 128, deep rings for one workgroup per CU
    Q8_RING_ROW(16, 2, 2, 2, 2, 64, 8)     // 16
    Q8_RING_ROW(17, 2, 4, 2, 1, 64, 8)     // 17: the same with eight wavefronts
    Q8_RING_ROW(18, 2, 2, 2, 1, 64, 8)     // 18: 128 x 64, deep ring
    Q8_RING_ROW(19, 2, 2, 1, 1, 64, 8)     // 19: 64 x 64, deep ring (small maps, long reductions)
    Q8_RING_ROW(20, 2, 2, 1, 2, 64, 8)     // 20: 64 x 128, deep ring
    Q8_RING_ROW(21, 2, 2, 1, 1, 128, 4)    // 21: 64 x 64, 128 reduction bytes per step
    Q8_RING_ROW(22, 2, 2, 1, 2, 128, 4)    // 22: 64 x 128, 128 reduction bytes per step
    Q8_RING_ROW(23, 2, 2, 2, 1, 128, 4)    // 23: 128 x 64, 128 reduction bytes per step
    Q8_RING_ROW(24, 2, 2, 1, 1, 128, 8)    // 24: 64 x 64, 128 bytes per step, deep ring (128 KB)
};
#undef Q8_RING_ROW
constexpr int kNumRingVariants = sizeof(kRingVariants) / sizeof(kRingVariants[0]);

}  // namespace

// The variant numbers continue into the 3x3 tile family (q8_conv_halo.hip).
int num_halo_variants();
int launch_halo_variant(int variant, ConvParams& p, hipStream_t stream);
const char* halo_variant_name(int variant);

// ... and into the pointwise tile family (q8_conv_pw.hip)
int num_pw_variants();
int launch_pw_variant(int variant, ConvParams& p, hipStream_t stream);
const char* pw_variant_name(int variant);

// ... and into the split-reduction builds (q8_conv_split.hip)
int num_split_variants();
int launch_split_variant(int variant, ConvParams& p, hipStream_t stream);
const char* split_variant_name(int variant);

// ... and the persistent 3x3 family (q8_conv_p3.hip)
int num_p3_variants();
int launch_p3_variant(int variant, ConvParams& p, hipStream_t stream);
const char* p3_variant_name(int variant);

// ... and the image-row family (q8_conv_stem.hip)
int num_stem_variants();
int launch_stem_variant(int variant, ConvParams& p, hipStream_t stream);
const char* stem_variant_name(int variant);

int num_ring_variants() { return kNumRingVariants; }
int first_pw_variant() { return kNumRingVariants + num_halo_variants(); }
int first_split_variant() { return first_pw_variant() + num_pw_variants(); }
int first_p3_variant() { return first_split_variant() + num_split_variants(); }
int first_stem_variant() { return first_p3_variant() + num_p3_variants(); }
int num_stream_variants() { return first_stem_variant() + num_stem_variants(); }
int launch_stream_variant(int variant, ConvParams& p, hipStream_t stream) {
  if (variant < 0 || variant >= num_stream_variants()) return Q8_EINVAL;
  if (p.in_u8 | p.out_u8 | p.res_u8 | (p.m_vec != nullptr)) {
    // variants without an extended build fall back to the 128 x 128 ring of 3
    return launch_ring_ext_variant(variant < kNumRingExtVariants ? variant : 1, p, stream);
  }
  if (variant >= first_stem_variant())
    return launch_stem_variant(variant - first_stem_variant(), p, stream);
  if (variant >= first_p3_variant()) return launch_p3_variant(variant - first_p3_variant(), p, stream);
  if (variant >= first_split_variant())
    return launch_split_variant(variant - first_split_variant(), p, stream);
  if (variant >= first_pw_variant()) return launch_pw_variant(variant - first_pw_variant(), p, stream);
  if (variant >= kNumRingVariants) return launch_halo_variant(variant - kNumRingVariants, p, stream);
  return kRingVariants[variant].launch(p, stream);
}
const char* stream_variant_name(int variant) {
  if (variant >= first_stem_variant()) return stem_variant_name(variant - first_stem_variant());
  if (variant >= first_p3_variant()) return p3_variant_name(variant - first_p3_variant());
  if (variant >= first_split_variant()) return split_variant_name(variant - first_split_variant());
  if (variant >= first_pw_variant()) return pw_variant_name(variant - first_pw_variant());
  if (variant >= kNumRingVariants) return halo_variant_name(variant - kNumRingVariants);
  return variant >= 0 ? kRingVariants[variant].name : "unsupported";
}

}  // namespace q8
