// The builds of the image-row tile family (see q8_conv_stem_kernel.h) and their table: codes
// in memory with vertical stride 1 or 2, and the real-valued image with Eq. Q applied on the
// way in, with or without the max-pool behind the layer.  A layer a build cannot take goes to
// the generic kernel (codes) or is reported as unsupported (real-valued image).
#include "q8_conv_stem_kernel.h"

namespace q8 {
namespace {

int launch_stem_or_generic(ConvParams& p, hipStream_t stream) {
  const StemImage none{};
  if (stem_applicable<2>(p)) return launch_stem<2, false, false>(p, none, stream);
  if (stem_applicable<1>(p)) return launch_stem<1, false, false>(p, none, stream);
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

// Eq. Q + the layer (+ the 3x3 / 2 max-pool): p describes the layer over the zero frame, im
// the image inside it.  dry_run: only say whether a build takes it.
int launch_stem_image(ConvParams& p, const StemImage& im, int pool, bool dry_run,
                      hipStream_t stream) {
  const bool fits = im.top >= 0 && im.left >= 0 && im.top + im.H <= p.H && im.left + im.W <= p.W &&
                    im.W <= 256 && im.C >= 1 && im.C <= 4;
  if (!fits) return Q8_EUNSUPPORTED;
  if (pool) {
    if (!stem_applicable<2>(p) || im.Wp * 4 > 256 ||
        (long)p.N * im.Hp * im.Wp * p.out_cs >= 0x7fffffffL)
      return Q8_EUNSUPPORTED;
    return dry_run ? Q8_OK : launch_stem<2, true, true>(p, im, stream);
  }
  if (stem_applicable<2>(p)) return dry_run ? Q8_OK : launch_stem<2, true, false>(p, im, stream);
  if (stem_applicable<1>(p)) return dry_run ? Q8_OK : launch_stem<1, true, false>(p, im, stream);
  return Q8_EUNSUPPORTED;
}

}  // namespace q8
