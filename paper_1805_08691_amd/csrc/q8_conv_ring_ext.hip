// The extended builds of the main convolution kernel (see q8_conv_ring_kernel.h): unsigned
// activation codes (border correction, unsigned residual / output) and per-output-channel
// scales.
#include "q8_conv_ring_kernel.h"

namespace q8 {

int launch_ring_ext_variant(int variant, ConvParams& p, hipStream_t stream) {
  switch (variant) {
#define Q8_RING_CASE(I, WP, WC, TP, TC, BK, ST) \
  case I:                                       \
    return launch_ring<WP, WC, TP, TC, BK, ST, 1>(p, stream);
    Q8_RING_EXT_LIST(Q8_RING_CASE)
#undef Q8_RING_CASE
    default:
      return Q8_EINVAL;
  }
}

}  // namespace q8
