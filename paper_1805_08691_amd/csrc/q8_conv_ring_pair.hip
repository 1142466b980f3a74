// The pair builds of the main convolution kernel (see q8_conv_ring_kernel.h): a convolution
// with 64 or 128 filters and the 1x1 layer behind it in one launch.
#include "q8_conv_ring_kernel.h"

namespace q8 {

int launch_pair_variant(ConvParams& p, hipStream_t stream) {
  if (p.K == 64) return launch_pair<2, 2, 2, 1, 64, 2>(p, stream);     // 128 pixels x 64
  if (p.K == 128) return launch_pair<2, 4, 2, 1, 64, 4>(p, stream);    // 128 pixels x 128
  return Q8_EUNSUPPORTED;
}

}  // namespace q8
