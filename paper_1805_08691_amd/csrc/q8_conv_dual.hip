// Two independent convolution layers in ONE launch (each Eq. A' exactly as q8_conv_int8
// computes it): the workgroups of the grid are dealt to the first layer's tiles, then to the
// second's.  Meant for layers that read the same tensor and do not depend on each other (the
// projection branch and the first 1x1 of a residual stage): one launch gap, one ramp-up and
// one tail instead of two, and the shared input is fetched while it is still in the L2.
#include "q8_conv_ring_kernel.h"

namespace q8 {
namespace {

template <int TP1, int TC1, int ST1, int TP2, int TC2, int ST2>
__global__ __launch_bounds__(256) void conv_i8_dual_kernel(const ConvParams p1, const ConvParams p2) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  const int n1 = p1.n_ptiles * p1.n_ctiles;
  int bid = blockIdx.x;
  if (bid < n1) {
    const int xcd = bid % kNumXcd, idx = bid / kNumXcd;
    const int base = n1 / kNumXcd, rem = n1 % kNumXcd;
    bid = xcd * base + (xcd < rem ? xcd : rem) + idx;
    conv_tile_ring<2, 2, TP1, TC1, 64, ST1, 1, 0>(p1, bid / p1.n_ctiles, bid % p1.n_ctiles, lds);
  } else {
    // workgroups n1 + 8k + r all sit on one XCD: the same renumbering on the local index
    bid -= n1;
    const int n2 = p2.n_ptiles * p2.n_ctiles;
    const int xcd = bid % kNumXcd, idx = bid / kNumXcd;
    const int base = n2 / kNumXcd, rem = n2 % kNumXcd;
    bid = xcd * base + (xcd < rem ? xcd : rem) + idx;
    conv_tile_ring<2, 2, TP2, TC2, 64, ST2, 1, 0>(p2, bid / p2.n_ctiles, bid % p2.n_ctiles, lds);
  }
#endif
}

template <int TP1, int TC1, int ST1, int TP2, int TC2, int ST2>
int launch_dual(ConvParams& p1, ConvParams& p2, hipStream_t stream) {
  constexpr int BP1 = 2 * TP1 * 32, BC1 = 2 * TC1 * 32, BP2 = 2 * TP2 * 32, BC2 = 2 * TC2 * 32;
  constexpr int L1 = ST1 * (BP1 + BC1) * 64, L2 = ST2 * (BP2 + BC2) * 64;
  constexpr int kLds = L1 > L2 ? L1 : L2;
  static_assert(kLds <= 65536, "within the default dynamic LDS limit");
  p1.n_ptiles = (p1.M + BP1 - 1) / BP1; p1.n_ctiles = (p1.K + BC1 - 1) / BC1;
  p2.n_ptiles = (p2.M + BP2 - 1) / BP2; p2.n_ctiles = (p2.K + BC2 - 1) / BC2;
  const long nblk = (long)p1.n_ptiles * p1.n_ctiles + (long)p2.n_ptiles * p2.n_ctiles;
  if (nblk > 0x7fffffffL) return Q8_EUNSUPPORTED;
  hipLaunchKernelGGL((conv_i8_dual_kernel<TP1, TC1, ST1, TP2, TC2, ST2>), dim3((unsigned)nblk),
                     dim3(256), kLds, stream, p1, p2);
  return q8_launch_status();
}

}  // namespace

namespace {
// Tile shape of one layer by its size (four wavefronts each): 0 = 128 x 64 ring of 2,
// 1 = 128 x 128 ring of 3, 2 = 64 x 128 ring of 4, 3 = 64 x 64 ring of 4.
int dual_shape(const ConvParams& p) {
  const long t128 = ((long)(p.M + 127) / 128) * ((p.K + 127) / 128);
  const int nk = (p.red_len + 63) / 64;
  if (p.K <= 64) return 0;
  if (t128 >= 300 && nk > 4) return 1;
  if (nk <= 4 && t128 >= 512) return 0;
  if (t128 <= 64) return 3;
  return 2;
}
using DualLaunch = int (*)(ConvParams&, ConvParams&, hipStream_t);
DualLaunch dual_lookup(int s1, int s2) {
#define Q8_DUAL(A, B, ...) if (s1 == A && s2 == B) return &launch_dual<__VA_ARGS__>;
  Q8_DUAL(0, 0, 2, 1, 2, 2, 1, 2)
  Q8_DUAL(0, 2, 2, 1, 2, 1, 2, 4)
  Q8_DUAL(0, 3, 2, 1, 2, 1, 1, 4)
  Q8_DUAL(1, 0, 2, 2, 3, 2, 1, 2)
  Q8_DUAL(1, 1, 2, 2, 3, 2, 2, 3)
  Q8_DUAL(1, 2, 2, 2, 3, 1, 2, 4)
  Q8_DUAL(1, 3, 2, 2, 3, 1, 1, 4)
  Q8_DUAL(2, 2, 1, 2, 4, 1, 2, 4)
  Q8_DUAL(2, 3, 1, 2, 4, 1, 1, 4)
  Q8_DUAL(3, 3, 1, 1, 4, 1, 1, 4)
#undef Q8_DUAL
  return nullptr;
}
}  // namespace

bool dual_shapes_supported(const ConvParams& p1, const ConvParams& p2) {
  return dual_lookup(dual_shape(p1), dual_shape(p2)) != nullptr;
}
int launch_dual_variant(ConvParams& p1, ConvParams& p2, hipStream_t stream) {
  const DualLaunch f = dual_lookup(dual_shape(p1), dual_shape(p2));
  return f ? f(p1, p2, stream) : Q8_EUNSUPPORTED;
}

}  // namespace q8
