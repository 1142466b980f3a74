// Register-staged int8 implicit-GEMM convolution kernel (Eq. x / Eq. A' of arxiv
// 1805.08691).  Global -> registers -> LDS with one step of prefetch and two LDS buffers.
// It takes the shapes the streaming kernel does not: 4-channel images (a 16-byte chunk is
// 4 taps x 4 channels and needs per-pixel masking), fewer than 33 output channels
// (256 x 32 tile) and filters with more than 32 taps.
#include "q8_common.h"
#include "q8_conv_common.h"

namespace q8 {
namespace {

// MODE 0: C % 16 == 0 (a chunk = 16 channels of one tap).
// MODE 1: 4 stored channels per pixel (a chunk = 4 consecutive taps along the filter row).
template <int WP, int WC, int TP, int TC, int BK, int MODE>
__global__ __launch_bounds__(kThreads) void conv_i8_kernel(const ConvParams p) {
  constexpr int BP = WP * TP * 32;     // pixels per block
  constexpr int BC = WC * TC * 32;     // channels per block
  constexpr int CHUNKS = BK / 16;      // chunks per LDS row
  constexpr int ROWS_PER_PASS = kThreads / CHUNKS;
  constexpr int A_LOADS = (BC + ROWS_PER_PASS - 1) / ROWS_PER_PASS;
  constexpr int B_LOADS = BP / ROWS_PER_PASS;
  constexpr bool A_RAGGED = (BC % ROWS_PER_PASS) != 0;   // fewer filter rows than loader rows
  static_assert(WP * WC == 4, "four wavefronts per block");
  static_assert(BP % ROWS_PER_PASS == 0, "tile/loader mismatch");

  __shared__ __attribute__((aligned(16))) int8_t lds_a[2][BC * BK];
  __shared__ __attribute__((aligned(16))) int8_t lds_b[2][BP * BK];

  // XCD-aware tile order: consecutive workgroup ids go to different XCDs (each with its
  // own L2); give every XCD a contiguous run of tiles, channel tile fastest, so the
  // blocks sharing an activation tile run on the same L2.
  const int nblk = p.n_ptiles * p.n_ctiles;
  int bid = blockIdx.x;
  {
    const int xcd = bid % kNumXcd, idx = bid / kNumXcd;
    const int base = nblk / kNumXcd, rem = nblk % kNumXcd;
    bid = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  const int ctile = bid % p.n_ctiles;
  const int ptile = bid / p.n_ctiles;
  const int pix0 = ptile * BP;
  const int ch0 = ctile * BC;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_p = wave % WP;
  const int wave_c = wave / WP;

  // ---- loader state: this thread moves chunk column `lchunk` of rows lrow + j*ROWS_PER_PASS
  const int lchunk = tid % CHUNKS;
  const int lrow = tid / CHUNKS;

  int b_hi0[B_LOADS], b_wi0[B_LOADS];
  long b_img[B_LOADS];
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    int pix = pix0 + lrow + j * ROWS_PER_PASS;
    if (pix < p.M) {
      int n = pix / (p.Ho * p.Wo);
      int rem = pix - n * (p.Ho * p.Wo);
      int ho = rem / p.Wo;
      int wo = rem - ho * p.Wo;
      b_hi0[j] = ho * p.stride_h - p.pad_h;
      b_wi0[j] = wo * p.stride_w - p.pad_w;
      b_img[j] = (long)n * p.H * p.W * p.in_cs;
    } else {
      b_hi0[j] = -0x40000000;   // never inside the image
      b_wi0[j] = -0x40000000;
      b_img[j] = 0;
    }
  }
  // position of this thread's chunk in the reduction
  int red = lchunk * 16;           // byte offset in the reduction (also the filter offset)
  int tap_r, tap_s, tap_c;         // MODE 0: tap (r, s) and channel; MODE 1: r and chunk-in-row
  if constexpr (MODE == 0) {
    int tap = red / p.C;
    tap_c = red - tap * p.C;
    tap_r = tap / p.S;
    tap_s = tap - tap_r * p.S;
  } else {
    int ck = red >> 4;
    tap_r = ck / p.S4;
    tap_s = (ck - tap_r * p.S4) * 4;
    tap_c = 0;
  }

  v4i a_reg[A_LOADS], b_reg[B_LOADS];

  auto load_global = [&]() {
    const bool red_ok = red < p.red_len;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
      const int arow = lrow + j * ROWS_PER_PASS;            // LDS row <- permuted channel
      int ch = ch0 + (arow & ~31) + row_to_channel(arow & 31);
      v4i v = {0, 0, 0, 0};
      const bool row_ok = !A_RAGGED || (arow < BC);
      if (red_ok && row_ok && ch < p.K)
        v = *reinterpret_cast<const v4i*>(p.w + (size_t)ch * p.red_len + red);
      a_reg[j] = v;
    }
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
      v4i v = {0, 0, 0, 0};
      if constexpr (MODE == 0) {
        int hi = b_hi0[j] + tap_r * p.dil_h;
        int wi = b_wi0[j] + tap_s * p.dil_w;
        if (red_ok && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
          v = *reinterpret_cast<const v4i*>(p.x + b_img[j] +
                                            ((long)hi * p.W + wi) * p.in_cs + tap_c);
      } else {
        int hi = b_hi0[j] + tap_r;          // dilation 1 in this mode
        int wi = b_wi0[j] + tap_s;
        if (red_ok && (unsigned)hi < (unsigned)p.H && wi > -4 && wi < p.W) {
          const int8_t* src = p.x + b_img[j] + ((long)hi * p.W + wi) * 4;
          if (wi >= 0 && wi + 3 < p.W) {
            v = *reinterpret_cast<const v4i_a4*>(src);
          } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
              if ((unsigned)(wi + t) < (unsigned)p.W)
                v[t] = *reinterpret_cast<const int*>(src + 4 * t);
          }
        }
      }
      b_reg[j] = v;
    }
  };
  auto advance = [&]() {
    red += BK;
    if constexpr (MODE == 0) {
      tap_c += BK;
      while (tap_c >= p.C) {
        tap_c -= p.C;
        if (++tap_s == p.S) { tap_s = 0; ++tap_r; }
      }
    } else {
      int ck = red >> 4;
      tap_r = ck / p.S4;
      tap_s = (ck - tap_r * p.S4) * 4;
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
      int row = lrow + j * ROWS_PER_PASS;
      if (A_RAGGED && row >= BC) continue;
      *reinterpret_cast<v4i*>(&lds_a[buf][row * BK + swz<CHUNKS>(row, lchunk) * 16]) = a_reg[j];
    }
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
      int row = lrow + j * ROWS_PER_PASS;
      *reinterpret_cast<v4i*>(&lds_b[buf][row * BK + swz<CHUNKS>(row, lchunk) * 16]) = b_reg[j];
    }
  };

  v16i acc[TC][TP];
#pragma unroll
  for (int i = 0; i < TC; ++i)
#pragma unroll
    for (int j = 0; j < TP; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

  const int nk = (p.red_len + BK - 1) / BK;
  const int frag_row = lane & 31;       // row (A) / column (B) of the 32-wide MFMA tile
  const int frag_half = lane >> 5;      // which 16-byte half of a 32-byte reduction step

  load_global();
  store_lds(0);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) {
      advance();
      load_global();
    }
#pragma unroll
    for (int ks = 0; ks < BK / 32; ++ks) {
      v4i af[TC], bf[TP];
      const int chunk = 2 * ks + frag_half;
#pragma unroll
      for (int i = 0; i < TC; ++i) {
        int row = (wave_c * TC + i) * 32 + frag_row;
        af[i] = *reinterpret_cast<const v4i*>(&lds_a[buf][row * BK + swz<CHUNKS>(row, chunk) * 16]);
      }
#pragma unroll
      for (int j = 0; j < TP; ++j) {
        int row = (wave_p * TP + j) * 32 + frag_row;
        bf[j] = *reinterpret_cast<const v4i*>(&lds_b[buf][row * BK + swz<CHUNKS>(row, chunk) * 16]);
      }
#pragma unroll
      for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: a lane holds 16 consecutive channels of pixel column (lane & 31).
  // A complete tile with aligned rows takes the branch-free path.
  const bool fast_tile =
      p.vec16 && !p.acc_dump && !p.y_f32 && !p.y_deq && ch0 + BC <= p.K && pix0 + BP <= p.M;
#pragma unroll
  for (int j = 0; j < TP; ++j) {
    const int pix = pix0 + (wave_p * TP + j) * 32 + (lane & 31);
    if (pix >= p.M) continue;
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      const int ch = ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5);
      if (ch >= p.K) continue;
      int v[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) v[e] = acc[i][j][e];
      if (fast_tile) {
        int b[16], rw[4];
        load_bias16(p, ch, b);
        load_res16(p, pix, ch, rw);
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] += b[e];
        const float no_scales[16] = {};
        if (p.res) finish16_fast<true>(p, pix, ch, v, rw, no_scales);
        else finish16_fast<false>(p, pix, ch, v, rw, no_scales);
      } else {
        epilogue16(p, pix, ch, v);
      }
    }
  }
}

template <int WP, int WC, int TP, int TC, int MODE>
int launch_reg(ConvParams& p, hipStream_t stream) {
  constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
  p.n_ptiles = (p.M + BP - 1) / BP;
  p.n_ctiles = (p.K + BC - 1) / BC;
  long nblk = (long)p.n_ptiles * p.n_ctiles;
  if (nblk > 0x7fffffffL) return Q8_EUNSUPPORTED;
  hipLaunchKernelGGL((conv_i8_kernel<WP, WC, TP, TC, 64, MODE>), dim3((unsigned)nblk), dim3(kThreads),
                     0, stream, p);
  return q8_launch_status();
}

const char* const kRegNames[6] = {
    "conv_i8_kernel<2,2,2,2,64,0>", "conv_i8_kernel<4,1,2,2,64,0>", "conv_i8_kernel<4,1,2,1,64,0>",
    "conv_i8_kernel<2,2,2,2,64,1>", "conv_i8_kernel<4,1,2,2,64,1>", "conv_i8_kernel<4,1,2,1,64,1>"};

}  // namespace

// variant = 3 * mode + {0: 128 pixels x 128 channels, 1: 256 x 64, 2: 256 x 32}
int launch_reg_variant(int variant, ConvParams& p, hipStream_t stream) {
  switch (variant) {
    case 0: return launch_reg<2, 2, 2, 2, 0>(p, stream);
    case 1: return launch_reg<4, 1, 2, 2, 0>(p, stream);
    case 2: return launch_reg<4, 1, 2, 1, 0>(p, stream);
    case 3: return launch_reg<2, 2, 2, 2, 1>(p, stream);
    case 4: return launch_reg<4, 1, 2, 2, 1>(p, stream);
    case 5: return launch_reg<4, 1, 2, 1, 1>(p, stream);
    default: return Q8_EINVAL;
  }
}
const char* reg_variant_name(int variant) {
  return variant >= 0 && variant < 6 ? kRegNames[variant] : "unsupported";
}

}  // namespace q8
