// The 3x3 tile family of the int8 convolution (Eq. x / Eq. A' of arxiv 1805.08691): R = S = 3,
// stride 1, dilation 1, padding 1, C % 64 == 0.
//
// In the generic kernel every filter tap is a reduction step of its own that fetches the
// tap's activation rows again: nine fetches of (almost) the same pixels, all of them through
// the compute unit's one 64 B/clk path from the L2 into LDS, which is what bounds that kernel
// on 3x3 layers.  Here the activations of a tile are staged ONCE per 64-channel chunk as a
// patch with its halo and the nine taps read it at nine row offsets:
//
//  * In (n, h, w) pixel order the input pixel that output pixel i reads at tap (r, s) is
//    pixel i + (r-1) W + (s-1) whenever that tap lies inside the image.  The patch of a tile
//    of BP consecutive output pixels is therefore the BP + 2W + 2 consecutive input pixels
//    from W+1 before the tile's first pixel on, 64 bytes (one channel chunk) each, and tap
//    (r, s) of tile pixel i is patch row i + r W + s.  Taps outside the image (first / last
//    row or column; the neighbouring image) are not in that picture: a lane whose pixel has
//    such a tap reads a row of zeros instead (a 9-bit mask per pixel, made once).
//  * The patch of chunk c+1 is requested (global -> LDS, no registers) while the nine steps
//    of chunk c run, into the other of two patch buffers.  The filters go through the same
//    ring as in the generic kernel, one 64-byte slab per output channel and step.
//  * Patch rows are 64 bytes; the 16-byte slot of chunk k in row rho is k ^ ((rho >> 2) & 3),
//    so the 16 consecutive rows a quarter-wave reads at one tap fall into 16 distinct bank
//    groups whatever the tap's row offset is.
//
// Steps are ordered chunk-major (chunk c, taps 0..8), nine per loop pass with the ring position
// and every wait count known at compile time (STAGES = 3 divides 9).
#pragma once
#include "q8_conv_ring_kernel.h"

namespace q8 {
namespace {

// PL = patch loads per wavefront and chunk (a wavefront-wide load fills 16 rows): the patch
// buffer holds PL * NW * 16 rows, which must cover BP + 2W + 2.
//
// KW = 2: the reduction of a tile is split over two groups of WP * WC wavefronts inside the
// workgroup (Eq. x: integer sums regroup freely).  Group g runs the loop above on the channel
// chunks g, g + 2, ... with a filter ring and patch buffers of its own; both groups meet at
// every step's barrier, so a workgroup passes half as many barriers per tile -- what counts
// when a layer has few tiles per CU and a tile's time is its chain of steps.  At the end group
// 1 hands its accumulators to group 0 through LDS and group 0 runs the layer's tail.
//
// ST = ring depth of the filter slabs, 3 or 9 (the stage of a step is known at compile time:
// ST divides the nine taps).  Nine keeps eight slabs in flight per group: for the late layers,
// whose filters come from HBM in every pass and whose tiles are chains of 36 ... 72 steps.
template <int WP, int WC, int TP, int TC, int PL, int KW = 1, int ST = 3>
struct HaloShape {
  static constexpr int NW = WP * WC;                       // wavefronts per group
  static constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
  static constexpr int STAGES = ST;
  static constexpr int A_BYTES = BC * 64;                  // one filter slab
  static constexpr int PATCH_ROWS = PL * NW * 16;
  static constexpr int PATCH_BYTES = PATCH_ROWS * 64;
  static constexpr int GROUP_BYTES = STAGES * A_BYTES + 2 * PATCH_BYTES;   // ring + patches
  static constexpr int ZERO_OFF = KW * GROUP_BYTES;        // a row of zeros
  static constexpr int XCH_OFF = ZERO_OFF + 1024;          // KW = 2: accumulators of group 1
  static constexpr int XCH_BYTES = KW > 1 ? NW * TC * TP * 4096 : 0;
  static constexpr int LDS_BYTES = KW > 1 ? XCH_OFF + XCH_BYTES : ZERO_OFF + 64;
  static constexpr int max_w() { return (PATCH_ROWS - BP - 2) / 2; }
};

template <int WP, int WC, int TP, int TC, int PL, int KW = 1, int ST = 3>
__device__ __forceinline__ void conv_tile_halo3(const ConvParams& p, const int ptile,
                                                const int ctile, int8_t* const lds) {
#if defined(__HIP_DEVICE_COMPILE__)
  using Sh = HaloShape<WP, WC, TP, TC, PL, KW, ST>;
  constexpr int NW = Sh::NW, BP = Sh::BP, BC = Sh::BC, STAGES = Sh::STAGES;
  static_assert(STAGES == 3 || STAGES == 9, "the ring depth divides the nine taps");
  constexpr int A_BYTES = Sh::A_BYTES, PATCH_BYTES = Sh::PATCH_BYTES;
  constexpr int A_LOADS = BC / 16 / NW;          // filter loads per wavefront and step
  static_assert(NW == 4 || NW == 8, "four or eight wavefronts per block");
  static_assert((BC / 16) % NW == 0, "every wave issues the same filter loads");
  static_assert((STAGES - 2) * A_LOADS + PL < 64, "vmcnt is 6 bits");

  const int pix0 = ptile * BP;
  const int ch0 = ctile * BC;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kgroup = KW > 1 ? wave_all / NW : 0;           // which share of the reduction
  const int wave = KW > 1 ? wave_all % NW : wave_all;      // wavefront inside its group
  const int wave_p = wave % WP;
  const int wave_c = wave / WP;
  const int W = p.W;
  const int n_chunks = (p.C >> 6) / KW;                    // chunks of this group
  const int gbase = kgroup * Sh::GROUP_BYTES;              // the group's ring and patches

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, p.x_bytes, 0x00020000);

  int8_t* const ring = lds + gbase;
  int8_t* const patch = ring + STAGES * A_BYTES;
  // the row of zeros that masked taps read
  if (tid < 16) reinterpret_cast<int*>(lds + Sh::ZERO_OFF)[tid] = 0;

  // ---- filter loader: as in the generic kernel (lane l of a load fills row l / 4, slot l % 4)
  const int lrow = lane >> 2;
  const int lchunk_a = (lane & 3) ^ swz<4>(wave * 16 + lrow, 0);
  int a_off[A_LOADS];
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int row = (wave + NW * j) * 16 + lrow;
    const int ch = ch0 + (row & ~31) + row_to_channel(row & 31);
    a_off[j] = ch < p.K ? ch * p.red_len + lchunk_a * 16 : kOobOffset;
  }
  // ---- patch loader: load j of this wave fills patch rows (wave + NW j) 16 + lrow; row rho is
  // input pixel pix0 - W - 1 + rho of the whole tensor (zeros before its start / past its end)
  int b_off[PL];
  const int n_in = p.N * p.H * W;
#pragma unroll
  for (int j = 0; j < PL; ++j) {
    const int rho = (wave + NW * j) * 16 + lrow;
    const int q = pix0 - W - 1 + rho;
    const int slot = (lane & 3) ^ ((rho >> 2) & 3);
    b_off[j] = (q >= 0 && q < n_in) ? q * p.in_cs + slot * 16 : kOobOffset;
  }

  // ---- the pixels this lane feeds to the MFMA: patch row of tap (0,0), taps inside the image
  const int frag_row = lane & 31, frag_half = lane >> 5;
  int prow[TP];
  unsigned pmask[TP];
#pragma unroll
  for (int j = 0; j < TP; ++j) {
    const int i = (wave_p * TP + j) * 32 + frag_row;
    prow[j] = i;
    const int pix = pix0 + i;
    unsigned mask = 0;
    if (pix < p.M) {
      const int n = fast_div(pix, p.div_img_m, p.div_img_s);
      const int rem = pix - n * (p.H * W);
      const int h = fast_div(rem, p.div_row_m, p.div_row_s);
      const int w = rem - h * W;
      const unsigned cols = (w > 0 ? 1u : 0u) | 2u | (w + 1 < W ? 4u : 0u);
      if (h > 0) mask |= cols;
      mask |= cols << 3;
      if (h + 1 < p.H) mask |= cols << 6;
    }
    pmask[j] = mask;
  }

  // ---- accumulators start at the bias
  v16i acc[TC][TP];
#pragma unroll
  for (int i = 0; i < TC; ++i) {
    int b[16];
    load_bias16(p, ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5), b);
#pragma unroll
    for (int j = 0; j < TP; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = kgroup == 0 ? b[e] : 0;
  }
  int res_w[TC][TP][4];
  auto fetch_residual = [&]() {
    if (KW > 1 && kgroup != 0) return;
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
        load_res16(p, pix0 + (wave_p * TP + j) * 32 + (lane & 31),
                   ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5), res_w[i][j]);
  };

  const int p_C = p.C;
  // `chunk` counts the group's own chunks: its c-th chunk is channel chunk c * KW + kgroup
  auto issue_patch = [&](int chunk) {        // the patch of `chunk` into buffer chunk & 1
    int8_t* buf = patch + (chunk & 1) * PATCH_BYTES;
#pragma unroll
    for (int j = 0; j < PL; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc_x, (__attribute__((address_space(3))) void*)(buf + (wave + NW * j) * 1024), 16,
          b_off[j], (chunk * KW + kgroup) * 64, 0, 0);
  };
  auto issue_filters = [&](int chunk, int tap, int stage) {     // the slab of one step
    int8_t* buf = ring + stage * A_BYTES;
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc_w, (__attribute__((address_space(3))) void*)(buf + (wave + NW * j) * 1024), 16,
          a_off[j], tap * p_C + (chunk * KW + kgroup) * 64, 0, 0);
  };

  // ---- operand fragments: filters as in the generic kernel, activations from the patch
  int a_foff[2][TC];
  const int foff0 = frag_row * 64 + swz<4>(frag_row, frag_half) * 16;
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      a_foff[h][i] = (foff0 ^ (h * 32)) + (wave_c * TC + i) * 32 * 64;
      asm volatile("" : "+v"(a_foff[h][i]));
    }
  v4i af[2][TC], bf[2][TP];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
#pragma unroll
    for (int i = 0; i < TC; ++i) af[b][i] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < TP; ++j) bf[b][j] = v4i{0, 0, 0, 0};
  }
  // fragments of sub-step h (reduction bytes 32h .. 32h+31 of the step) of (chunk, tap)
  auto load_frags = [&](int chunk, auto tap_c, int stage, int h) {
    constexpr int TAP = decltype(tap_c)::value;
    const int8_t* a_base = ring + stage * A_BYTES;
#pragma unroll
    for (int i = 0; i < TC; ++i)
      af[h & 1][i] = *reinterpret_cast<const v4i*>(a_base + a_foff[h][i]);
    const int delta = (TAP / 3) * W + (TAP % 3);
    const int pbase = gbase + STAGES * A_BYTES + (chunk & 1) * PATCH_BYTES;
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      const int rho = prow[j] + delta;
      const int slot = (2 * h + frag_half) ^ ((rho >> 2) & 3);
      int addr = pbase + rho * 64 + slot * 16;
      addr = ((pmask[j] >> TAP) & 1u) ? addr : Sh::ZERO_OFF;
      bf[h & 1][j] = *reinterpret_cast<const v4i*>(lds + addr);
    }
  };
  // A wave with a single 32 x 32 tile would feed every MFMA the result of the one before it
  // and wait out its full latency each time: such builds sum the odd 32-byte sub-steps in a
  // second accumulator (integer sums: any grouping gives the same bits) and add it at the end.
  constexpr bool TWO_SUMS = TC * TP == 1;
  v16i acc_odd[1];
  if constexpr (TWO_SUMS) {
#pragma unroll
    for (int e = 0; e < 16; ++e) acc_odd[0][e] = 0;
  }
  auto mma = [&](int h) {
    if constexpr (TWO_SUMS) {
      if (h & 1)
        acc_odd[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[1][0], bf[1][0], acc_odd[0], 0, 0, 0);
      else
        acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[0][0], bf[0][0], acc[0][0], 0, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[h & 1][i], bf[h & 1][j], acc[i][j],
                                                            0, 0, 0);
    }
  };
  auto fold_sums = [&]() {
    if constexpr (TWO_SUMS) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[0][0][e] += acc_odd[0][e];
    }
  };

  using std::integral_constant;
  // One reduction step: tap TAP of `chunk`, ring buffer TAP % 3.  AHEAD = loads this wave
  // issued after the step's own filter slab was requested and that may still be in flight.
  // ISSUE: request the slab of the step two ahead; PATCH: request the next chunk's patch
  // (first step of a chunk, before the slab); LAST: the final step fetches the residual.
  auto step = [&](int chunk, auto tap_c, auto ahead_c, auto issue_c, auto patch_c, auto last_c) {
    constexpr int TAP = decltype(tap_c)::value;
    constexpr int STAGE = TAP % STAGES;
    wait_vmcnt<decltype(ahead_c)::value>();
    __builtin_amdgcn_s_waitcnt(0xc07f);      // this wave's LDS reads have returned
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    load_frags(chunk, tap_c, STAGE, 0);
    if constexpr (decltype(patch_c)::value) issue_patch(chunk + 1);
    if constexpr (decltype(issue_c)::value) {
      // step + STAGES - 1: a later tap of this chunk, or an early one of the next
      constexpr int T2 = (TAP + STAGES - 1) % 9;
      issue_filters(TAP + STAGES - 1 >= 9 ? chunk + 1 : chunk, T2, T2 % STAGES);
    }
    if constexpr (decltype(last_c)::value) fetch_residual();
    mma(1);                                  // second half of the previous step
    load_frags(chunk, tap_c, STAGE, 1);
    mma(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr integral_constant<bool, true> yes{};
  constexpr integral_constant<bool, false> no{};
#define Q8_TAP(T) integral_constant<int, (T)>{}
#define Q8_AHEAD(N) integral_constant<int, (N)>{}

  // prologue: patch of chunk 0, slabs of the first STAGES - 1 steps (of the first chunk, or
  // with a deep ring and one chunk... a chunk has nine steps, so always of the first chunk)
  issue_patch(0);
#pragma unroll
  for (int t = 0; t < STAGES - 1; ++t) issue_filters(0, t, t);
  __builtin_amdgcn_s_waitcnt(0xc07f);
  // Loads this wave issued after the slab of (chunk, tap) and that may still be in flight
  // when that step starts.  Every chunk but the last: each step requests the slab STAGES - 1
  // steps ahead, so STAGES - 2 slabs are younger; the first step also requests the next
  // chunk's patch, in front of its slab: those PL loads are younger than the slabs of taps
  // 1 .. STAGES - 2.  Last chunk: nothing beyond its ninth slab is requested.
  int chunk = 0;
#define Q8_MID(T) step(chunk, Q8_TAP(T), \
    Q8_AHEAD((STAGES - 2) * A_LOADS + (((T) >= 1 && (T) <= STAGES - 2) ? PL : 0)), yes, \
    integral_constant<bool, (T) == 0>{}, no)
#define Q8_END(T) step(chunk, Q8_TAP(T), \
    Q8_AHEAD((((T) + STAGES - 2 < 8 ? (T) + STAGES - 2 : 8) - (T)) * A_LOADS), \
    integral_constant<bool, ((T) + STAGES - 1 <= 8)>{}, no, integral_constant<bool, (T) == 8>{})
  for (; chunk + 1 < n_chunks; ++chunk) {
    Q8_MID(0); Q8_MID(1); Q8_MID(2); Q8_MID(3); Q8_MID(4); Q8_MID(5); Q8_MID(6); Q8_MID(7); Q8_MID(8);
  }
  Q8_END(0); Q8_END(1); Q8_END(2); Q8_END(3); Q8_END(4); Q8_END(5); Q8_END(6); Q8_END(7); Q8_END(8);
#undef Q8_MID
#undef Q8_END
  mma(1);
  fold_sums();
#undef Q8_TAP
#undef Q8_AHEAD

  if constexpr (KW > 1) {
    // group 1's accumulators through LDS to group 0 (lane-major 16-byte cells: no conflicts)
    int8_t* const xch = lds + Sh::XCH_OFF + wave * (TC * TP * 4096);
    if (kgroup != 0) {
#pragma unroll
      for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            *reinterpret_cast<v4i*>(xch + (((i * TP + j) * 4 + q) * 64 + lane) * 16) =
                v4i{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2],
                    acc[i][j][4 * q + 3]};
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (kgroup != 0) return;
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const v4i o = *reinterpret_cast<const v4i*>(xch + (((i * TP + j) * 4 + q) * 64 + lane) * 16);
#pragma unroll
          for (int k = 0; k < 4; ++k) acc[i][j][4 * q + k] += o[k];
        }
  }

  finish_tile<TP, TC, 0>(p, acc, res_w, pix0, ch0, BP, BC, wave_p, wave_c, lane);
#endif  // __HIP_DEVICE_COMPILE__
}

template <int WP, int WC, int TP, int TC, int PL, int KW = 1, int ST = 3>
__global__ __launch_bounds__(WP * WC * KW * 64) void conv_i8_halo3_kernel(const ConvParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  const int nblk = p.n_ptiles * p.n_ctiles;
  int bid = blockIdx.x;
  {
    const int xcd = bid % kNumXcd, idx = bid / kNumXcd;
    const int base = nblk / kNumXcd, rem = nblk % kNumXcd;
    bid = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
#ifdef Q8_TRACE
  const unsigned long long q8_t0 = __builtin_amdgcn_s_memrealtime();
#endif
  const int ptile = p.ptile_fastest ? bid % p.n_ptiles : bid / p.n_ctiles;
  const int ctile = p.ptile_fastest ? bid / p.n_ptiles : bid % p.n_ctiles;
  conv_tile_halo3<WP, WC, TP, TC, PL, KW, ST>(p, ptile, ctile, lds);
#ifdef Q8_TRACE
  q8_trace_record(p, q8_t0);
#endif
#endif
}

// Whether the 3x3 family takes this layer with this shape (else the generic kernel does).
template <int WP, int WC, int TP, int TC, int PL, int KW = 1>
bool halo3_applicable(const ConvParams& p) {
  return (p.C / 64) % KW == 0 && p.R == 3 && p.S == 3 && p.stride_h == 1 && p.stride_w == 1 && p.dil_h == 1 &&
         p.dil_w == 1 && p.pad_h == 1 && p.pad_w == 1 && p.C % 64 == 0 && p.S4 == 0 &&
         p.W <= HaloShape<WP, WC, TP, TC, PL>::max_w() && !p.in_u8 && !p.out_u8 && !p.res_u8 &&
         !p.m_vec && !p.w2;
}

template <int WP, int WC, int TP, int TC, int PL, int KW = 1, int ST = 3>
int launch_halo3(ConvParams& p, hipStream_t stream) {
  using Sh = HaloShape<WP, WC, TP, TC, PL, KW, ST>;
  p.n_ptiles = (p.M + Sh::BP - 1) / Sh::BP;
  p.n_ctiles = (p.K + Sh::BC - 1) / Sh::BC;
  const long nblk = (long)p.n_ptiles * p.n_ctiles;
  if (nblk > 0x7fffffffL) return Q8_EUNSUPPORTED;
  auto kernel = conv_i8_halo3_kernel<WP, WC, TP, TC, PL, KW, ST>;
  if constexpr (Sh::LDS_BYTES > 65536) {
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
        Sh::LDS_BYTES);
    if (attr != hipSuccess) return Q8_EHIP;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)nblk), dim3(Sh::NW * KW * 64), Sh::LDS_BYTES, stream, p);
  return q8_launch_status();
}

}  // namespace
}  // namespace q8
