// The image-row tile family of the int8 convolution (Eq. x / Eq. A' of arxiv 1805.08691): the
// first layer of a network -- an R x S filter (S <= 8) with a stride over a 4-channel image that
// carries its own padding as a zero frame, K <= 64 output channels, output rows of at most 128
// pixels (ResNet-50's 7x7 / 2 on 224 x 224).
//
// One filter row over eight taps x four channels is 32 bytes: exactly the reduction depth of
// one 32 x 32 x 32 MFMA.  So no im2col is needed at all: the 32 bytes an output pixel reads of
// input row r start at byte 4 * stride_w * pixel of that row, and the rows of the image, as
// they lie in memory, ARE the activation operand.  A workgroup
//  * keeps all filters in LDS (K rows of R x 32 bytes, 272-byte pitch so that 16 lanes on 16
//    consecutive rows hit 16 distinct bank groups),
//  * walks down a strip of output rows of one image with a ring of 16 input rows in LDS:
//    each new output row needs only stride_h new input rows, which are requested
//    (global -> LDS, one wave-wide load per row) while the current row is computed,
//  * computes one output row per pass: wave w owns pixels 32 w .. 32 w + 31 and all 64
//    channels, R x 2 MFMAs, operands straight from LDS (activations as two 8-byte reads),
//  * writes the row's codes through a row-ordered staging tile: an output row is one
//    contiguous run of Wo x K bytes in NHWC.
// The generic kernel spends ~450 vector instructions per wave on this layer's addressing;
// here the addressing of a whole row is a handful of scalar operations.
#pragma once
#include "q8_conv_ring_kernel.h"

namespace q8 {
namespace {

struct StemShape {
  static constexpr int NW = 4, BP = 128, BC = 64;
  static constexpr int FILT_PITCH = 272;                         // bytes per filter row in LDS
  static constexpr int FILT_BYTES = BC * FILT_PITCH;             // 17 x 1 KB
  static constexpr int SLOTS_IN = 16, ROW_BYTES = 1024;          // ring of input rows
  static constexpr int RING_BYTES = SLOTS_IN * ROW_BYTES + 1024; // + slack behind the last row
  static constexpr int S_BYTES = BP * BC;
  static constexpr int LDS_BYTES = FILT_BYTES + RING_BYTES + S_BYTES;
};

// p.n_ptiles = strips per image, p.n_ctiles = output rows per strip (set by launch_stem).
__global__ __launch_bounds__(256) void conv_i8_stem_kernel(const ConvParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  using Sh = StemShape;
  constexpr int NW = Sh::NW, BP = Sh::BP, BC = Sh::BC, SLOTS = BC / 16;
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int8_t* const filt = lds;
  int8_t* const ring = lds + Sh::FILT_BYTES;
  int8_t* const stage = lds + Sh::FILT_BYTES + Sh::RING_BYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int R = p.R, sh = p.stride_h;
  const int strips = p.n_ptiles, rows_per_strip = p.n_ctiles;
  const int n = blockIdx.x / strips;
  const int ho_first = (blockIdx.x - n * strips) * rows_per_strip;
  const int ho_end = min(ho_first + rows_per_strip, p.Ho);

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, p.x_bytes, 0x00020000);

  // ---- filters, once: LDS row rho (272 bytes: the R * 32 filter bytes, then padding) holds
  // channel (rho & ~31) + row_to_channel(rho & 31); 16-byte cell number i * 64 + lane of load i
  {
    const int cells = p.red_len >> 4;                    // 16-byte cells of one filter
#pragma unroll
    for (int j = 0; j < 5; ++j) {
      const int i = wave + NW * j;                       // loads 0 .. 16 cover 64 rows x 17 cells
      if (i < 17) {
        const int cell = i * 64 + lane;
        const int rho = cell / 17, k = cell - rho * 17;
        const int ch = (rho & ~31) + row_to_channel(rho & 31);
        const int off = (k < cells && ch < p.K) ? ch * p.red_len + k * 16 : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_w, (__attribute__((address_space(3))) void*)(filt + i * 1024), 16, off, 0, 0, 0);
      }
    }
  }
  // ---- input rows: row hi of image n goes to ring slot hi % 16, requested by wave hi % 4 as
  // one wave-wide load of 1 KB (the bytes behind the row's end belong to the next row, or read
  // as zeros past the tensor: they only meet pixels that are not stored)
  const int row_bytes = p.W * 4;
  const int img_off = n * p.H * row_bytes;
  auto issue_row = [&](int hi) {
    if ((hi & 3) == wave && hi < p.H)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc_x, (__attribute__((address_space(3))) void*)(ring + (hi & 15) * Sh::ROW_BYTES), 16,
          img_off + hi * row_bytes + lane * 16, 0, 0, 0);
  };
  for (int r = 0; r < R; ++r) issue_row(ho_first * sh + r);

  // ---- fragments.  Filters: LDS row tc * 32 + (lane & 31), bytes r * 32 + 16 * (lane >> 5).
  // Activations: pixel 32 wave + (lane & 31) of the output row, same half.
  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int a_off = frag_row * Sh::FILT_PITCH + 16 * frag_half;
  const int b_off = (wave * 32 + frag_row) * (p.stride_w * 4) + 16 * frag_half;
  int bias_v[2][16];
#pragma unroll
  for (int tc = 0; tc < 2; ++tc) load_bias16(p, tc * 32 + 16 * frag_half, bias_v[tc]);
  const float no_scales[16] = {};

  wait_vmcnt<0>();
  __syncthreads();
  for (int ho = ho_first; ho < ho_end; ++ho) {
    // the rows the NEXT output row adds (their slots were last read eight or more rows ago)
    if (ho + 1 < ho_end)
      for (int r = R - sh; r < R; ++r) issue_row((ho + 1) * sh + r);

    v16i acc[2];
#pragma unroll
    for (int tc = 0; tc < 2; ++tc)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[tc][e] = bias_v[tc][e];
    // four filter rows at a time: their fragments are requested together (rows beyond R read
    // valid LDS and are not used)
#pragma unroll
    for (int r0 = 0; r0 < 8; r0 += 4) {
      if (r0 < R) {
        v4i af[4][2], bf[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int8_t* const row = ring + ((ho * sh + r0 + r) & 15) * Sh::ROW_BYTES + b_off;
          const long long b0 = *reinterpret_cast<const long long*>(row);
          const long long b1 = *reinterpret_cast<const long long*>(row + 8);
          bf[r] = v4i{(int)b0, (int)(b0 >> 32), (int)b1, (int)(b1 >> 32)};
#pragma unroll
          for (int tc = 0; tc < 2; ++tc)
            af[r][tc] = *reinterpret_cast<const v4i*>(filt + tc * 32 * Sh::FILT_PITCH + a_off +
                                                      (r0 + r) * 32);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (r0 + r < R) {
#pragma unroll
            for (int tc = 0; tc < 2; ++tc)
              acc[tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[r][tc], bf[r], acc[tc], 0, 0, 0);
          }
      }
    }

    // ---- epilogue through the staging tile
    {
      const int row = wave * 32 + frag_row;
#pragma unroll
      for (int tc = 0; tc < 2; ++tc) {
        const int slot = tc * 2 + frag_half;
        int v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = acc[tc][e];
        const int rw[4] = {0, 0, 0, 0};
        *reinterpret_cast<v4i*>(stage + row * BC + ((slot ^ swz_out<SLOTS>(row)) << 4)) =
            codes16_fast<false>(p, v, rw, no_scales);
      }
    }
    // the rows requested above have landed (so have the stores of the row before, long ago)
    wait_vmcnt<0>();
    __syncthreads();
    {
      int8_t* const y0 = p.y + ((size_t)(n * p.Ho + ho) * p.Wo) * p.out_cs + p.out_off;
#pragma unroll
      for (int c = tid; c < BP * SLOTS; c += NW * 64) {      // two stores per lane
        const int row = c / SLOTS, g = c % SLOTS;
        if (row < p.Wo && g * 16 < p.K)
          *reinterpret_cast<v4i*>(y0 + (size_t)row * p.out_cs + g * 16) =
              *reinterpret_cast<const v4i*>(stage + row * BC + ((g ^ swz_out<SLOTS>(row)) << 4));
      }
    }
    // every wave has read the staging tile (its stores took the data) before the next row's
    // codes are written into it; the stores themselves stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
  }
  wait_vmcnt<0>();
#endif
}

inline bool stem_applicable(const ConvParams& p) {
  return p.S4 == 2 && p.S == 1 && p.C == 32 && p.in_cs == 4 && p.R <= 8 && p.K <= 64 &&
         (p.K & 15) == 0 && p.Wo <= 128 && p.W <= 240 && p.stride_h >= 1 && p.stride_h <= 4 && p.stride_w <= 2 &&
         p.R + p.stride_h <= 12 && p.pad_h == 0 && p.pad_w == 0 && p.vec16 && !p.res &&
         !p.acc_dump && !p.y_f32 && !p.in_u8 && !p.out_u8 && !p.res_u8 && !p.m_vec && !p.w2 &&
         !p.tap_sums && (long)p.N * p.H * p.W * 4 < 0x7fffffffL;
}

inline int launch_stem(ConvParams& p, hipStream_t stream) {
  using Sh = StemShape;
  auto kernel = conv_i8_stem_kernel;
  static const hipError_t attr = hipFuncSetAttribute(
      reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
      Sh::LDS_BYTES);
  if (attr != hipSuccess) return Q8_EHIP;
  static const int resident = [&]() {
    int per_cu = 0, dev = 0, cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      cus = prop.multiProcessorCount;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kernel),
                                                     256, Sh::LDS_BYTES) != hipSuccess || per_cu < 1)
      per_cu = 1;
    return per_cu * cus;
  }();
  // strips per image: about as many workgroups as stay resident, at least four rows each
  int strips = (resident + p.N - 1) / p.N;
  if (strips > (p.Ho + 3) / 4) strips = (p.Ho + 3) / 4;
  if (strips < 1) strips = 1;
  const int rows_per_strip = (p.Ho + strips - 1) / strips;
  strips = (p.Ho + rows_per_strip - 1) / rows_per_strip;
  p.n_ptiles = strips;
  p.n_ctiles = rows_per_strip;
  const long grid = (long)p.N * strips;
  if (grid > 0x7fffffffL) return Q8_EUNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), Sh::LDS_BYTES, stream, p);
  return q8_launch_status();
}

}  // namespace
}  // namespace q8
