// The persistent 3x3 tile family of the int8 convolution (Eq. x / Eq. A' of arxiv 1805.08691):
// 3x3, stride 1, padding 1, C = 64 input channels, K <= 64 output channels -- the middle layer
// of a bottleneck block on a large map, which moves far more bytes than it multiplies.
//
// It joins the two ideas of its neighbours: like the pointwise family, a workgroup is
// persistent -- ALL filters of the layer (nine taps x 64 channels x 64 bytes = 36 KB) stay in
// LDS for the whole launch, the workgroup walks over pixel tiles, and the next tile's
// activations are requested (global -> LDS) before the current tile is computed; like the 3x3
// family, a tile's activations are a patch (the tile's 128 pixels plus one map row and one
// pixel on either side) that the nine taps read at nine row offsets, a tap outside the image
// reading a row of zeros.  Between two tiles there is no barrier-locked reduction loop at all:
// the eighteen half steps of a tile read only LDS, so the compiler schedules them freely.
// Codes leave through a row-ordered staging tile (whole 64-byte rows per wave-wide store).
#pragma once
#include "q8_conv_ring_kernel.h"

namespace q8 {
namespace {

template <int PL>
struct P3Shape {
  static constexpr int NW = 4, WP = 2, WC = 2, TP = 2;
  static constexpr int BP = WP * TP * 32, BC = 64;              // 128 pixels x 64 channels
  static constexpr int A_BYTES = 9 * BC * 64;                    // every filter of the layer
  static constexpr int PATCH_ROWS = PL * NW * 16;                // rows NW * PL loads fill
  static constexpr int PATCH_BYTES = PATCH_ROWS * 64;
  static constexpr int S_BYTES = BP * BC;                        // staging: codes out
  static constexpr int ZERO_OFF = A_BYTES + 2 * PATCH_BYTES + S_BYTES;   // a row of zeros
  static constexpr int LDS_BYTES = ZERO_OFF + 64;
  // the patch of a tile: BP pixels, W + 1 rows in front, W + 1 behind
  static constexpr int max_w() { return (PATCH_ROWS - BP - 2) / 2; }
};

template <int PL>
__global__ __launch_bounds__(256) void conv_i8_p3_kernel(const ConvParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  using Sh = P3Shape<PL>;
  constexpr int NW = Sh::NW, WP = Sh::WP, TP = Sh::TP, BP = Sh::BP, BC = Sh::BC;
  constexpr int SLOTS = BC / 16;
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int8_t* const lds_a = lds;
  int8_t* const patch = lds + Sh::A_BYTES;
  int8_t* const stage = lds + Sh::A_BYTES + 2 * Sh::PATCH_BYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_p = wave % WP, wave_c = wave / WP;
  const int W = p.W, M = p.M;
  const int n_in = p.N * p.H * W;

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, p.x_bytes, 0x00020000);
  if (tid < 16) reinterpret_cast<int*>(lds + Sh::ZERO_OFF)[tid] = 0;

  // ---- the filters, once: tap t is a slab of 64 rows x 64 bytes; this wave fills rows
  // 16 wave .. 16 wave + 15 of every slab (lane l: row l / 4, slot l % 4)
  const int lrow = lane >> 2;
  {
    const int row = wave * 16 + lrow;
    const int ch = (row & ~31) + row_to_channel(row & 31);
    const int lchunk = (lane & 3) ^ swz<4>(row, 0);
    const int off = ch < p.K ? ch * p.red_len + lchunk * 16 : kOobOffset;
#pragma unroll
    for (int t = 0; t < 9; ++t)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc_w, (__attribute__((address_space(3))) void*)(lds_a + t * (BC * 64) + wave * 1024), 16,
          off, t * 64, 0, 0);
  }

  // ---- patch loader: load j of this wave fills patch rows (wave + NW j) 16 + lrow; row rho is
  // input pixel pix0 - W - 1 + rho of the whole tensor (zeros before its start / past its end)
  auto issue_patch = [&](int ptile, int buf) {
    const int pix0 = ptile * BP;
#pragma unroll
    for (int j = 0; j < PL; ++j) {
      const int rho = (wave + NW * j) * 16 + lrow;
      const int q = pix0 - W - 1 + rho;
      const int slot = (lane & 3) ^ ((rho >> 2) & 3);
      const int off = (q >= 0 && q < n_in) ? q * p.in_cs + slot * 16 : kOobOffset;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc_x,
          (__attribute__((address_space(3))) void*)(patch + buf * Sh::PATCH_BYTES + (wave + NW * j) * 1024),
          16, off, 0, 0, 0);
    }
  };

  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int a_foff0 = frag_row * 64 + swz<4>(frag_row, frag_half) * 16 + wave_c * 32 * 64;
  int bias_v[16];
  load_bias16(p, wave_c * 32 + 16 * (lane >> 5), bias_v);
  const float no_scales[16] = {};

  // patch offsets of this lane's fragments, per tap, half step and pixel tile of the wave: the
  // same in every tile (a tile's patch always starts W + 1 pixels in front of the tile)
  int b_foff[9][2][TP];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < TP; ++j) {
        const int rho = (wave_p * TP + j) * 32 + frag_row + (t / 3) * W + (t % 3);
        b_foff[t][h][j] = rho * 64 + (((2 * h + frag_half) ^ ((rho >> 2) & 3)) << 4);
      }

  // every workgroup is a walker of its own: tiles blockIdx.x, + gridDim.x, ...
  int ptile = blockIdx.x;
  if (ptile < p.n_ptiles) issue_patch(ptile, 0);
  for (int it = 0; ptile < p.n_ptiles; ++it, ptile += gridDim.x) {
    const int buf = it & 1;
    const int next = ptile + gridDim.x;
    const int pix0 = ptile * BP;
    // which taps of this lane's pixels lie inside the image
    unsigned pmask[TP];
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      const int pix = pix0 + (wave_p * TP + j) * 32 + frag_row;
      unsigned mask = 0;
      if (pix < M) {
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
    // the other patch buffer is free: every wave passed the barrier behind the last tile
    if (next < p.n_ptiles) {
      issue_patch(next, buf ^ 1);
      wait_vmcnt<PL>();
    } else {
      wait_vmcnt<0>();
    }
    __syncthreads();                    // filters (first pass) and this tile's patch are in LDS

    v16i acc[TP];
#pragma unroll
    for (int j = 0; j < TP; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][e] = bias_v[e];
    const int pbase = Sh::A_BYTES + buf * Sh::PATCH_BYTES;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const v4i af = *reinterpret_cast<const v4i*>(lds_a + t * (BC * 64) + (a_foff0 ^ (h * 32)));
        v4i bf[TP];
#pragma unroll
        for (int j = 0; j < TP; ++j) {
          const int addr = ((pmask[j] >> t) & 1u) ? pbase + b_foff[t][h][j] : Sh::ZERO_OFF;
          bf[j] = *reinterpret_cast<const v4i*>(lds + addr);
        }
#pragma unroll
        for (int j = 0; j < TP; ++j)
          acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af, bf[j], acc[j], 0, 0, 0);
      }
    }

    // ---- epilogue through the staging tile (free: the copy-out of the tile before ended in
    // front of a barrier)
    {
      const int slot = wave_c * 2 + (lane >> 5);
#pragma unroll
      for (int j = 0; j < TP; ++j) {
        const int row = (wave_p * TP + j) * 32 + (lane & 31);
        int v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = acc[j][e];
        const int rw[4] = {0, 0, 0, 0};
        *reinterpret_cast<v4i*>(stage + row * BC + ((slot ^ swz_out<SLOTS>(row)) << 4)) =
            codes16_fast<false>(p, v, rw, no_scales);
      }
    }
    __syncthreads();
    {
      int8_t* const y0 = p.y + (size_t)pix0 * p.out_cs + p.out_off;
#pragma unroll
      for (int c = tid; c < BP * SLOTS; c += NW * 64) {
        const int row = c / SLOTS, g = c % SLOTS;
        if (pix0 + row < M && g * 16 < p.K)
          *reinterpret_cast<v4i*>(y0 + (size_t)row * p.out_cs + g * 16) =
              *reinterpret_cast<const v4i*>(stage + row * BC + ((g ^ swz_out<SLOTS>(row)) << 4));
      }
    }
    // every wave has read this tile's patch and the staging tile before the next pass
    // requests a patch into this buffer / writes codes into the staging tile
    __syncthreads();
  }
  wait_vmcnt<0>();
#endif
}

template <int PL>
bool p3_applicable(const ConvParams& p) {
  return p.R == 3 && p.S == 3 && p.stride_h == 1 && p.stride_w == 1 && p.dil_h == 1 &&
         p.dil_w == 1 && p.pad_h == 1 && p.pad_w == 1 && p.C == 64 && p.S4 == 0 && p.K <= 64 &&
         (p.K & 15) == 0 && p.W <= P3Shape<PL>::max_w() && p.vec16 && !p.res && !p.acc_dump &&
         !p.y_f32 && !p.y_deq && !p.in_u8 && !p.out_u8 && !p.res_u8 && !p.m_vec && !p.w2 && !p.tap_sums;
}

template <int PL>
int launch_p3(ConvParams& p, hipStream_t stream) {
  using Sh = P3Shape<PL>;
  p.n_ptiles = (p.M + Sh::BP - 1) / Sh::BP;
  p.n_ctiles = 1;
  auto kernel = conv_i8_p3_kernel<PL>;
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
  // as many workgroups as stay resident, every one with the same number of tiles (+- 1)
  const int passes = (p.n_ptiles + resident - 1) / resident;
  const int grid = (p.n_ptiles + passes - 1) / passes;
  hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), Sh::LDS_BYTES, stream, p);
  return q8_launch_status();
}

}  // namespace
}  // namespace q8
