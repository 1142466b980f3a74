// The block-tiled build of the persistent 3x3 family (Eq. x / Eq. A' of arxiv 1805.08691):
// 3x3, stride 1, padding 1, C = 64 input channels, K <= 64 output channels, maps of any width.
//
// The persistent 3x3 kernel (q8_conv_p3_kernel.h) cuts the output into runs of 128 consecutive
// pixels; the activations such a run reads are the run plus a whole map row on either side, so
// on a wide map (a detector's 300 x 300 first block) a tile would stage many times the pixels
// it computes.  Here a tile is a BLOCK of 8 rows x 16 columns of one image and its patch the
// 10 x 18 input pixels around it (1.4 times the tile).  Every patch row stands for one input
// position, so a position outside the image is simply a row of zeros in the patch (its load
// is sent out of the buffer's range): no per-tap masks, no selects -- the nine taps of output
// pixel (ty, tx) read patch rows (ty + r) * 18 + tx + s.  Everything else is the persistent
// kernel: all filters of the layer resident in LDS, workgroups walking over tiles with the
// next tile's patch in flight, eighteen half steps per tile that read only LDS, codes leaving
// through a row-ordered staging tile (an output row of the block is 16 x K contiguous bytes).
#pragma once
#include "q8_conv_ring_kernel.h"

namespace q8 {
namespace {

struct P3bShape {
  static constexpr int NW = 4, WP = 2, WC = 2, TP = 2;
  static constexpr int TH = 8, TW = 16;                          // output block
  static constexpr int PW = TW + 2, PATCH_PIX = (TH + 2) * PW;   // 10 x 18 input positions
  static constexpr int BP = TH * TW, BC = 64;                    // 128 pixels x 64 channels
  static constexpr int A_BYTES = 9 * BC * 64;                    // every filter of the layer
  static constexpr int PL = 3;                                   // patch loads per wave: 192 rows
  static constexpr int PATCH_ROWS = PL * NW * 16;
  static constexpr int PATCH_BYTES = PATCH_ROWS * 64;
  static constexpr int S_BYTES = BP * BC;                        // staging: codes out
  static constexpr int LDS_BYTES = A_BYTES + 2 * PATCH_BYTES + S_BYTES;
  static_assert(PATCH_ROWS >= PATCH_PIX, "the loads cover the patch");
};

// p.n_ptiles = tiles in all (N * tiles_h * tiles_w), p.n_ctiles = tiles_w (set by launch_p3b).
__global__ __launch_bounds__(256) void conv_i8_p3b_kernel(const ConvParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  using Sh = P3bShape;
  constexpr int NW = Sh::NW, WP = Sh::WP, TP = Sh::TP, BP = Sh::BP, BC = Sh::BC;
  constexpr int TH = Sh::TH, TW = Sh::TW, PW = Sh::PW, PL = Sh::PL;
  constexpr int SLOTS = BC / 16;
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int8_t* const lds_a = lds;
  int8_t* const patch = lds + Sh::A_BYTES;
  int8_t* const stage = lds + Sh::A_BYTES + 2 * Sh::PATCH_BYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_p = wave % WP, wave_c = wave / WP;
  const int H = p.H, W = p.W;
  const int tiles_w = p.n_ctiles;
  const int tiles_img = ((H + TH - 1) / TH) * tiles_w;

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_y =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.y, 0, p.M * p.out_cs, 0x00020000);

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

  // ---- patch loader: load j of this wave fills patch rows (wave + NW j) 16 + lrow; patch row
  // rho is input position (h0 - 1 + rho / 18, w0 - 1 + rho % 18) of the tile's image, 16-byte
  // slot (lane & 3) ^ ((rho >> 2) & 3) of its 64 channels
  int pr_y[PL], pr_x[PL], pr_slot[PL];
#pragma unroll
  for (int j = 0; j < PL; ++j) {
    const int rho = (wave + NW * j) * 16 + lrow;
    pr_y[j] = rho < Sh::PATCH_PIX ? rho / PW : -4096;            // beyond the patch: never inside
    pr_x[j] = rho % PW;
    pr_slot[j] = ((lane & 3) ^ ((rho >> 2) & 3)) * 16;
  }
  // tile number -> image and block origin
  auto tile_origin = [&](int tile, int& n, int& h0, int& w0) {
    n = tile / tiles_img;
    const int rem = tile - n * tiles_img;
    const int th = rem / tiles_w;
    h0 = th * TH;
    w0 = (rem - th * tiles_w) * TW;
  };
  auto issue_patch = [&](int tile, int buf) {
    int n, h0, w0;
    tile_origin(tile, n, h0, w0);
#pragma unroll
    for (int j = 0; j < PL; ++j) {
      const int h = h0 - 1 + pr_y[j], w = w0 - 1 + pr_x[j];
      const bool inside = (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W;
      const int off = inside ? ((n * H + h) * W + w) * p.in_cs + pr_slot[j] : kOobOffset;
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
  // same in every tile
  int b_foff[9][2][TP];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int j = 0; j < TP; ++j) {
        const int i = (wave_p * TP + j) * 32 + frag_row;          // pixel of the block
        const int rho = ((i / TW) + t / 3) * PW + (i % TW) + t % 3;
        b_foff[t][h][j] = rho * 64 + (((2 * h + frag_half) ^ ((rho >> 2) & 3)) << 4);
      }

  // every workgroup is a walker of its own: tiles blockIdx.x, + gridDim.x, ...
  int tile = blockIdx.x;
  if (tile < p.n_ptiles) issue_patch(tile, 0);
  for (int it = 0; tile < p.n_ptiles; ++it, tile += gridDim.x) {
    const int buf = it & 1;
    const int next = tile + gridDim.x;
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
    const int8_t* const pbase = patch + buf * Sh::PATCH_BYTES;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const v4i af = *reinterpret_cast<const v4i*>(lds_a + t * (BC * 64) + (a_foff0 ^ (h * 32)));
        v4i bf[TP];
#pragma unroll
        for (int j = 0; j < TP; ++j) bf[j] = *reinterpret_cast<const v4i*>(pbase + b_foff[t][h][j]);
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
      int n, h0, w0;
      tile_origin(tile, n, h0, w0);
#pragma unroll
      for (int k = 0; k < BP * SLOTS / (NW * 64); ++k) {
        const int c = tid + k * NW * 64;
        const int row = c / SLOTS, g = c % SLOTS;             // pixel of the block, channel group
        const int h = h0 + row / TW, w = w0 + row % TW;
        const v4i codes =
            *reinterpret_cast<const v4i*>(stage + row * BC + ((g ^ swz_out<SLOTS>(row)) << 4));
        const int off = (h < H && w < W && g * 16 < p.K)
                            ? ((n * H + h) * W + w) * p.out_cs + p.out_off + g * 16
                            : kOobOffset;
        __builtin_amdgcn_raw_buffer_store_b128(codes, rsrc_y, off, 0, 0);
      }
    }
    // every wave has read this tile's patch and the staging tile before the next pass
    // requests a patch into this buffer / writes codes into the staging tile
    __syncthreads();
  }
  wait_vmcnt<0>();
#endif
}

inline bool p3b_applicable(const ConvParams& p) {
  return p.R == 3 && p.S == 3 && p.stride_h == 1 && p.stride_w == 1 && p.dil_h == 1 &&
         p.dil_w == 1 && p.pad_h == 1 && p.pad_w == 1 && p.C == 64 && p.S4 == 0 && p.K <= 64 &&
         (p.K & 15) == 0 && p.vec16 && !p.res && !p.acc_dump && !p.y_f32 && !p.y_deq && !p.in_u8 &&
         !p.out_u8 && !p.res_u8 && !p.m_vec && !p.w2 && !p.tap_sums &&
         (long)p.M * p.out_cs < 0x7fffffffL;
}

inline int launch_p3b(ConvParams& p, hipStream_t stream) {
  using Sh = P3bShape;
  const long tiles_w = (p.W + Sh::TW - 1) / Sh::TW, tiles_h = (p.H + Sh::TH - 1) / Sh::TH;
  const long tiles = (long)p.N * tiles_h * tiles_w;
  if (tiles > 0x7fffffffL) return Q8_EUNSUPPORTED;
  p.n_ptiles = (int)tiles;
  p.n_ctiles = (int)tiles_w;
  auto kernel = conv_i8_p3b_kernel;
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
