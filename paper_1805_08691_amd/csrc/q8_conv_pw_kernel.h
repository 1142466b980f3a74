// The pointwise (1x1, stride 1, no padding) tile family of the int8 convolution (Eq. x / Eq. A'
// of arxiv 1805.08691) for few input channels (C = 64, 128 or 256): layers that move far more
// bytes than they multiply.
//
// With one workgroup per output tile such a layer is bound by the life cycle of a workgroup,
// not by bandwidth: launch, argument fetch, ONE memory latency for its operands, a moment of
// matrix work, the drain of its stores -- about 4.5 us for 28 KB, and only four or five
// workgroups fit a compute unit.  Here a workgroup is persistent and pipelined instead:
//  * it keeps the filters of ITS channel tile in LDS for the whole launch and walks over pixel
//    tiles;
//  * the activations (and the residual tile of the fused sum) of the NEXT pixel tile are
//    requested, global -> LDS, before the current tile is computed, so a compute unit always
//    has loads in flight while it multiplies, requantises and stores;
//  * residual and output pass through an LDS staging tile in row order.  A lane of the MFMA
//    layout owns 16 consecutive channels of one pixel, so a wave-wide access straight from
//    registers would touch 32 pixel rows with 32 bytes in each (a pure copy with that pattern
//    moves 3.9 TB/s where a linear one moves 5.9); through the staging tile every wave-wide
//    access is 1 KB of whole rows.
// The workgroups that share a pixel tile (one per channel tile) run on the same XCD, so the
// activations are fetched into one L2 only.
#pragma once
#include "q8_conv_ring_kernel.h"

namespace q8 {
namespace {

template <int TC, int KS>
struct PwShape {
  static constexpr int NW = 4, WP = 2, WC = 2, TP = 2;
  static constexpr int BP = WP * TP * 32, BC = WC * TC * 32;   // 128 pixels x 64 / 128 channels
  static constexpr int A_BYTES = KS * BC * 64;                  // the channel tile's filters
  static constexpr int B_BYTES = KS * BP * 64;                  // one pixel tile's activations
  static constexpr int S_BYTES = BP * BC;                       // staging: residual in, codes out
  static constexpr int LDS_BYTES = A_BYTES + 2 * B_BYTES + 2 * S_BYTES;
};

template <int TC, int KS>
__global__ __launch_bounds__(256) void conv_i8_pw_kernel(const ConvParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  using Sh = PwShape<TC, KS>;
  constexpr int NW = Sh::NW, WP = Sh::WP, TP = Sh::TP, BP = Sh::BP, BC = Sh::BC;
  constexpr int SLOTS = BC / 16;
  constexpr int A_LOADS = KS * BC / 16 / NW, B_LOADS = KS * BP / 16 / NW, R_LOADS = BP * BC / 1024 / NW;
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int8_t* const lds_a = lds;
  int8_t* const lds_b = lds + Sh::A_BYTES;
  int8_t* const lds_s = lds + Sh::A_BYTES + 2 * Sh::B_BYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_p = wave % WP, wave_c = wave / WP;

  // ---- which tiles: the n_ctiles workgroups of a group share pixel tiles and sit on one XCD
  const int n_ct = p.n_ctiles;
  const int xcd = blockIdx.x % kNumXcd, wl = blockIdx.x / kNumXcd;
  const int ctile = wl % n_ct;
  const int n_groups = gridDim.x / n_ct;                 // gridDim.x is a multiple of 8 * n_ct
  const int group = (wl / n_ct) * kNumXcd + xcd;
  const int ch0 = ctile * BC;

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(p.res ? p.res : p.x), 0, p.res ? p.res_bytes : 0, 0x00020000);
  const bool has_res = p.res != nullptr;

  // ---- loaders.  A wave-wide load fills 16 rows of 64 bytes; lane l: row l / 4, slot l % 4,
  // which holds chunk (l % 4) ^ swz(row) of the row's 64-byte reduction step.
  const int lrow = lane >> 2;
  // filters, once: load j covers step j / (BC/16/NW)..., rows (wave + NW jj) 16 + lrow of the step
  {
    const int lchunk = (lane & 3) ^ swz<4>(wave * 16 + lrow, 0);
#pragma unroll
    for (int j = 0; j < A_LOADS; ++j) {
      const int step = j / (BC / 16 / NW), jj = j % (BC / 16 / NW);
      const int row = (wave + NW * jj) * 16 + lrow;
      const int ch = ch0 + (row & ~31) + row_to_channel(row & 31);
      const int off = ch < p.K ? ch * p.red_len + step * 64 + lchunk * 16 : kOobOffset;
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc_w,
          (__attribute__((address_space(3))) void*)(lds_a + step * BC * 64 + (wave + NW * jj) * 1024),
          16, off, 0, 0, 0);
    }
  }
  // activations of a pixel tile: per-lane offsets inside the tile (pixel row, chunk), the
  // tile's first pixel goes into the scalar offset
  int b_off[B_LOADS];
  {
    const int lchunk = (lane & 3) ^ swz<4>(wave * 16 + lrow, 0);
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
      const int step = j / (BP / 16 / NW), jj = j % (BP / 16 / NW);
      const int row = (wave + NW * jj) * 16 + lrow;
      b_off[j] = row * p.in_cs + step * 64 + lchunk * 16;
    }
  }
  int r_off[R_LOADS];
#pragma unroll
  for (int j = 0; j < R_LOADS; ++j) {
    const int c = (wave + NW * j) * 64 + lane;
    const int row = c / SLOTS;
    const int ch = ch0 + (((c % SLOTS) ^ swz_out<SLOTS>(row)) << 4);
    r_off[j] = ch < p.K ? row * p.res_cs + p.res_off + ch : kOobOffset;
  }
  const int M = p.M;
  int b_row[BP / 16 / NW], r_row[R_LOADS];       // the tile rows behind those offsets
#pragma unroll
  for (int jj = 0; jj < BP / 16 / NW; ++jj) b_row[jj] = (wave + NW * jj) * 16 + lrow;
#pragma unroll
  for (int j = 0; j < R_LOADS; ++j) r_row[j] = ((wave + NW * j) * 64 + lane) / SLOTS;
  auto issue_tile = [&](int ptile, int buf) {
    const int pix0 = ptile * BP;
    // the tile's first pixel goes into the scalar offset; a row beyond the last pixel gets an
    // out-of-range vector offset and reads as zeros
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j) {
      const int step = j / (BP / 16 / NW), jj = j % (BP / 16 / NW);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc_x,
          (__attribute__((address_space(3))) void*)(lds_b + buf * Sh::B_BYTES + step * BP * 64 +
                                                     (wave + NW * jj) * 1024),
          16, pix0 + b_row[jj] < M ? b_off[j] : kOobOffset, pix0 * p.in_cs, 0, 0);
    }
    if (has_res) {
#pragma unroll
      for (int j = 0; j < R_LOADS; ++j)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_r,
            (__attribute__((address_space(3))) void*)(lds_s + buf * Sh::S_BYTES + (wave + NW * j) * 1024),
            16, pix0 + r_row[j] < M ? r_off[j] : kOobOffset, pix0 * p.res_cs, 0, 0);
    }
  };

  // ---- fragments
  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int foff0 = frag_row * 64 + swz<4>(frag_row, frag_half) * 16;
  int bias_v[TC][16];
#pragma unroll
  for (int i = 0; i < TC; ++i) load_bias16(p, ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5), bias_v[i]);

  int ptile = group;
  if (ptile < p.n_ptiles) issue_tile(ptile, 0);
  const float no_scales[16] = {};
  for (int it = 0; ptile < p.n_ptiles; ++it, ptile += n_groups) {
    const int buf = it & 1;
    const int next = ptile + n_groups;
    // the other buffers are free: every wave passed the barrier behind the copy-out that
    // last read them
    if (next < p.n_ptiles) {
      issue_tile(next, buf ^ 1);
      if (has_res) wait_vmcnt<B_LOADS + R_LOADS>(); else wait_vmcnt<B_LOADS>();
    } else {
      wait_vmcnt<0>();
    }
    __syncthreads();                                   // this tile's operands are in LDS
    v16i acc[TC][TP];
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = bias_v[i][e];
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        v4i af[TC], bf[TP];
#pragma unroll
        for (int i = 0; i < TC; ++i)
          af[i] = *reinterpret_cast<const v4i*>(lds_a + s * BC * 64 + (foff0 ^ (h * 32)) +
                                                (wave_c * TC + i) * 32 * 64);
#pragma unroll
        for (int j = 0; j < TP; ++j)
          bf[j] = *reinterpret_cast<const v4i*>(lds_b + buf * Sh::B_BYTES + s * BP * 64 +
                                                (foff0 ^ (h * 32)) + (wave_p * TP + j) * 32 * 64);
#pragma unroll
        for (int i = 0; i < TC; ++i)
#pragma unroll
          for (int j = 0; j < TP; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
      }
    // ---- epilogue through the staging tile
    int8_t* const stage = lds_s + buf * Sh::S_BYTES;
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      const int slot = (wave_c * TC + i) * 2 + (lane >> 5);
#pragma unroll
      for (int j = 0; j < TP; ++j) {
        const int row = (wave_p * TP + j) * 32 + (lane & 31);
        v4i* const cell =
            reinterpret_cast<v4i*>(stage + row * BC + ((slot ^ swz_out<SLOTS>(row)) << 4));
        int v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = acc[i][j][e];
        if (has_res) {
          const v4i r = *cell;
          const int rw[4] = {r[0], r[1], r[2], r[3]};
          *cell = codes16_fast<true>(p, v, rw, no_scales);
        } else {
          const int rw[4] = {0, 0, 0, 0};
          *cell = codes16_fast<false>(p, v, rw, no_scales);
        }
      }
    }
    __syncthreads();
    {
      const int pix0 = ptile * BP;
      int8_t* const y0 = p.y + (size_t)pix0 * p.out_cs + p.out_off + ch0;
#pragma unroll
      for (int c = tid; c < BP * SLOTS; c += NW * 64) {
        const int row = c / SLOTS, g = c % SLOTS;
        if (pix0 + row < M && ch0 + g * 16 < p.K)
          *reinterpret_cast<v4i*>(y0 + (size_t)row * p.out_cs + g * 16) =
              *reinterpret_cast<const v4i*>(stage + row * BC + ((g ^ swz_out<SLOTS>(row)) << 4));
      }
    }
    // the copy-out's LDS reads are done before anyone requests the tile after next into
    // this staging buffer (the barrier at the top of the next iteration comes too late for
    // that request, which the NEXT iteration issues before its barrier)
    __syncthreads();
  }
#endif
}

template <int TC, int KS>
bool pw_applicable(const ConvParams& p) {
  const bool pointwise = p.R == 1 && p.S == 1 && p.stride_h == 1 && p.stride_w == 1 &&
                         p.pad_h == 0 && p.pad_w == 0;
  return pointwise && p.S4 == 0 && p.C == KS * 64 && (p.K & 15) == 0 && p.vec16 && !p.acc_dump &&
         !p.y_f32 && !p.y_deq && !p.in_u8 && !p.out_u8 && !p.res_u8 && !p.m_vec && !p.w2 &&
         (!p.res || (p.res_bytes > 0 && (long)p.M * p.res_cs < 0x7fffffffL)) &&
         (long)p.M * p.in_cs < 0x7fffffffL;
}

template <int TC, int KS>
int launch_pw(ConvParams& p, hipStream_t stream) {
  using Sh = PwShape<TC, KS>;
  p.n_ptiles = (p.M + Sh::BP - 1) / Sh::BP;
  p.n_ctiles = (p.K + Sh::BC - 1) / Sh::BC;
  auto kernel = conv_i8_pw_kernel<TC, KS>;
  if constexpr (Sh::LDS_BYTES > 65536) {
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
        Sh::LDS_BYTES);
    if (attr != hipSuccess) return Q8_EHIP;
  }
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
  // whole groups (one workgroup per channel tile) on every XCD, no more than stay resident and
  // no more than there are pixel tiles
  const int unit = kNumXcd * p.n_ctiles;
  long groups = resident / unit;
  const long need = (p.n_ptiles + kNumXcd - 1) / kNumXcd;
  if (groups > need) groups = need;
  if (groups < 1) groups = 1;
  hipLaunchKernelGGL(kernel, dim3((unsigned)(groups * unit)), dim3(256), Sh::LDS_BYTES, stream, p);
  return q8_launch_status();
}

}  // namespace
}  // namespace q8
