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
//    each new output row needs only stride_h new input rows, which are requested ahead,
//  * computes one output row per pass: wave w owns pixels 32 w .. 32 w + 31 and all 64
//    channels, R x 2 MFMAs, operands straight from LDS (activations as two 8-byte reads),
//  * writes the row's codes through a row-ordered staging tile: an output row is one
//    contiguous run of Wo x K bytes in NHWC.
// Two options turn the layer into the whole head of a network in one launch:
//  F32IN: the input is the real-valued image [N][H][W][C <= 4]; the workgroup applies Eq. Q to
//         the rows it loads and builds the zero frame in LDS -- the int8 image never exists
//         in memory;
//  POOL:  the 3x3 / stride 2 / padding 1 max-pool behind the layer: the maximum over three
//         output rows is kept in registers (on the rounded, clamped fp32 values, whose order
//         is that of the codes), the maximum over three columns is taken on the codes in the
//         staging tile, and only the pooled rows are written.
#pragma once
#include "q8_conv_ring_kernel.h"
#include "q8_quant.h"

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

// Bytewise maximum of signed bytes flipped to unsigned order (x ^ 0x80 per byte), on the
// even and the odd bytes of a word as two pairs of 16-bit lanes.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
struct SplitBytes { u16x2 even, odd; };
__device__ __forceinline__ SplitBytes split_bytes(unsigned w) {
  SplitBytes s;
  s.even = __builtin_bit_cast(u16x2, w & 0x00ff00ffu);
  s.odd = __builtin_bit_cast(u16x2, (w >> 8) & 0x00ff00ffu);
  return s;
}
__device__ __forceinline__ SplitBytes max_bytes(SplitBytes a, SplitBytes b) {
  SplitBytes m;
  m.even = __builtin_elementwise_max(a.even, b.even);
  m.odd = __builtin_elementwise_max(a.odd, b.odd);
  return m;
}
__device__ __forceinline__ unsigned join_bytes(SplitBytes s) {
  return __builtin_bit_cast(unsigned, s.even) | (__builtin_bit_cast(unsigned, s.odd) << 8);
}

// p.n_ptiles = strips per image, p.n_ctiles = output rows (POOL: pooled rows) per strip, set by
// launch_stem.  SH: the vertical stride (the number of image rows a new output row adds).
template <int SH, bool F32IN, bool POOL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void conv_i8_stem_kernel(const ConvParams p, const StemImage im) {
#if defined(__HIP_DEVICE_COMPILE__)
  using Sh = StemShape;
  constexpr int NW = Sh::NW, BP = Sh::BP, BC = Sh::BC, SLOTS = BC / 16;
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int8_t* const filt = lds;
  int8_t* const ring = lds + Sh::FILT_BYTES;
  int8_t* const stage = lds + Sh::FILT_BYTES + Sh::RING_BYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int R = p.R;
  constexpr int sh = SH;
  const int strips = p.n_ptiles, rows_per_strip = p.n_ctiles;
  const int n = blockIdx.x / strips;
  // output rows [ho_first, ho_end) of image n; POOL: those under pooled rows [j_first, j_end)
  const int j_first = (blockIdx.x - n * strips) * rows_per_strip;
  const int j_end = min(j_first + rows_per_strip, POOL ? im.Hp : p.Ho);
  const int ho_first = POOL ? max(2 * j_first - 1, 0) : j_first;
  const int ho_end = POOL ? min(2 * j_end, p.Ho) : j_end;

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, p.x_bytes, 0x00020000);
  const int y_rows = POOL ? p.N * im.Hp * im.Wp : p.M;
  const __amdgpu_buffer_rsrc_t rsrc_y =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.y, 0, y_rows * p.out_cs, 0x00020000);

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

  // ---- input rows: row hi of the frame goes to ring slot hi % 16.
  // Codes in memory: every wave requests a quarter of the row (64 lanes x 4 bytes), so that all
  // waves have the same number of requests in flight.  The bytes behind the row's end belong to
  // the next row, or read as zeros past the tensor: they only meet zero filter bytes or pixels
  // that are not stored.
  const int row_bytes = p.W * 4;
  const int lane_off = n * p.H * row_bytes + wave * 256 + lane * 4;
  auto issue_row = [&](int hi) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(
        rsrc_x,
        (__attribute__((address_space(3))) void*)(ring + (hi & 15) * Sh::ROW_BYTES + wave * 256), 4,
        lane_off + hi * row_bytes, 0, 0, 0);
  };
  // Real-valued image: thread t holds pixel t of a row.  A row of the frame above or below the
  // image is a row of zeros; the frame's columns left and right of the image are zeroed once,
  // below, and never written again.  Every request is made unconditionally, from an address
  // clamped into the image (what it brings is dropped when the row is quantised): the number
  // of requests in flight is then the same in every pass and the waits can be exact.
  const float inv_q = F32IN ? __fdiv_rn(1.0f, im.q) : 0.0f;
  const int c_off1 = min(1, im.C - 1), c_off2 = min(2, im.C - 1), c_off3 = min(3, im.C - 1);
  const float* const img = im.r + ((size_t)n * im.H * im.W + min(tid, im.W - 1)) * im.C;
  auto load_row = [&](int hi, float (&f)[4]) {
    const int h = min(max(hi - im.top, 0), im.H - 1);
    const float* const src = img + (size_t)h * im.W * im.C;
    f[0] = src[0];
    f[1] = src[c_off1];
    f[2] = src[c_off2];
    f[3] = src[c_off3];
  };
  auto store_row = [&](int hi, const float (&f)[4]) {
    const bool row_inside = (unsigned)(hi - im.top) < (unsigned)im.H;
    int z[4] = {0, 0, 0, 0};
    if (row_inside) {
#pragma unroll
      for (int c = 0; c < 3; ++c) z[c] = quant1_fast(f[c], im.q, inv_q, im.lo, im.hi);
      if (im.C > 3) z[3] = quant1_fast(f[3], im.q, inv_q, im.lo, im.hi);
      if (im.C < 3) z[2] = 0;
      if (im.C < 2) z[1] = 0;
    }
    if (tid < im.W)
      *reinterpret_cast<unsigned*>(ring + (hi & 15) * Sh::ROW_BYTES + (im.left + tid) * 4) =
          pack4(z[0], z[1], z[2], z[3]);
  };

  if constexpr (F32IN) {
    for (int c = tid; c < Sh::RING_BYTES / 16; c += NW * 64)
      *reinterpret_cast<v4i*>(ring + c * 16) = v4i{0, 0, 0, 0};
    __syncthreads();
#pragma unroll
    for (int r0 = 0; r0 < 8; r0 += 4) {          // the first output row's image rows, four at a time
      if (r0 < R) {
        float f[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r) load_row(ho_first * sh + r0 + r, f[r]);
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (r0 + r < R) store_row(ho_first * sh + r0 + r, f[r]);
      }
    }
  } else {
    // the rows of the strip's first output row, and what the second one adds
    for (int r = 0; r < R; ++r) issue_row(ho_first * sh + r);
    if (ho_first + 1 < ho_end)
      for (int r = R - sh; r < R; ++r) issue_row((ho_first + 1) * sh + r);
  }

  // ---- fragments.  Filters: LDS row tc * 32 + (lane & 31), bytes r * 32 + 16 * (lane >> 5).
  // Activations: pixel 32 wave + (lane & 31) of the output row, same half.
  const int frag_row = lane & 31, frag_half = lane >> 5;
  const int a_off = frag_row * Sh::FILT_PITCH + 16 * frag_half;
  const int b_off = (wave * 32 + frag_row) * (p.stride_w * 4) + 16 * frag_half;
  v16i bias_v[2];
#pragma unroll
  for (int tc = 0; tc < 2; ++tc) {
    int b[16];
    load_bias16(p, tc * 32 + 16 * frag_half, b);
#pragma unroll
    for (int e = 0; e < 16; ++e) bias_v[tc][e] = b[e];
  }
  const float code_lo = p.relu ? 0.0f : -128.0f;          // ReLU folded into the lower bound
  constexpr float kMagic = 12582912.0f;                   // 1.5 * 2^23: t + kMagic rounds t to an
                                                          // integer, held in the low mantissa bits
  // POOL: running maximum of the ACCUMULATORS over the output rows of the open pooling window.
  // The layer's tail (scale by m > 0, clamp, Round) never decreases when the accumulator
  // grows, so the maximum of the codes is the code of the maximum: the tail runs once per
  // pooled row, on the window's maximum.
  v16i win[2];
#pragma unroll
  for (int tc = 0; tc < 2; ++tc)
#pragma unroll
    for (int e = 0; e < 16; ++e) win[tc][e] = (int)0x80000000;

  wait_vmcnt<0>();
  __syncthreads();

  // Real-valued image: two register buffers of image rows, each requested two passes before
  // it is quantised into the ring (pre_a: what output rows ho_first + 1, + 3, ... add).
  float pre_a[SH][4], pre_b[SH][4];
  auto new_row = [&](int ho, int s) { return ho * sh + R - sh + s; };   // s-th row that ho adds
  if constexpr (F32IN) {
#pragma unroll
    for (int s = 0; s < SH; ++s) load_row(new_row(ho_first + 1, s), pre_a[s]);
#pragma unroll
    for (int s = 0; s < SH; ++s) load_row(new_row(ho_first + 2, s), pre_b[s]);
  }

  // One output row.  pre (real-valued image): the rows output row ho + 1 adds.
  auto row_pass = [&](int ho, float (&pre)[SH][4]) {
    if constexpr (!F32IN) {
      // Codes: request the rows the output row after the next adds (R + 2 SH <= 16: their
      // slots hold rows that no wave reads any more).  In flight, oldest first: the next
      // row's SH requests, the stores of the row before, these SH requests.
      if (ho + 2 < ho_end)
        for (int r = R - sh; r < R; ++r) issue_row((ho + 2) * sh + r);
    }

    // a few filter rows at a time: their fragments are requested together (rows beyond R read
    // valid LDS and are not used); the bias is the first MFMA's addend
    constexpr int GR = POOL ? 2 : 4;                   // POOL holds 32 more registers
    v16i acc[2];
#pragma unroll
    for (int r0 = 0; r0 < 8; r0 += GR) {
      if (r0 < R) {
        v4i af[GR][2], bf[GR];
#pragma unroll
        for (int r = 0; r < GR; ++r) {
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
        for (int r = 0; r < GR; ++r)
          if (r0 + r < R) {
#pragma unroll
            for (int tc = 0; tc < 2; ++tc)
              acc[tc] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                  af[r][tc], bf[r], (r0 + r == 0) ? bias_v[tc] : acc[tc], 0, 0, 0);
          }
      }
    }

    // ---- POOL: an even output row 2j joins the window of pooled row j; an odd row 2j + 1
    // closes it -- the window's maximum is what goes on -- and opens the next one.
    bool emit = true;
    int y_row = ho;                                    // the output row the staging tile holds
    if constexpr (POOL) {
      const bool odd = ho & 1;
      emit = (odd && ho != ho_first) || (!odd && ho == p.Ho - 1);
      y_row = ho >> 1;
      if (odd) {
#pragma unroll
        for (int tc = 0; tc < 2; ++tc)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int a = acc[tc][e];
            acc[tc][e] = max(win[tc][e], a);
            win[tc][e] = a;
          }
      } else {
#pragma unroll
        for (int tc = 0; tc < 2; ++tc)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[tc][e] = win[tc][e] = max(win[tc][e], acc[tc][e]);
      }
    }
    // ---- the layer's tail (the fixed fp32 sequence: convert, scale, clamp with ReLU as the
    // lower bound, Round by adding 1.5 * 2^23, low byte = code) into the staging tile
    if (emit) {
      const int row = wave * 32 + frag_row;
#pragma unroll
      for (int tc = 0; tc < 2; ++tc) {
        const int slot = tc * 2 + frag_half;
        unsigned t[16];
#pragma unroll
        for (int e = 0; e < 16; ++e)
          t[e] = __float_as_uint(
              __builtin_amdgcn_fmed3f((float)acc[tc][e] * p.m, code_lo, 127.0f) + kMagic);
        v4i out;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const unsigned w01 = __builtin_amdgcn_perm(t[4 * a + 1], t[4 * a], 0x0c0c0400u);
          const unsigned w23 = __builtin_amdgcn_perm(t[4 * a + 3], t[4 * a + 2], 0x0c0c0400u);
          out[a] = (int)__builtin_amdgcn_perm(w23, w01, 0x05040100u);
        }
        *reinterpret_cast<v4i*>(stage + row * BC + ((slot ^ swz_out<SLOTS>(row)) << 4)) = out;
      }
    }
    if constexpr (F32IN) {
      // the next output row's image rows into the ring (R + SH <= 16: slots nobody reads);
      // the buffer then takes what the row three further down adds
      if (ho + 1 < ho_end) {
#pragma unroll
        for (int s = 0; s < SH; ++s) store_row(new_row(ho + 1, s), pre[s]);
      }
#pragma unroll
      for (int s = 0; s < SH; ++s) load_row(new_row(ho + 3, s), pre[s]);
    } else {
      // the next output row's image rows have landed; the stores of the row before and the
      // requests made above may still be in flight
      if (ho + 2 < ho_end) wait_vmcnt<2 + SH>(); else wait_vmcnt<2>();
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // this wave's LDS writes are done
    __builtin_amdgcn_s_barrier();
    if (emit) {
      // exactly two store instructions per wave (what the counts above rely on): a lane with
      // nothing to store issues its store out of the buffer's range, where it is dropped
      if constexpr (POOL) {
        // thread = (pooled pixel, 16-channel group): the maximum over columns 2w-1, 2w, 2w+1
        const int wp = tid / SLOTS, g = tid % SLOTS;
        SplitBytes m[4];
#pragma unroll
        for (int k = 0; k < 3; ++k) {
          int col = 2 * wp - 1 + k;
          col = col < 0 ? 0 : (col >= p.Wo ? 2 * wp : col);     // outside: repeat a column inside
          col = col >= BP ? BP - 1 : col;                       // (threads beyond the row: any)
          const v4i cell =
              *reinterpret_cast<const v4i*>(stage + col * BC + ((g ^ swz_out<SLOTS>(col)) << 4));
#pragma unroll
          for (int a = 0; a < 4; ++a) {
            const SplitBytes sb = split_bytes((unsigned)cell[a] ^ 0x80808080u);
            m[a] = k == 0 ? sb : max_bytes(m[a], sb);
          }
        }
        v4i codes;
#pragma unroll
        for (int a = 0; a < 4; ++a) codes[a] = (int)(join_bytes(m[a]) ^ 0x80808080u);
        const int y_off = ((n * im.Hp + y_row) * im.Wp) * p.out_cs + p.out_off;
        const int off = (wp < im.Wp && g * 16 < p.K) ? y_off + wp * p.out_cs + g * 16 : kOobOffset;
        __builtin_amdgcn_raw_buffer_store_b128(codes, rsrc_y, off, 0, 0);
      } else {
        const int y_off = ((n * p.Ho + y_row) * p.Wo) * p.out_cs + p.out_off;
#pragma unroll
        for (int k = 0; k < BP * SLOTS / (NW * 64); ++k) {
          const int c = tid + k * NW * 64;
          const int row = c / SLOTS, g = c % SLOTS;
          const v4i codes =
              *reinterpret_cast<const v4i*>(stage + row * BC + ((g ^ swz_out<SLOTS>(row)) << 4));
          const int off = (row < p.Wo && g * 16 < p.K) ? y_off + row * p.out_cs + g * 16 : kOobOffset;
          __builtin_amdgcn_raw_buffer_store_b128(codes, rsrc_y, off, 0, 0);
        }
      }
      // Every wave has read the staging tile (its stores took the data) before the next
      // codes are written into it; the stores themselves stay in flight.  POOL: the tile is
      // written again two passes later at the earliest, behind the next pass's barrier --
      // except when the image's last output row is an even one and closes a window by itself.
      if (!POOL || ho + 2 == p.Ho) {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
      }
    }
  };
  for (int ho = ho_first; ho < ho_end; ho += 2) {
    row_pass(ho, pre_a);
    if (ho + 1 < ho_end) row_pass(ho + 1, pre_b);
  }
  wait_vmcnt<0>();
#endif
}

// Layers the family takes (codes in memory; the F32IN / POOL entry adds its own conditions).
template <int SH>
bool stem_applicable(const ConvParams& p) {
  return p.stride_h == SH && p.R + 2 * SH <= 16 && p.S4 == 2 && p.S == 1 && p.C == 32 &&
         p.in_cs == 4 && p.R <= 8 && p.K <= 64 && (p.K & 15) == 0 && p.Wo <= 128 && p.W <= 240 &&
         p.stride_w <= 2 && p.pad_h == 0 && p.pad_w == 0 && p.vec16 && !p.res && !p.acc_dump &&
         !p.y_f32 && !p.y_deq && !p.in_u8 && !p.out_u8 && !p.res_u8 && !p.m_vec && !p.w2 && !p.tap_sums &&
         (long)p.N * p.H * p.W * 4 < 0x7fffffffL && (long)p.M * p.out_cs < 0x7fffffffL;
}

template <int SH, bool F32IN, bool POOL>
int launch_stem(ConvParams& p, const StemImage& im, hipStream_t stream) {
  using Sh = StemShape;
  auto kernel = conv_i8_stem_kernel<SH, F32IN, POOL>;
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
  // Strips per image: about as many workgroups as HALF the resident slots -- the layer's
  // other part-batch launch runs beside this one (two pipelines), and a second round of
  // workgroups costs more than longer strips do (ResNet-50's head at 2 x 32 images: 0.711 ->
  // 0.700 ms per step with 5 instead of 3 pooled rows per strip) -- between four and six rows
  // each (POOL: three to six pooled rows, i.e. 7 .. 13 output rows of which one is computed
  // twice).
  const int rows = POOL ? im.Hp : p.Ho, least = POOL ? 3 : 4, most = 6;
  int strips = (resident / 2 + p.N - 1) / p.N;
  if (strips < 1) strips = 1;
  int rows_per_strip = (rows + strips - 1) / strips;
  rows_per_strip = rows_per_strip < least ? least : (rows_per_strip > most ? most : rows_per_strip);
  strips = (rows + rows_per_strip - 1) / rows_per_strip;
  p.n_ptiles = strips;
  p.n_ctiles = rows_per_strip;
  const long grid = (long)p.N * strips;
  if (grid > 0x7fffffffL) return Q8_EUNSUPPORTED;
  hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), Sh::LDS_BYTES, stream, p, im);
  return q8_launch_status();
}

}  // namespace
}  // namespace q8
