// Device-side pieces shared by the convolution kernels: parameter block, the
// filter-row permutation, the fused epilogue (Eq. A' tail, Eq. +, conv+ReLU / conv+sum
// fusion of arxiv 1805.08691), the LDS slot swizzle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#pragma clang fp contract(off)   // the epilogue's op order is part of the result

namespace q8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v4i_a4 __attribute__((ext_vector_type(4), aligned(4)));

constexpr int kThreads = 256;
constexpr int kNumXcd = 8;

struct ConvParams {
  const int8_t* __restrict__ x;
  const int8_t* __restrict__ w;       // packed filters: [K][red_len] bytes
  const int32_t* __restrict__ bias;
  const int8_t* __restrict__ res;
  int8_t* __restrict__ y;
  int32_t* __restrict__ acc_dump;
  // real-valued output (a layer that leaves the quantised domain): fp32 [M][out_cs] written
  // instead of y; then m is the accumulator's factor q_x*q_w and m_r the residual's q_res
  float* __restrict__ y_f32;
  int f32_vec4;   // 1: fp32 output addresses of 4-channel groups are 16-byte aligned
  // Eq. D on the layer's own output codes in the same launch: fp32 [M][out_cs] laid out like
  // y, y_deq[i] = q_deq * code[i]; null: codes only
  float* __restrict__ y_deq;
  float q_deq;
  int N, H, W, C, K, R, S;
  int stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
  int Ho, Wo;
  int in_cs, out_cs, out_off, res_cs, res_off;
  int M;          // N*Ho*Wo
  int red_len;    // reduction bytes per filter (R*S*C, or R*S4*16 in the 4-channel mode)
  int S4;         // 4-channel mode: 16-byte chunks per filter row (ceil(S/4))
  int n_ptiles, n_ctiles;
  // Which tiles an XCD works on (each XCD has an L2 of its own and takes a contiguous run of
  // the tile order).  0: channel tile fastest -- an XCD holds few pixel tiles and every filter;
  // 1: pixel tile fastest -- an XCD holds few channel tiles and every pixel.  The host picks
  // what fetches fewer bytes over all eight L2s (filters 8 times, or activations 8 times).
  int ptile_fastest;
  int x_bytes, w_bytes;   // sizes of the activation and filter tensors (buffer descriptors)
  int res_bytes;          // size of the residual tensor, 0 if none or beyond 2 GiB
  unsigned div_img_m, div_img_s;   // division of a pixel index by Ho*Wo (see fast_div)
  unsigned div_row_m, div_row_s;   // division by Wo
  // unsigned p = 8 activation codes (0..255), stored as code - 128 (= code ^ 0x80) so that
  // the signed MFMA can take them: the input offset is undone through the bias (+128 times
  // the filter sum, folded by the host) or, in a layer with padding, through the table of
  // start values per rectangle of taps inside the image (see u8_start_index)
  const int32_t* __restrict__ tap_sums;   // [((R+1)*(S+1))^2][K] start values, or null
  int in_u8, out_u8, res_u8;
  const float* __restrict__ m_vec;   // [K] per-output-channel scales replacing m, or null
  float m, m_r;
  int relu;
  int vec4;       // 1: out/res addresses of 4-channel groups are 4-byte aligned
  int vec16;      // 1: out/res addresses of 16-channel groups are 16-byte aligned
  // A second, 1x1 layer run on the tile's own output while it is still in LDS (the pair
  // build of the main kernel; K == the tile's channel count, so a workgroup holds every
  // channel of its pixels).  The first layer's y / out_* / res* are then unused: its codes
  // (scale m, ReLU relu) never leave the chip.
  const int8_t* __restrict__ w2;       // [K2][K] filters of the second layer, null: no pair
  const int32_t* __restrict__ bias2;
  const int8_t* __restrict__ res2;
  int8_t* __restrict__ y2;
  int K2, w2_bytes;
  int out_cs2, out_off2, res_cs2, res_off2;
  float m2, m_r2;
  int relu2, vec4_2, vec16_2;
  // Split reduction (the split builds of the main kernel): n_split workgroups share an output
  // tile, each over a contiguous range of reduction steps.  ws_slabs holds one int32 partial
  // tile per (tile, part), ws_counters one arrival counter per tile (zero between launches).
  int n_split;
  int* __restrict__ ws_counters;
  int* __restrict__ ws_slabs;
#ifdef Q8_TRACE
  unsigned long long* trace;      // measurement build only: workgroup log
  unsigned long long trace_cap;
#endif
};

// The real-valued image of the image-row family's fused builds (pixel (h, w) of image n lies
// at pixel (top + h, left + w) of the zero frame the layer's descriptor describes) and the
// extent of the pooled output.
struct StemImage {
  const float* r;     // [N][H][W][C] fp32
  int H, W, C, top, left;
  float q, lo, hi;    // Eq. Q: factor and code range
  int Hp, Wp;         // with the max-pool: pooled rows and columns
};

// x / d for 0 <= x < 2^31 with host-made constants s = ceil(log2 d), m = ceil(2^(31+s) / d):
// m * d exceeds 2^(31+s) by less than d <= 2^s, so x * m / 2^(31+s) exceeds x / d by less
// than 1/d and has the same integer part.
struct FastDiv {
  unsigned m, s;
};
inline FastDiv make_fast_div(unsigned d) {      // host side, 1 <= d < 2^31
  unsigned s = 0;
  while ((1ull << s) < d) ++s;
  const unsigned long long pw = 1ull << (31 + s);
  return FastDiv{(unsigned)((pw + d - 1) / d), s};
}
__device__ __forceinline__ int fast_div(int x, unsigned m, unsigned s) {
  return (int)(__umulhi((unsigned)x << 1, m) >> s);
}

// Bits [0, k) set, for any k (negative: none, 32 or more: all).
__device__ __forceinline__ unsigned bits_below(int k) {
  return k <= 0 ? 0u : (k >= 32 ? 0xffffffffu : (1u << k) - 1u);
}

// Filter row (within a 32-row MFMA tile) -> output channel.  The 32x32 MFMA leaves, in
// accumulator register 4a+b of a lane in half g, row 8a+4g+b.  Feeding channel 16g+4a+b
// as that row makes the 16 accumulators of a lane 16 CONSECUTIVE channels of one pixel,
// so the epilogue needs one 16-byte residual load and one 16-byte store per lane.
__device__ __forceinline__ int row_to_channel(int row) {
  return (((row >> 2) & 1) << 4) | ((row >> 3) << 2) | (row & 3);
}

// Unsigned input codes are stored minus 128, and sum z w = sum (z - 128) w + 128 * sum w: the
// signed contraction of the stored bytes has to start at bias + 128 * (sum of the filter
// taps the pixel really reads).  A tap in the padding contributes nothing to Eq. A' (the
// stored zero the kernel reads there stands for code 128, not 0), and the taps inside the
// image form a rectangle [r_lo, r_hi) x [s_lo, s_hi) of the filter, so the host tabulates
// the start value of every rectangle:
//   u8_start[idx * K + k] = bias[k] + 128 * sum_{r_lo <= r < r_hi, s_lo <= s < s_hi, c} z_w[k][r][s][c],
//   idx = ((r_lo * (R+1) + r_hi) * (S+1) + s_lo) * (S+1) + s_hi,
// and a pixel's accumulators are loaded from its rectangle's row instead of from the bias.
__device__ __forceinline__ int u8_start_index(const ConvParams& p, int pix) {
  int r_lo = 0, r_hi = p.R, s_lo = 0, s_hi = p.S;          // beyond M: any valid row
  if (pix < p.M) {
    const int n = fast_div(pix, p.div_img_m, p.div_img_s);
    const int rem = pix - n * (p.Ho * p.Wo);
    const int ho = fast_div(rem, p.div_row_m, p.div_row_s);
    const int wo = rem - ho * p.Wo;
    const int hi0 = ho * p.stride_h - p.pad_h;
    const int wi0 = wo * p.stride_w - p.pad_w;
    r_lo = p.R; r_hi = 0; s_lo = p.S; s_hi = 0;
    for (int r = 0; r < p.R; ++r)
      if ((unsigned)(hi0 + r * p.dil_h) < (unsigned)p.H) { r_lo = min(r_lo, r); r_hi = r + 1; }
    for (int s2 = 0; s2 < p.S; ++s2)
      if ((unsigned)(wi0 + s2 * p.dil_w) < (unsigned)p.W) { s_lo = min(s_lo, s2); s_hi = s2 + 1; }
    if (r_hi <= r_lo || s_hi <= s_lo) r_lo = r_hi = s_lo = s_hi = 0;     // nothing inside
  }
  return ((r_lo * (p.R + 1) + r_hi) * (p.S + 1) + s_lo) * (p.S + 1) + s_hi;
}

// The 16 start values of channels [ch, ch+16) from table row `idx` (zero beyond K).
__device__ __forceinline__ void load_start16(const ConvParams& p, int idx, int ch, int (&b)[16]) {
  const int nvalid = p.K - ch;
#pragma unroll
  for (int e = 0; e < 16; ++e) b[e] = 0;
  if (nvalid <= 0) return;
  const int32_t* row = p.tap_sums + (size_t)idx * p.K + ch;
  if (nvalid >= 16 && (p.K & 3) == 0) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const v4i q = *reinterpret_cast<const v4i*>(row + 4 * a);
#pragma unroll
      for (int k = 0; k < 4; ++k) b[4 * a + k] = q[k];
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e)
      if (e < nvalid) b[e] = row[e];
  }
}

// ---- Epilogue pieces, all for 16 consecutive channels [ch, ch+16) of one pixel ------------

// Bias of the 16 channels (zero where there is no bias or the channel is beyond K).
__device__ __forceinline__ void load_bias16(const ConvParams& p, int ch, int (&b)[16]) {
  const int nvalid = p.K - ch;
#pragma unroll
  for (int e = 0; e < 16; ++e) b[e] = 0;
  if (!p.bias || nvalid <= 0) return;
  if (nvalid >= 16) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      v4i bv = *reinterpret_cast<const v4i*>(p.bias + ch + 4 * a);
#pragma unroll
      for (int k = 0; k < 4; ++k) b[4 * a + k] = bv[k];
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e)
      if (e < nvalid) b[e] = p.bias[ch + e];
  }
}

// Per-channel scales of the 16 channels (1 where the channel is beyond K).
__device__ __forceinline__ void load_scale16(const ConvParams& p, int ch, float (&mv)[16]) {
  const int nvalid = p.K - ch;
#pragma unroll
  for (int e = 0; e < 16; ++e) mv[e] = 1.0f;
  if (nvalid >= 16 && (p.K & 3) == 0) {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const v4i q = *reinterpret_cast<const v4i*>(p.m_vec + ch + 4 * a);
#pragma unroll
      for (int k = 0; k < 4; ++k) mv[4 * a + k] = __int_as_float(q[k]);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e)
      if (e < nvalid) mv[e] = p.m_vec[ch + e];
  }
}

// The 16 residual codes, packed four to a word (zero where absent).
__device__ __forceinline__ void load_res16(const ConvParams& p, int pix, int ch, int (&rw)[4]) {
  rw[0] = rw[1] = rw[2] = rw[3] = 0;
  const int nvalid = p.K - ch;
  if (!p.res || nvalid <= 0 || pix >= p.M) return;
  const int8_t* r = p.res + (size_t)pix * p.res_cs + p.res_off + ch;
  if (nvalid >= 16 && p.vec16) {
    v4i q = *reinterpret_cast<const v4i*>(r);
    rw[0] = q[0]; rw[1] = q[1]; rw[2] = q[2]; rw[3] = q[3];
  } else {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      if (p.vec4 && 4 * a + 3 < nvalid) {
        rw[a] = *reinterpret_cast<const int*>(r + 4 * a);
      } else {
#pragma unroll
        for (int b = 0; b < 4; ++b)
          if (4 * a + b < nvalid) rw[a] |= ((int)(uint8_t)r[4 * a + b]) << (8 * b);
      }
    }
  }
}

// Tail of Eq. A' with the fused sum: v = accumulators (bias included), rw = residual codes.
// fp32 scale, residual term, ReLU, clamp, Round, int8 pack, store (and the accumulator dump).
__device__ __forceinline__ void finish16(const ConvParams& p, int pix, int ch, const int (&v)[16],
                                         const int (&rw)[4]) {
  const int nvalid = p.K - ch;          // > 0 guaranteed by the caller
  const bool full = nvalid >= 16;
  if (p.acc_dump) {
    int32_t* d = p.acc_dump + (size_t)pix * p.K + ch;
    if (full && (p.K & 3) == 0) {
#pragma unroll
      for (int a = 0; a < 4; ++a)
        *reinterpret_cast<v4i*>(d + 4 * a) = v4i{v[4 * a], v[4 * a + 1], v[4 * a + 2], v[4 * a + 3]};
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (e < nvalid) d[e] = v[e];
    }
  }
  float t[16];
  if (p.m_vec) {
    float mv[16];
    load_scale16(p, ch, mv);
#pragma unroll
    for (int e = 0; e < 16; ++e) t[e] = (float)v[e] * mv[e];
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) t[e] = (float)v[e] * p.m;
  }
  if (p.res) {
    const int res_add = p.res_u8 ? 128 : 0;        // stored byte + 128 = unsigned code
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int code = (int)(int8_t)((rw[e >> 2] >> (8 * (e & 3))) & 0xff) + res_add;
      float u = (float)code * p.m_r;
      t[e] = t[e] + u;
    }
  }
  if (p.y_f32) {      // Eq. D only: no clamp, no Round
    float* o = p.y_f32 + (size_t)pix * p.out_cs + p.out_off + ch;
    if (p.relu) {
#pragma unroll
      for (int e = 0; e < 16; ++e) t[e] = fmaxf(t[e], 0.0f);
    }
    if (full && p.f32_vec4) {
#pragma unroll
      for (int a = 0; a < 4; ++a)
        *reinterpret_cast<float4*>(o + 4 * a) =
            float4{t[4 * a], t[4 * a + 1], t[4 * a + 2], t[4 * a + 3]};
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (e < nvalid) o[e] = t[e];
    }
    return;
  }
  const float lo = p.out_u8 ? 0.0f : -128.0f, hi = p.out_u8 ? 255.0f : 127.0f;
  const int out_sub = p.out_u8 ? 128 : 0;          // unsigned code - 128 = stored byte
  unsigned zw[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    float u = t[e];
    if (p.relu) u = fmaxf(u, 0.0f);
    u = fminf(fmaxf(u, lo), hi);
    zw[e >> 2] |= ((unsigned)((int)rintf(u) - out_sub) & 0xffu) << (8 * (e & 3));
  }
  if (p.y_deq) {      // Eq. D on the codes just made (signed codes only)
    float* r = p.y_deq + (size_t)pix * p.out_cs + p.out_off + ch;
    float dq[16];
#pragma unroll
    for (int e = 0; e < 16; ++e)
      dq[e] = p.q_deq * (float)(int8_t)((zw[e >> 2] >> (8 * (e & 3))) & 0xff);
    if (full && p.f32_vec4) {
#pragma unroll
      for (int a = 0; a < 4; ++a)
        *reinterpret_cast<float4*>(r + 4 * a) =
            float4{dq[4 * a], dq[4 * a + 1], dq[4 * a + 2], dq[4 * a + 3]};
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e)
        if (e < nvalid) r[e] = dq[e];
    }
  }
  int8_t* o = p.y + (size_t)pix * p.out_cs + p.out_off + ch;
  if (full && p.vec16) {
    *reinterpret_cast<v4i*>(o) = v4i{(int)zw[0], (int)zw[1], (int)zw[2], (int)zw[3]};
  } else {
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      if (p.vec4 && 4 * a + 3 < nvalid) {
        *reinterpret_cast<unsigned*>(o + 4 * a) = zw[a];
      } else {
#pragma unroll
        for (int b = 0; b < 4; ++b)
          if (4 * a + b < nvalid) o[4 * a + b] = (int8_t)((zw[a] >> (8 * b)) & 0xff);
      }
    }
  }
}

// The same tail for a COMPLETE group (all 16 channels valid, 16-byte aligned addresses, no
// accumulator dump), branch-free and with as few vector instructions per element as the
// fixed arithmetic allows: convert, scale, (residual: convert, scale, add), one median for
// ReLU + clamp, and Round by adding 1.5 * 2^23 -- for |t| <= 128 the fp32 sum is the
// round-half-to-even integer and its low byte is the two's-complement int8 code -- then
// byte permutes to pack four codes per word.  Bit-identical to finish16.
// U8: the output may be unsigned codes stored minus 128 (run-time flag: a different clamp
// and one XOR per packed word); RES_U8: the residual holds such codes.
// PC: one scale per output channel (mv) instead of p.m.
template <bool HAS_RES, bool U8 = false, bool RES_U8 = false, bool PC = false>
__device__ __forceinline__ v4i codes16_fast(const ConvParams& p, const int (&v)[16],
                                            const int (&rw)[4], const float (&mv)[16]) {
  const bool out_u8 = U8 && p.out_u8;
  const float lo = (p.relu || out_u8) ? 0.0f : -128.0f;   // ReLU folded into the lower bound
  const float hi = out_u8 ? 255.0f : 127.0f;
  unsigned r[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    float t = (float)v[e] * (PC ? mv[e] : p.m);
    if (HAS_RES) {
      float code;
      if (RES_U8)      // stored byte ^ 0x80 = the unsigned code: one unsigned byte convert
        code = (float)(uint8_t)((((unsigned)rw[e >> 2] ^ 0x80808080u) >> (8 * (e & 3))) & 0xffu);
      else
        code = (float)(int8_t)((rw[e >> 2] >> (8 * (e & 3))) & 0xff);
      const float u = code * p.m_r;
      t = t + u;
    }
    t = __builtin_amdgcn_fmed3f(t, lo, hi);
    r[e] = __float_as_uint(t + 12582912.0f);      // low byte = the code (0..255 or int8)
  }
  const unsigned flip = out_u8 ? 0x80808080u : 0u;   // code - 128 = code ^ 0x80 in a byte
  v4i out;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const unsigned w01 = __builtin_amdgcn_perm(r[4 * a + 1], r[4 * a], 0x0c0c0400u);
    const unsigned w23 = __builtin_amdgcn_perm(r[4 * a + 3], r[4 * a + 2], 0x0c0c0400u);
    out[a] = (int)(__builtin_amdgcn_perm(w23, w01, 0x05040100u) ^ flip);
  }
  return out;
}

template <bool HAS_RES, bool U8 = false, bool RES_U8 = false, bool PC = false>
__device__ __forceinline__ void finish16_fast(const ConvParams& p, int pix, int ch,
                                              const int (&v)[16], const int (&rw)[4],
                                              const float (&mv)[16]) {
  *reinterpret_cast<v4i*>(p.y + (size_t)pix * p.out_cs + p.out_off + ch) =
      codes16_fast<HAS_RES, U8, RES_U8, PC>(p, v, rw, mv);
}

// Whole epilogue in one go (register-staged kernel).
__device__ __forceinline__ void epilogue16(const ConvParams& p, int pix, int ch, int (&v)[16]) {
  int b[16], rw[4];
  load_bias16(p, ch, b);
  load_res16(p, pix, ch, rw);
#pragma unroll
  for (int e = 0; e < 16; ++e) v[e] += b[e];
  finish16(p, pix, ch, v, rw);
}

// 16-byte chunk index -> physical chunk slot inside an LDS row (XOR swizzle so that the
// 16 rows a quarter-wave reads at one reduction offset fall into distinct bank groups).
template <int CHUNKS>
__device__ __forceinline__ int swz(int row, int chunk) {
  if constexpr (CHUNKS == 4) {
    int f = (((row >> 2) & 1) << 1) | (((row >> 1) ^ (row >> 3)) & 1);
    return chunk ^ f;
  } else {
    // 128-byte rows: two rows share a 256-byte bank line, so the slot must differ for the
    // eight row pairs a quarter-wave touches
    return chunk ^ ((row >> 1) & (CHUNKS - 1));
  }
}

// Staging tile of the coalesced epilogue: rows of SLOTS 16-byte channel groups, one row per
// pixel; the slot of group g in row r is g ^ swz_out(r), so that both the lanes of an MFMA
// tile (32 consecutive rows, one group) and a linear sweep over the tile touch all banks.
template <int SLOTS>
__device__ __forceinline__ int swz_out(int row) {
  static_assert(SLOTS == 2 || SLOTS == 4 || SLOTS == 8 || SLOTS == 16, "16-byte groups per row");
  if constexpr (SLOTS == 4) return (row >> 2) & 3;        // 64-byte rows: four rows per bank sweep
  else if constexpr (SLOTS == 2) return (row >> 3) & 1;
  else return (row >> 1) & (SLOTS - 1) & 7;               // 128-byte rows and wider
}

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}


// Entry points of the kernel translation units (host side).
int launch_reg_variant(int variant, ConvParams& p, hipStream_t stream);      // q8_conv_reg.hip
int launch_stream_variant(int variant, ConvParams& p, hipStream_t stream);   // q8_conv_ring.hip
int launch_ring_ext_variant(int variant, ConvParams& p, hipStream_t stream);   // q8_conv_ring_ext.hip
int launch_pair_variant(ConvParams& p, hipStream_t stream);   // q8_conv_ring_pair.hip: K = 64 or 128
const char* stream_variant_name(int variant);
const char* reg_variant_name(int variant);

}  // namespace q8
