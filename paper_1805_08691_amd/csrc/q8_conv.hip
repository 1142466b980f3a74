// int8 x int8 -> int32 implicit-GEMM convolution with the fused requantising epilogue
// (Eq. x, Eq. A' and the conv+ReLU / conv+sum fusions of arxiv 1805.08691), for gfx950.
//
// GEMM view: rows = output channels (filters, the MFMA A operand), columns = output
// pixels n*Ho*Wo (activations, the MFMA B operand), reduction = R*S*C bytes.  With NHWC
// activations and KRSC filters both operands are contiguous along the reduction, so a
// 16-byte chunk (16 channels of one tap) is the unit moved from HBM to LDS and from LDS
// into an MFMA operand register quad.  v_mfma_i32_32x32x32_i8 consumes, per lane, 16
// reduction bytes of one row/column; integer sums are exact, so any assignment of
// reduction bytes to lanes is correct as long as A and B use the same one.
//
// The accumulator layout of the 32x32 MFMA puts four consecutive rows (= channels) of one
// column (= pixel) in four consecutive registers of a lane, which is what the epilogue
// wants: bias, scale, residual, ReLU, Round, clamp on four channels, one packed store.
#include <type_traits>
#include "q8_common.h"
#pragma clang fp contract(off)   // the epilogue's op order is part of the result

namespace {

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
  int N, H, W, C, K, R, S;
  int stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
  int Ho, Wo;
  int in_cs, out_cs, out_off, res_cs, res_off;
  int M;          // N*Ho*Wo
  int red_len;    // reduction bytes per filter (R*S*C, or R*S4*16 in the 4-channel mode)
  int S4;         // 4-channel mode: 16-byte chunks per filter row (ceil(S/4))
  int n_ptiles, n_ctiles;
  int x_bytes, w_bytes;   // sizes of the activation and filter tensors (buffer descriptors)
  float m, m_r;
  int relu;
  int vec4;       // 1: out/res addresses of 4-channel groups are 4-byte aligned
  int vec16;      // 1: out/res addresses of 16-channel groups are 16-byte aligned
};

// Filter row (within a 32-row MFMA tile) -> output channel.  The 32x32 MFMA leaves, in
// accumulator register 4a+b of a lane in half g, row 8a+4g+b.  Feeding channel 16g+4a+b
// as that row makes the 16 accumulators of a lane 16 CONSECUTIVE channels of one pixel,
// so the epilogue needs one 16-byte residual load and one 16-byte store per lane.
__device__ __forceinline__ int row_to_channel(int row) {
  return (((row >> 2) & 1) << 4) | ((row >> 3) << 2) | (row & 3);
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
#pragma unroll
  for (int e = 0; e < 16; ++e) t[e] = (float)v[e] * p.m;
  if (p.res) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      float u = (float)(int8_t)((rw[e >> 2] >> (8 * (e & 3))) & 0xff) * p.m_r;
      t[e] = t[e] + u;
    }
  }
  unsigned zw[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    float u = t[e];
    if (p.relu) u = fmaxf(u, 0.0f);
    u = fminf(fmaxf(u, -128.0f), 127.0f);
    zw[e >> 2] |= ((unsigned)((int)rintf(u)) & 0xffu) << (8 * (e & 3));
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

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

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

  // ---- epilogue: a lane holds 16 consecutive channels of pixel column (lane & 31)
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
      epilogue16(p, pix, ch, v);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Main kernel (C % 16 == 0, R*S <= 32): chunks go from global memory straight into LDS
// (buffer_load_dwordx4 ... lds, no register staging) through a ring of STAGES buffers, so
// several reduction steps of loads are in flight per workgroup while the MFMAs of the
// current step run.  One bare barrier per reduction step.
//
// A wavefront-wide direct load writes 64 x 16 bytes to consecutive LDS addresses, i.e. 16
// rows of 64 bytes.  Which global chunk lands in which slot is chosen on the global side:
// lane l fills row l/4, physical slot l%4, and therefore fetches logical chunk
// (l%4) ^ swz(row) of that row.
//
// Addressing uses raw buffer descriptors: a per-lane 32-bit offset that is computed once,
// plus a wave-uniform offset per reduction step, so a load costs a handful of VALU
// instructions.  A chunk that must read as zero (padding, pixel or channel beyond the
// tensor, reduction tail) gets an offset beyond the descriptor's size: the hardware's
// range check then returns zeros.
//
// UNIFORM (C % 64 == 0): every lane of the block is in the same filter tap during one
// reduction step, so the tap offset is a scalar.  Otherwise each lane tracks its own tap.
constexpr int kOobOffset = (int)0x80000000;   // >= any descriptor size (tensors are < 2 GiB)

template <int WP, int WC, int TP, int TC, int BK, int STAGES, int UNIFORM>
__global__ __launch_bounds__(kThreads) void conv_i8_dma_kernel(const ConvParams p) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub: buffer
                                      // descriptor types exist for the device target alone
  constexpr int CHUNKS = BK / 16;          // 16-byte chunks per LDS row
  constexpr int RPW = 64 / CHUNKS;         // rows filled by one wavefront-wide load (1 KB)
  constexpr int NH = BK / 32;              // MFMA sub-steps (32 reduction bytes) per step
  constexpr int BP = WP * TP * 32;
  constexpr int BC = WC * TC * 32;
  constexpr int A_GROUPS = BC / RPW, B_GROUPS = BP / RPW;
  constexpr int A_LOADS = A_GROUPS / 4, B_LOADS = B_GROUPS / 4;
  constexpr int LOADS = A_LOADS + B_LOADS;                   // per lane per stage
  constexpr int A_BYTES = BC * BK, STAGE_BYTES = (BC + BP) * BK;
  static_assert(BK == 64 || BK == 128, "reduction bytes per step");
  static_assert(WP * WC == 4, "four wavefronts per block");
  static_assert(A_GROUPS % 4 == 0 && B_GROUPS % 4 == 0, "every wave issues the same loads");
  static_assert(STAGES >= 2 && STAGES <= 4, "ring depth");
  static_assert((STAGES - 2) * LOADS < 64, "vmcnt is 6 bits");

  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];   // STAGES * STAGE_BYTES

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
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_p = wave % WP;
  const int wave_c = wave / WP;

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.x, 0, p.x_bytes, 0x00020000);

  // ---- loader state: lane l of wave w fills, in its j-th load, row (w + 4j)*RPW + l/CHUNKS,
  // physical slot l % CHUNKS.  The swizzle term only depends on row bits that do not change
  // with j, so the logical chunk a lane fetches is fixed.
  const int lrow = lane / CHUNKS;
  const int lchunk = (lane % CHUNKS) ^ swz<CHUNKS>(wave * RPW + lrow, 0);

  int a_off[A_LOADS];                  // filter row offset + chunk, or out of range
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int row = (wave + 4 * j) * RPW + lrow;
    const int ch = ch0 + (row & ~31) + row_to_channel(row & 31);
    a_off[j] = ch < p.K ? ch * p.red_len + lchunk * 16 : kOobOffset;
  }
  int b_off[B_LOADS];                  // offset of tap (0,0), channel 0 (+ chunk if UNIFORM)
  unsigned b_mask[B_LOADS];            // bit t: tap t of this pixel lies inside the image
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    const int pix = pix0 + (wave + 4 * j) * RPW + lrow;
    unsigned mask = 0;
    int off = 0;
    if (pix < p.M) {
      const int n = pix / (p.Ho * p.Wo);
      const int rem = pix - n * (p.Ho * p.Wo);
      const int ho = rem / p.Wo;
      const int wo = rem - ho * p.Wo;
      const int hi0 = ho * p.stride_h - p.pad_h;
      const int wi0 = wo * p.stride_w - p.pad_w;
      off = ((n * p.H + hi0) * p.W + wi0) * p.in_cs + (UNIFORM ? lchunk * 16 : 0);
      int t = 0;
      for (int r = 0; r < p.R; ++r) {
        const bool hok = (unsigned)(hi0 + r * p.dil_h) < (unsigned)p.H;
        for (int s2 = 0; s2 < p.S; ++s2, ++t)
          if (hok && (unsigned)(wi0 + s2 * p.dil_w) < (unsigned)p.W) mask |= 1u << t;
      }
    }
    b_off[j] = off;
    b_mask[j] = mask;
  }

  // ---- position in the reduction
  const int dw_step = p.dil_w * p.in_cs;                     // offset step of one tap along S
  const int dh_step = p.dil_h * p.W * p.in_cs - p.S * dw_step;   // extra step when a row wraps
  // UNIFORM: scalars shared by the block.  Otherwise: this lane's own chunk.
  int step_base = 0;                     // reduction byte offset of the next step to issue
  int tap = 0, tap_s = 0, tap_c = 0, tap_delta = 0;
  if (!UNIFORM) {
    const int red = lchunk * 16;
    tap = red / p.C;
    tap_c = red - tap * p.C;
    const int r = tap / p.S;
    tap_s = tap - r * p.S;
    tap_delta = (r * p.dil_h * p.W + tap_s * p.dil_w) * p.in_cs;
  }

  auto issue_stage = [&](int buf) {
    int8_t* stage = lds + buf * STAGE_BYTES;
    if constexpr (UNIFORM) {
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_w, (__attribute__((address_space(3))) void*)(stage + (wave + 4 * j) * 1024), 16,
            a_off[j], step_base, 0, 0);
      const int delta = tap_delta + tap_c;
#pragma unroll
      for (int j = 0; j < B_LOADS; ++j) {
        const int voff = ((b_mask[j] >> tap) & 1u) ? b_off[j] + delta : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_x,
            (__attribute__((address_space(3))) void*)(stage + A_BYTES + (wave + 4 * j) * 1024), 16,
            voff, 0, 0, 0);
      }
      step_base += BK;
      // advance (branch-free, so the whole step stays one scheduling region)
      tap_c += BK;
      const int wrap_c = tap_c >= p.C ? 1 : 0;
      tap_c = wrap_c ? 0 : tap_c;
      tap += wrap_c;
      tap_s += wrap_c;
      tap_delta += wrap_c ? dw_step : 0;
      const int wrap_s = tap_s == p.S ? 1 : 0;
      tap_s = wrap_s ? 0 : tap_s;
      tap_delta += wrap_s ? dh_step : 0;
    } else {
      const bool red_ok = step_base + lchunk * 16 < p.red_len;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        const int voff = red_ok ? a_off[j] : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_w, (__attribute__((address_space(3))) void*)(stage + (wave + 4 * j) * 1024), 16,
            voff, step_base, 0, 0);
      }
      const int delta = tap_delta + tap_c;
#pragma unroll
      for (int j = 0; j < B_LOADS; ++j) {
        const bool ok = red_ok && ((b_mask[j] >> tap) & 1u);
        const int voff = ok ? b_off[j] + delta : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_x,
            (__attribute__((address_space(3))) void*)(stage + A_BYTES + (wave + 4 * j) * 1024), 16,
            voff, 0, 0, 0);
      }
      step_base += BK;
      tap_c += BK;
      while (tap_c >= p.C) {
        tap_c -= p.C;
        ++tap;
        tap_delta += dw_step;
        if (++tap_s == p.S) { tap_s = 0; tap_delta += dh_step; }
      }
    }
  };

  // Accumulators start at the bias (Eq. A': the int32 bias shares the accumulator's factor).
  // These loads are issued before any stage load, so the in-order vmcnt bookkeeping of
  // the ring is unaffected, and their latency hides behind the first stages.
  v16i acc[TC][TP];
#pragma unroll
  for (int i = 0; i < TC; ++i) {
    int b[16];
    load_bias16(p, ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5), b);
#pragma unroll
    for (int j = 0; j < TP; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = b[v];
  }
  const int nk = (p.red_len + BK - 1) / BK;
  const int frag_row = lane & 31;
  const int frag_half = lane >> 5;

  // Residual codes (fused element-wise sum).  With a short reduction (every step fits in
  // the prologue) they are requested first of all, so one memory latency covers bias,
  // residual and operands; otherwise they are requested in the last step.
  int res_w[TC][TP][4];
  auto fetch_residual = [&]() {
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
        load_res16(p, pix0 + (wave_p * TP + j) * 32 + (lane & 31),
                   ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5), res_w[i][j]);
  };
  const bool early_residual = nk <= STAGES - 1;
  if (early_residual) fetch_residual();

  // Operand fragments of the 32-byte sub-steps of a reduction step, double-buffered in
  // registers.  The loop is software-pipelined inside one wavefront: the LDS reads of a
  // sub-step are issued one phase before the MFMAs that consume them, and the MFMAs of the
  // last sub-step of step kt-1 run after the barrier of step kt, so LDS latency, the
  // barrier and the issue of the global loads all overlap matrix work.
  v4i af[2][TC], bf[2][TP];
  int a_foff[NH][TC], b_foff[NH][TP];        // LDS offsets inside a stage, per sub-step
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    const int chunk = 2 * h + frag_half;
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      const int row = (wave_c * TC + i) * 32 + frag_row;
      a_foff[h][i] = row * BK + swz<CHUNKS>(row, chunk) * 16;
      asm volatile("" : "+v"(a_foff[h][i]));     // keep in a register, do not recompute
    }
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      const int row = (wave_p * TP + j) * 32 + frag_row;
      b_foff[h][j] = A_BYTES + row * BK + swz<CHUNKS>(row, chunk) * 16;
      asm volatile("" : "+v"(b_foff[h][j]));
    }
  }
#pragma unroll
  for (int b = 0; b < 2; ++b) {
#pragma unroll
    for (int i = 0; i < TC; ++i) af[b][i] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < TP; ++j) bf[b][j] = v4i{0, 0, 0, 0};
  }
  auto load_frags = [&](const int8_t* stage, int h) {
#pragma unroll
    for (int i = 0; i < TC; ++i)
      af[h & 1][i] = *reinterpret_cast<const v4i*>(stage + a_foff[h][i]);
#pragma unroll
    for (int j = 0; j < TP; ++j)
      bf[h & 1][j] = *reinterpret_cast<const v4i*>(stage + b_foff[h][j]);
  };
  auto mma = [&](int h) {
#pragma unroll
    for (int i = 0; i < TC; ++i)
#pragma unroll
      for (int j = 0; j < TP; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[h & 1][i], bf[h & 1][j], acc[i][j],
                                                          0, 0, 0);
  };

  // One reduction step.  LATER = steps issued after step kt that may still be in flight
  // when step kt must have landed; ISSUE = whether a further step is issued; LAST = whether
  // the residual codes are fetched (no stage load follows, so vmcnt bookkeeping is over).
  auto step = [&](int kt, auto later_c, auto issue_c, auto last_c) {
    constexpr int LATER = decltype(later_c)::value;
    wait_vmcnt<LATER * LOADS>();
    // Bare barrier (no fence: a fence would drain the loads of the later steps too).
    // Step kt is now visible to all waves, and everyone has read step kt-1 out of LDS
    // (its last fragments are in registers already).
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int8_t* stage = lds + (kt % STAGES) * STAGE_BYTES;
    load_frags(stage, 0);
    if constexpr (decltype(issue_c)::value) issue_stage((kt + STAGES - 1) % STAGES);
    if constexpr (decltype(last_c)::value) {
      if (!early_residual) fetch_residual();
    }
    mma(NH - 1);                        // last sub-step of step kt-1 (zeros on the first step)
#pragma unroll
    for (int h = 1; h < NH; ++h) {
      load_frags(stage, h);
      mma(h - 1);
    }
    // Instruction order inside the step (one scheduling region): the LDS reads of the
    // first sub-step; then MFMAs with one global->LDS load after each (a wavefront issues
    // in order: spreading the loads lets a load that waits for queue space hide behind a
    // running MFMA); the LDS reads of sub-step h are spread between the MFMAs of h-1.
    if constexpr (!decltype(last_c)::value) {
      constexpr int kMma = TC * TP, kFrag = TC + TP;
      constexpr int kVmem = decltype(issue_c)::value ? LOADS : 0;
      __builtin_amdgcn_sched_group_barrier(0x100, kFrag, 0);              // DS reads, sub-step 0
      int vmem_left = kVmem;
#pragma unroll
      for (int h = 0; h < NH; ++h) {
#pragma unroll
        for (int g = 0; g < kMma; ++g) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);              // one MFMA
          if (vmem_left > 0) {
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);            // one VMEM read
            --vmem_left;
          }
          if (h + 1 < NH && g < kFrag)
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);            // one DS read
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  using std::integral_constant;

  // prologue: up to STAGES-1 reduction steps in flight
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nk) issue_stage(s);
  // steady state: every step finds STAGES-2 later steps in flight and issues one more
  int kt = 0;
  for (; kt + STAGES - 1 < nk; ++kt)
    step(kt, integral_constant<int, STAGES - 2>{}, integral_constant<bool, true>{},
         integral_constant<bool, false>{});
  // drain: the last min(STAGES-1, nk) steps, with fewer and fewer loads behind them
  if constexpr (STAGES >= 4) {
    if (nk - kt == 3) {
      step(kt, integral_constant<int, 2>{}, integral_constant<bool, false>{},
           integral_constant<bool, false>{});
      ++kt;
    }
  }
  if constexpr (STAGES >= 3) {
    if (nk - kt == 2) {
      step(kt, integral_constant<int, 1>{}, integral_constant<bool, false>{},
           integral_constant<bool, false>{});
      ++kt;
    }
  }
  step(kt, integral_constant<int, 0>{}, integral_constant<bool, false>{},
       integral_constant<bool, true>{});
  mma(NH - 1);

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
      finish16(p, pix, ch, v, res_w[i][j]);
    }
  }
#endif  // __HIP_DEVICE_COMPILE__
}

// dense KRSC (true C <= 4) -> [K][R][S4][4 taps][4 channels], zero filled
__global__ void pack_c4_kernel(const int8_t* __restrict__ w, int K, int R, int S, int C, int S4,
                               int8_t* __restrict__ out) {
  const int row_len = R * S4 * 16;
  const size_t total = (size_t)K * row_len;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (size_t)gridDim.x * blockDim.x) {
    int k = (int)(i / row_len);
    int o = (int)(i - (size_t)k * row_len);
    int r = o / (S4 * 16);
    int o2 = o - r * S4 * 16;
    int s = o2 >> 2, c = o2 & 3;
    int8_t v = 0;
    if (s < S && c < C) v = w[(((size_t)k * R + r) * S + s) * C + c];
    out[i] = v;
  }
}

__global__ void copy_bytes_kernel(const int8_t* __restrict__ src, size_t n, int8_t* __restrict__ dst) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

int out_extent(int in, int pad, int dil, int k, int stride) {
  long span = (long)dil * (k - 1) + 1;
  long t = (long)in + 2L * pad - span;
  if (t < 0) return 0;
  return (int)(t / stride) + 1;
}

bool desc_sane(const q8_conv_desc* d) {
  return d && d->N >= 0 && d->H >= 1 && d->W >= 1 && d->C >= 1 && d->K >= 1 && d->R >= 1 &&
         d->S >= 1 && d->stride_h >= 1 && d->stride_w >= 1 && d->pad_h >= 0 && d->pad_w >= 0 &&
         d->dil_h >= 1 && d->dil_w >= 1;
}

// 0: 16-channel chunks; 1: 4-channel pixels; -1: unsupported
int conv_mode(const q8_conv_desc* d) {
  if (d->C % 16 == 0) return 0;
  if (d->C <= 4) return 1;
  return -1;
}

// Kernel variants.  "dma" = direct-to-LDS ring kernel (C % 16 == 0, K > 32, R*S <= 32);
// "reg" = register-staged kernel (4-channel images, K <= 32, R*S > 32).
enum Variant {
  V_DMA64_128x128_S2, V_DMA64_128x128_S3, V_DMA64_128x128_S4, V_DMA64_256x64_S2, V_DMA64_256x64_S3,
  V_DMA128_128x128_S2, V_DMA128_128x128_S3, V_DMA128_256x64_S2, V_DMA128_256x64_S3,
  V_REG_128x128, V_REG_256x64, V_REG_256x32, V_REG4_128x128, V_REG4_256x64, V_REG4_256x32, V_COUNT
};
const char* const kVariantNames[V_COUNT] = {
    "conv_i8_dma_kernel<2,2,2,2,64,2>", "conv_i8_dma_kernel<2,2,2,2,64,3>",
    "conv_i8_dma_kernel<2,2,2,2,64,4>", "conv_i8_dma_kernel<4,1,2,2,64,2>",
    "conv_i8_dma_kernel<4,1,2,2,64,3>",
    "conv_i8_dma_kernel<2,2,2,2,128,2>", "conv_i8_dma_kernel<2,2,2,2,128,3>",
    "conv_i8_dma_kernel<4,1,2,2,128,2>", "conv_i8_dma_kernel<4,1,2,2,128,3>",
    "conv_i8_kernel<2,2,2,2,64,0>", "conv_i8_kernel<4,1,2,2,64,0>",
    "conv_i8_kernel<4,1,2,1,64,0>", "conv_i8_kernel<2,2,2,2,64,1>", "conv_i8_kernel<4,1,2,2,64,1>",
    "conv_i8_kernel<4,1,2,1,64,1>"};

int g_variant_override = -1;   // tests / tuning: force a "dma" variant where it is applicable

int pick_variant(const q8_conv_desc* d) {
  const int mode = conv_mode(d);
  if (g_variant_override >= 0 && g_variant_override < V_REG_128x128 && mode == 0 && d->K > 32 &&
      d->R * d->S <= 32)
    return g_variant_override;
  if (mode == 1) return d->K > 64 ? V_REG4_128x128 : d->K > 32 ? V_REG4_256x64 : V_REG4_256x32;
  if (d->K <= 32) return V_REG_256x32;
  if (d->R * d->S > 32) return d->K > 64 ? V_REG_128x128 : V_REG_256x64;   // tap mask is 32 bits
  const int red = d->R * d->S * d->C;
  const bool wide = d->K > 64;
  if (d->C % 128 == 0) {
    // full 128-byte lines per row and step: the L2 -> LDS path is ~1.6x faster than with
    // 64-byte segments, and there are half as many barriers
    const int nk = red / 128;
    if (wide) return nk <= 2 ? V_DMA128_128x128_S2 : V_DMA128_128x128_S3;
    return nk <= 2 ? V_DMA128_256x64_S2 : V_DMA128_256x64_S3;
  }
  const int nk = (red + 63) / 64;     // reduction steps of 64 bytes
  if (wide) return nk <= 1 ? V_DMA64_128x128_S2 : nk <= 4 ? V_DMA64_128x128_S3 : V_DMA64_128x128_S4;
  return nk <= 1 ? V_DMA64_256x64_S2 : V_DMA64_256x64_S3;
}

template <int BP, int BC, typename F>
int launch_tiles(ConvParams& p, F&& launch_fn) {
  p.n_ptiles = (p.M + BP - 1) / BP;
  p.n_ctiles = (p.K + BC - 1) / BC;
  long nblk = (long)p.n_ptiles * p.n_ctiles;
  if (nblk > 0x7fffffffL) return Q8_EUNSUPPORTED;
  launch_fn(dim3((unsigned)nblk));
  return q8_launch_status();
}

template <int WP, int WC, int TP, int TC, int MODE>
int launch_reg(ConvParams& p, hipStream_t stream) {
  return launch_tiles<WP * TP * 32, WC * TC * 32>(p, [&](dim3 grid) {
    hipLaunchKernelGGL((conv_i8_kernel<WP, WC, TP, TC, 64, MODE>), grid, dim3(kThreads), 0, stream, p);
  });
}

template <int WP, int WC, int TP, int TC, int BK, int STAGES, int UNIFORM>
int launch_dma_grid(const ConvParams& p, dim3 grid, hipStream_t stream) {
  constexpr int kLdsBytes = STAGES * (WP * TP + WC * TC) * 32 * BK;
  auto kernel = conv_i8_dma_kernel<WP, WC, TP, TC, BK, STAGES, UNIFORM>;
  if constexpr (kLdsBytes > 65536) {
    // more than 64 KB of LDS per workgroup has to be requested once per kernel
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr != hipSuccess) return Q8_EHIP;
  }
  hipLaunchKernelGGL(kernel, grid, dim3(kThreads), kLdsBytes, stream, p);
  return q8_launch_status();
}

template <int WP, int WC, int TP, int TC, int BK, int STAGES>
int launch_dma(ConvParams& p, hipStream_t stream) {
  constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
  p.n_ptiles = (p.M + BP - 1) / BP;
  p.n_ctiles = (p.K + BC - 1) / BC;
  long nblk = (long)p.n_ptiles * p.n_ctiles;
  if (nblk > 0x7fffffffL) return Q8_EUNSUPPORTED;
  if (p.C % BK == 0)
    return launch_dma_grid<WP, WC, TP, TC, BK, STAGES, 1>(p, dim3((unsigned)nblk), stream);
  return launch_dma_grid<WP, WC, TP, TC, BK, STAGES, 0>(p, dim3((unsigned)nblk), stream);
}

}  // namespace

extern "C" {

int q8_conv_out_h(const q8_conv_desc* d) {
  if (!desc_sane(d)) return 0;
  return out_extent(d->H, d->pad_h, d->dil_h, d->R, d->stride_h);
}
int q8_conv_out_w(const q8_conv_desc* d) {
  if (!desc_sane(d)) return 0;
  return out_extent(d->W, d->pad_w, d->dil_w, d->S, d->stride_w);
}

size_t q8_packed_weight_bytes(const q8_conv_desc* d) {
  if (!desc_sane(d)) return 0;
  int mode = conv_mode(d);
  if (mode == 0) return (size_t)d->K * d->R * d->S * d->C;
  if (mode == 1) return (size_t)d->K * d->R * ((d->S + 3) / 4) * 16;
  return 0;
}

int q8_pack_weights(const q8_conv_desc* d, const int8_t* z_w_krsc_dev, void* packed_dev,
                    void* stream) {
  Q8_REQUIRE(desc_sane(d) && z_w_krsc_dev && packed_dev, Q8_EINVAL);
  int mode = conv_mode(d);
  Q8_REQUIRE(mode >= 0, Q8_EUNSUPPORTED);
  Q8_REQUIRE(q8_aligned(packed_dev, 16), Q8_EALIGN);
  size_t bytes = q8_packed_weight_bytes(d);
  int blocks = (int)((bytes + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  if (mode == 0)
    hipLaunchKernelGGL(copy_bytes_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       z_w_krsc_dev, bytes, (int8_t*)packed_dev);
  else
    hipLaunchKernelGGL(pack_c4_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       z_w_krsc_dev, d->K, d->R, d->S, d->C, (d->S + 3) / 4, (int8_t*)packed_dev);
  return q8_launch_status();
}

int q8_conv_int8(const q8_conv_desc* d, const int8_t* z_x, const void* z_w_packed,
                 const int32_t* bias_i32, float q_x, float q_w, float q_out,
                 const int8_t* residual, float q_res, int8_t* z_y, int32_t* acc_dump,
                 void* stream) {
  Q8_REQUIRE(desc_sane(d), Q8_EINVAL);
  Q8_REQUIRE(q8_finite_pos(q_x) && q8_finite_pos(q_w) && q8_finite_pos(q_out), Q8_EINVAL);
  Q8_REQUIRE(residual == nullptr || q8_finite_pos(q_res), Q8_EINVAL);
  const int mode = conv_mode(d);
  Q8_REQUIRE(mode >= 0, Q8_EUNSUPPORTED);

  ConvParams p{};
  p.N = d->N; p.H = d->H; p.W = d->W; p.C = d->C; p.K = d->K; p.R = d->R; p.S = d->S;
  p.stride_h = d->stride_h; p.stride_w = d->stride_w; p.pad_h = d->pad_h; p.pad_w = d->pad_w;
  p.dil_h = d->dil_h; p.dil_w = d->dil_w;
  p.Ho = q8_conv_out_h(d); p.Wo = q8_conv_out_w(d);
  p.in_cs = d->in_c_stride ? d->in_c_stride : (mode == 1 ? 4 : d->C);
  p.out_cs = d->out_c_stride ? d->out_c_stride : d->K;
  p.out_off = d->out_c_off;
  p.res_cs = d->res_c_stride ? d->res_c_stride : d->K;
  p.res_off = d->res_c_off;
  Q8_REQUIRE(p.in_cs >= d->C && p.out_off >= 0 && p.res_off >= 0, Q8_EINVAL);
  Q8_REQUIRE(p.out_cs >= p.out_off + d->K, Q8_EINVAL);
  Q8_REQUIRE(residual == nullptr || p.res_cs >= p.res_off + d->K, Q8_EINVAL);

  const long M = (long)d->N * p.Ho * p.Wo;
  if (M == 0) return Q8_OK;
  Q8_REQUIRE(M <= 0x7fffffffL, Q8_EUNSUPPORTED);
  Q8_REQUIRE((long)d->H * d->W * p.in_cs <= 0x7fffffffL, Q8_EUNSUPPORTED);
  Q8_REQUIRE(z_x && z_w_packed && z_y, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(z_w_packed, 16), Q8_EALIGN);
  if (mode == 0) {
    Q8_REQUIRE(p.in_cs % 16 == 0 && q8_aligned(z_x, 16), Q8_EALIGN);
    p.red_len = d->R * d->S * d->C;
    p.S4 = 0;
  } else {
    Q8_REQUIRE(p.in_cs == 4 && q8_aligned(z_x, 4), Q8_EALIGN);
    Q8_REQUIRE(d->dil_w == 1 && d->dil_h == 1, Q8_EUNSUPPORTED);
    p.S4 = (d->S + 3) / 4;
    p.red_len = d->R * p.S4 * 16;
  }
  Q8_REQUIRE(bias_i32 == nullptr || q8_aligned(bias_i32, 16), Q8_EALIGN);
  Q8_REQUIRE(acc_dump == nullptr || q8_aligned(acc_dump, 16), Q8_EALIGN);

  {
    const long xb = (long)d->N * d->H * d->W * p.in_cs, wb = (long)d->K * p.red_len;
    Q8_REQUIRE(xb < 0x7fffffffL && wb < 0x7fffffffL, Q8_EUNSUPPORTED);   // 32-bit buffer offsets
    p.x_bytes = (int)xb;
    p.w_bytes = (int)wb;
  }
  p.x = z_x; p.w = (const int8_t*)z_w_packed; p.bias = bias_i32; p.res = residual; p.y = z_y;
  p.acc_dump = acc_dump;
  p.M = (int)M;
  p.relu = d->relu ? 1 : 0;
  {
    float prod = q_x * q_w;      // the x rule: factor of the accumulator
    p.m = prod / q_out;
    p.m_r = residual ? q_res / q_out : 0.0f;
  }
  auto aligned_to = [&](int a) {
    return p.out_cs % a == 0 && p.out_off % a == 0 && q8_aligned(z_y, a) &&
           (residual == nullptr ||
            (p.res_cs % a == 0 && p.res_off % a == 0 && q8_aligned(residual, a)));
  };
  p.vec4 = aligned_to(4) ? 1 : 0;
  p.vec16 = aligned_to(16) ? 1 : 0;

  hipStream_t s = (hipStream_t)stream;
  switch (pick_variant(d)) {
    case V_DMA64_128x128_S2: return launch_dma<2, 2, 2, 2, 64, 2>(p, s);
    case V_DMA64_128x128_S3: return launch_dma<2, 2, 2, 2, 64, 3>(p, s);
    case V_DMA64_128x128_S4: return launch_dma<2, 2, 2, 2, 64, 4>(p, s);
    case V_DMA64_256x64_S2: return launch_dma<4, 1, 2, 2, 64, 2>(p, s);
    case V_DMA64_256x64_S3: return launch_dma<4, 1, 2, 2, 64, 3>(p, s);
    case V_DMA128_128x128_S2: return launch_dma<2, 2, 2, 2, 128, 2>(p, s);
    case V_DMA128_128x128_S3: return launch_dma<2, 2, 2, 2, 128, 3>(p, s);
    case V_DMA128_256x64_S2: return launch_dma<4, 1, 2, 2, 128, 2>(p, s);
    case V_DMA128_256x64_S3: return launch_dma<4, 1, 2, 2, 128, 3>(p, s);
    case V_REG_128x128: return launch_reg<2, 2, 2, 2, 0>(p, s);
    case V_REG_256x64: return launch_reg<4, 1, 2, 2, 0>(p, s);
    case V_REG_256x32: return launch_reg<4, 1, 2, 1, 0>(p, s);
    case V_REG4_128x128: return launch_reg<2, 2, 2, 2, 1>(p, s);
    case V_REG4_256x64: return launch_reg<4, 1, 2, 2, 1>(p, s);
    default: return launch_reg<4, 1, 2, 1, 1>(p, s);
  }
}

int q8_conv_force_variant(int index) {
  if (index < -1 || index >= V_REG_128x128) return Q8_EINVAL;
  g_variant_override = index;
  return Q8_OK;
}

const char* q8_conv_variant(const q8_conv_desc* d) {
  if (!desc_sane(d) || conv_mode(d) < 0) return "unsupported";
  return kVariantNames[pick_variant(d)];
}

}  // extern "C"
