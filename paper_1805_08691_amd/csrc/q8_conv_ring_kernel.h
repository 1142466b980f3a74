// Main int8 implicit-GEMM convolution kernel (Eq. x / Eq. A' of arxiv 1805.08691) for
// gfx950: C % 16 == 0 (or an unpadded 4-channel image), more than 32 output channels, at
// most 32 filter taps.
//
// One workgroup (4 or 8 wavefronts) per output tile.  Chunks go from global memory straight into
// LDS (buffer_load_dwordx4 ... lds, no register staging) through a ring of STAGES buffers,
// so several reduction steps of loads are in flight per workgroup while the MFMAs of the
// current step run.  One bare s_barrier per reduction step.
//
// A wavefront-wide direct load writes 64 x 16 bytes to consecutive LDS addresses, i.e. RPW
// rows of BK bytes.  Which global chunk lands in which slot is chosen on the global side:
// lane l fills row l / CHUNKS, physical slot l % CHUNKS, and therefore fetches logical chunk
// (l % CHUNKS) ^ swz(row) of that row (XOR swizzle: conflict-free ds_read_b128 operand reads).
//
// Addressing uses raw buffer descriptors: a per-lane 32-bit offset that is computed once
// (for activations: once per filter tap), plus a wave-uniform scalar offset per reduction
// step, so the loads of the steady state need no vector arithmetic.  A chunk that must read as zero (padding, pixel or channel beyond the
// tensor, reduction tail) gets an offset beyond the descriptor's size: the hardware's
// range check then returns zeros.
//
// UNIFORM = 1 (C % BK == 0): every lane of the block is in the same filter tap during one
// reduction step, so the tap offset is a scalar.  UNIFORM = 2 (S == 1 and BK % C == 0: a
// column filter over few channels, which is also how an unpadded 4-channel image arrives):
// a step covers BK / C whole taps; which of them a lane reads is fixed, and all lanes move
// on by BK / C taps per step, so a lane adds a constant to a scalar.  UNIFORM = 0: each
// lane tracks its own tap.
#pragma once
#include <stdlib.h>
#include <type_traits>
#include "q8_common.h"
#include "q8_conv_common.h"

namespace q8 {
namespace {

constexpr int kOobOffset = (int)0x80000000;   // >= any descriptor size (tensors are < 2 GiB)

#ifdef Q8_TRACE
// Measurement build only: every workgroup logs (start, end) on the 100 MHz clock and what
// identifies its launch into p.trace (word 0 = number of records, 3 words per record).
__device__ __forceinline__ void q8_trace_record(const ConvParams& p, unsigned long long t0) {
  if (threadIdx.x == 0 && p.trace && (blockIdx.x & 15) == 0) {     // one workgroup in 16
    const unsigned long long t1 = __builtin_amdgcn_s_memrealtime();
    const unsigned long long slot = atomicAdd(p.trace, 1ull);
    if (slot < p.trace_cap) {
      p.trace[1 + 3 * slot] = t0;
      p.trace[2 + 3 * slot] = t1;
      p.trace[3 + 3 * slot] = ((unsigned long long)(((uintptr_t)p.y >> 12) & 0x7ffff) << 45) |
                              ((unsigned long long)(unsigned)p.M << 26) |
                              ((unsigned long long)(unsigned)p.K << 14) | ((unsigned)p.C << 2) |
                              (p.R == 3 ? 1u : 0u) | (p.res ? 2u : 0u);
    }
  }
}
#endif

// Epilogue of one tile (tail of Eq. A' with the fused sum): acc[i][j] = the 32 x 32 MFMA tiles of
// this wavefront (channel tile i, pixel tile j; a lane holds 16 consecutive channels of one
// pixel), res_w the residual codes fetched for them.  A complete tile with aligned rows takes
// the branch-free path (complete in pixels; in channels either complete or K a multiple of
// the 16-channel group a lane holds, the groups beyond K being skipped).
template <int TP, int TC, int U8>
__device__ __forceinline__ void finish_tile(const ConvParams& p, const v16i (&acc)[TC][TP],
                                            const int (&res_w)[TC][TP][4], const int pix0,
                                            const int ch0, const int BP, const int BC,
                                            const int wave_p, const int wave_c, const int lane) {
  const bool fast_tile = p.vec16 && !p.acc_dump && !p.y_f32 && !p.y_deq && pix0 + BP <= p.M &&
                         (ch0 + BC <= p.K || (p.K & 15) == 0);
  auto finish_all = [&](auto mode_c) __attribute__((always_inline)) {
    // 0 general; 1 fast; 2 fast + residual; 3, 4, 5: fast with unsigned codes (no
    // residual, signed residual, unsigned residual); 6, 7: fast with per-channel scales
    // (no residual, residual)
    constexpr int MODE = decltype(mode_c)::value;
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      const int ch = ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5);
      if (ch >= p.K) continue;
      float mv[16] = {};
      if constexpr (MODE >= 6) load_scale16(p, ch, mv);
#pragma unroll
      for (int j = 0; j < TP; ++j) {
        const int pix = pix0 + (wave_p * TP + j) * 32 + (lane & 31);
        if (MODE == 0 && pix >= p.M) continue;
        int v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = acc[i][j][e];
        if constexpr (MODE == 0) finish16(p, pix, ch, v, res_w[i][j]);
        else if constexpr (MODE <= 2) finish16_fast<MODE == 2>(p, pix, ch, v, res_w[i][j], mv);
        else if constexpr (MODE <= 5)
          finish16_fast<MODE >= 4, true, MODE == 5>(p, pix, ch, v, res_w[i][j], mv);
        else finish16_fast<MODE == 7, false, false, true>(p, pix, ch, v, res_w[i][j], mv);
      }
    }
  };
  if (!fast_tile) finish_all(std::integral_constant<int, 0>{});
  else if (U8 && p.m_vec) {
    if (p.res) finish_all(std::integral_constant<int, 7>{});
    else finish_all(std::integral_constant<int, 6>{});
  } else if (!p.res) finish_all(std::integral_constant<int, U8 ? 3 : 1>{});
  else if (U8 && p.res_u8) finish_all(std::integral_constant<int, 5>{});
  else finish_all(std::integral_constant<int, U8 ? 4 : 2>{});
}

// U8 = 1: the extended build of the kernel: unsigned activation codes (border correction,
// unsigned residual / output) and per-output-channel scales; kept apart so that the plain
// build's register count, and with it the number of resident wavefronts, stays what it is.
//
// PAIR = 1: the layer is followed by a 1x1 layer that reads nothing else (a bottleneck's
// 3x3 -> 1x1).  The tile spans all K channels, so the workgroup holds every channel of its
// pixels: their int8 codes go to LDS instead of HBM and serve as the activation operand of
// the second layer, all of whose filters wait in LDS behind the ring (requested at kernel
// start).  The two layers' arithmetic is exactly that of two launches.
//
// conv_tile_ring computes ONE output tile (pixel tile `ptile`, channel tile `ctile`) with the
// workgroup's WP*WC wavefronts, using `lds` (STAGES * (BP + BC) * BK bytes, 1 KB aligned) as
// the operand ring.  No vector-memory operation of the workgroup may be outstanding on entry
// (the ring counts its own loads); the caller synchronises the workgroup before `lds` is
// used again.
//
// SPLIT = 1: the reduction of a tile is split over p.n_split workgroups (Eq. x: the integer
// accumulator is a plain sum, so any grouping of its terms gives the same bits).  Workgroup
// `part` runs its share of the reduction steps, stores its partial accumulators in its slab of
// the workspace and bumps the tile's arrival counter; the workgroup that arrives last adds the
// other slabs to its own registers, clears the counter for the next launch and runs the
// epilogue.  Nobody waits for anybody: a workgroup either finishes the tile or leaves.
template <int WP, int WC, int TP, int TC, int BK, int STAGES, int UNIFORM, int U8, int PAIR = 0,
          int SPLIT = 0>
__device__ __forceinline__ void conv_tile_ring(const ConvParams& p, const int ptile,
                                               const int ctile, int8_t* const lds,
                                               const int part = 0) {
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub: buffer
                                      // descriptor types exist for the device target alone
  constexpr int CHUNKS = BK / 16;          // 16-byte chunks per LDS row
  constexpr int RPW = 64 / CHUNKS;         // rows filled by one wavefront-wide load (1 KB)
  constexpr int NH = BK / 32;              // MFMA sub-steps (32 reduction bytes) per step
  constexpr int BP = WP * TP * 32;
  constexpr int BC = WC * TC * 32;
  constexpr int A_GROUPS = BC / RPW, B_GROUPS = BP / RPW;
  constexpr int NW = WP * WC;              // wavefronts per workgroup (4 or 8)
  constexpr int A_LOADS = A_GROUPS / NW, B_LOADS = B_GROUPS / NW;
  constexpr int LOADS = A_LOADS + B_LOADS;                   // per lane per stage
  constexpr int A_BYTES = BC * BK, STAGE_BYTES = (BC + BP) * BK;
  static_assert(BK == 64 || BK == 128, "reduction bytes per step");
  static_assert(NW == 4 || NW == 8, "four or eight wavefronts per block");
  static_assert(A_GROUPS % NW == 0 && B_GROUPS % NW == 0, "every wave issues the same loads");
  static_assert(STAGES >= 2 && STAGES <= 8, "ring depth");
  static_assert((STAGES - 2) * LOADS < 64, "vmcnt is 6 bits");

  const int pix0 = ptile * BP;
  const int ch0 = ctile * BC;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_p = wave % WP;
  const int wave_c = wave / WP;

  const __amdgpu_buffer_rsrc_t rsrc_w =
      __builtin_amdgcn_make_buffer_rsrc((void*)p.w, 0, p.w_bytes, 0x00020000);
  // The activation descriptor starts (pad_h rows + pad_w pixels) BEFORE the tensor: a lane's
  // offset of tap (0,0) of its pixel is then never negative, also where that tap lies in
  // the padding, and can stay in the vector offset while the tap's own (uniform,
  // non-negative) offset goes into the scalar offset.  Nothing is read in front of the
  // tensor: a tap in the padding gets an out-of-range vector offset.
  const int x_shift = (p.pad_h * p.W + p.pad_w) * p.in_cs;
  const __amdgpu_buffer_rsrc_t rsrc_x =
      __builtin_amdgcn_make_buffer_rsrc((void*)(p.x - x_shift), 0, p.x_bytes + x_shift, 0x00020000);

  // ---- loader state: lane l of wave w fills, in its j-th load, row (w + 4j)*RPW + l/CHUNKS,
  // physical slot l % CHUNKS.  The swizzle term only depends on row bits that do not change
  // with j, so the logical chunk a lane fetches is fixed.
  const int lrow = lane / CHUNKS;
  const int lchunk = (lane % CHUNKS) ^ swz<CHUNKS>(wave * RPW + lrow, 0);

  int a_off[A_LOADS];                  // filter row offset + chunk, or out of range
#pragma unroll
  for (int j = 0; j < A_LOADS; ++j) {
    const int row = (wave + NW * j) * RPW + lrow;
    const int ch = ch0 + (row & ~31) + row_to_channel(row & 31);
    a_off[j] = ch < p.K ? ch * p.red_len + lchunk * 16 : kOobOffset;
  }
  const bool pointwise = p.R * p.S == 1 && p.stride_h * p.stride_w == 1 && (p.pad_h | p.pad_w) == 0;
  int b_off[B_LOADS];                  // offset of tap (0,0), channel 0 (+ chunk if UNIFORM)
  unsigned b_mask[B_LOADS];            // bit t: tap t of this pixel lies inside the image
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    const int pix = pix0 + (wave + NW * j) * RPW + lrow;
    unsigned mask = 0;
    int off = 0;
    if (pix < p.M && pointwise) {
      // output pixel = input pixel, no padding
      off = pix * p.in_cs + (UNIFORM == 1 ? lchunk * 16 : 0);
      mask = 1u;
    } else if (pix < p.M) {
      const int n = fast_div(pix, p.div_img_m, p.div_img_s);
      const int rem = pix - n * (p.Ho * p.Wo);
      const int ho = fast_div(rem, p.div_row_m, p.div_row_s);
      const int wo = rem - ho * p.Wo;
      const int hi0 = ho * p.stride_h - p.pad_h;
      const int wi0 = wo * p.stride_w - p.pad_w;
      off = ((n * p.H + hi0) * p.W + wi0) * p.in_cs + x_shift + (UNIFORM == 1 ? lchunk * 16 : 0);
      if ((p.pad_h | p.pad_w) == 0) {
        mask = bits_below(p.R * p.S);      // no padding: every tap of an output pixel is inside
      } else if (p.dil_h == 1 && p.dil_w == 1) {
        // taps inside the image: rows [r_lo, r_hi), columns [s_lo, s_hi)
        const unsigned cols = bits_below(min(p.S, p.W - wi0)) & ~bits_below(-wi0);
        const int r_lo = -hi0, r_hi = p.H - hi0;
        for (int r = 0; r < p.R; ++r)
          if (r >= r_lo && r < r_hi) mask |= cols << (r * p.S);
      } else {
        int t = 0;
        for (int r = 0; r < p.R; ++r) {
          const bool hok = (unsigned)(hi0 + r * p.dil_h) < (unsigned)p.H;
          for (int s2 = 0; s2 < p.S; ++s2, ++t)
            if (hok && (unsigned)(wi0 + s2 * p.dil_w) < (unsigned)p.W) mask |= 1u << t;
        }
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
  // UNIFORM == 2: the lane's tap inside a step and its channel offset inside that tap
  const int row_step = p.dil_h * p.W * p.in_cs;
  const int tap_l = UNIFORM == 2 ? (lchunk * 16) / p.C : 0;
  const int lane_red = lchunk * 16;                    // the lane's reduction byte inside a step
  int b_rowoff[B_LOADS];
  unsigned b_mask_l[B_LOADS];
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) {
    b_rowoff[j] = b_off[j] + tap_l * row_step + (lane_red - tap_l * p.C);
    b_mask_l[j] = b_mask[j] >> tap_l;
  }
  if (UNIFORM == 0) {
    const int red = lchunk * 16;
    tap = red / p.C;
    tap_c = red - tap * p.C;
    const int r = tap / p.S;
    tap_s = tap - r * p.S;
    tap_delta = (r * p.dil_h * p.W + tap_s * p.dil_w) * p.in_cs;
  }

  int b_voff[B_LOADS];                   // UNIFORM: what the B loads of the current tap use
  int tap_changed = 0;
#pragma unroll
  for (int j = 0; j < B_LOADS; ++j) b_voff[j] = (b_mask[j] & 1u) ? b_off[j] : kOobOffset;
  auto refresh_taps = [&]() {            // UNIFORM, after the tap moved on
#pragma unroll
    for (int j = 0; j < B_LOADS; ++j)
      b_voff[j] = ((b_mask[j] >> tap) & 1u) ? b_off[j] : kOobOffset;
  };

  // What the reduction loop reads of `p`, in registers: when `p` lives in global memory (a
  // layer list) the compiler barriers of the loop would otherwise force a reload per step.
  const int p_C = p.C, p_S = p.S, p_red_len = p.red_len;
  // the reduction steps of this workgroup: all of them, or its share of a split reduction
  int nk = (p.red_len + BK - 1) / BK;
  if constexpr (SPLIT) {
    static_assert(UNIFORM == 1 && !U8 && !PAIR, "split reduction: plain uniform-tap builds");
    const int k_first = (int)((long)nk * part / p.n_split);
    nk = (int)((long)nk * (part + 1) / p.n_split) - k_first;
    const int per_tap = p_C / BK;                  // steps per filter tap
    tap = k_first / per_tap;
    tap_c = (k_first - tap * per_tap) * BK;
    const int r = tap / p_S;
    tap_s = tap - r * p_S;
    tap_delta = (r * p.dil_h * p.W + tap_s * p.dil_w) * p.in_cs;
    step_base = k_first * BK;
    refresh_taps();
  }
  auto issue_stage = [&](int buf) {
    int8_t* stage = lds + buf * STAGE_BYTES;
    if constexpr (UNIFORM == 1) {
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_w, (__attribute__((address_space(3))) void*)(stage + (wave + NW * j) * 1024), 16,
            a_off[j], step_base, 0, 0);
      // per lane: the pixel's offset, or "out of range" if the current tap lies in the
      // padding (refreshed only when the tap changes); uniform: the tap's own offset
      const int delta = tap_delta + tap_c;
#pragma unroll
      for (int j = 0; j < B_LOADS; ++j)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_x,
            (__attribute__((address_space(3))) void*)(stage + A_BYTES + (wave + NW * j) * 1024), 16,
            b_voff[j], delta, 0, 0);
      step_base += BK;
      // advance (branch-free, so the whole step stays one scheduling region)
      tap_c += BK;
      const int wrap_c = tap_c >= p_C ? 1 : 0;
      tap_c = wrap_c ? 0 : tap_c;
      tap += wrap_c;
      tap_s += wrap_c;
      tap_delta += wrap_c ? dw_step : 0;
      const int wrap_s = tap_s == p_S ? 1 : 0;
      tap_s = wrap_s ? 0 : tap_s;
      tap_delta += wrap_s ? dh_step : 0;
      tap_changed = wrap_c;
    } else if constexpr (UNIFORM == 2) {
      const bool red_ok = step_base + lane_red < p_red_len;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        const int voff = red_ok ? a_off[j] : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_w, (__attribute__((address_space(3))) void*)(stage + (wave + NW * j) * 1024), 16,
            voff, step_base, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < B_LOADS; ++j) {
        const bool ok = red_ok && ((b_mask_l[j] >> tap) & 1u);
        const int voff = ok ? b_rowoff[j] : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_x,
            (__attribute__((address_space(3))) void*)(stage + A_BYTES + (wave + NW * j) * 1024), 16,
            voff, tap_delta, 0, 0);
      }
      step_base += BK;
      const int taps_per_step = BK / p_C;
      tap += taps_per_step;
      tap_delta += taps_per_step * row_step;
    } else {
      const bool red_ok = step_base + lchunk * 16 < p_red_len;
#pragma unroll
      for (int j = 0; j < A_LOADS; ++j) {
        const int voff = red_ok ? a_off[j] : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_w, (__attribute__((address_space(3))) void*)(stage + (wave + NW * j) * 1024), 16,
            voff, step_base, 0, 0);
      }
      const int delta = tap_delta + tap_c;
#pragma unroll
      for (int j = 0; j < B_LOADS; ++j) {
        const bool ok = red_ok && ((b_mask[j] >> tap) & 1u);
        const int voff = ok ? b_off[j] + delta : kOobOffset;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            rsrc_x,
            (__attribute__((address_space(3))) void*)(stage + A_BYTES + (wave + NW * j) * 1024), 16,
            voff, 0, 0, 0);
      }
      step_base += BK;
      tap_c += BK;
      while (tap_c >= p_C) {
        tap_c -= p_C;
        ++tap;
        tap_delta += dw_step;
        if (++tap_s == p_S) { tap_s = 0; tap_delta += dh_step; }
      }
    }
  };

  // Accumulators start at the bias (Eq. A': the int32 bias shares the accumulator's factor).
  // These loads are issued before any stage load, so the in-order vmcnt bookkeeping of
  // the ring is unaffected, and their latency hides behind the first stages.
  v16i acc[TC][TP];
  // Unsigned input codes (stored minus 128) in a layer with padding: a pixel's accumulators
  // start at the table row of the rectangle of taps it reads inside the image (see
  // u8_start_index) instead of at the bias.
  if (U8 && p.tap_sums) {
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      const int idx = u8_start_index(p, pix0 + (wave_p * TP + j) * 32 + (lane & 31));
#pragma unroll
      for (int i = 0; i < TC; ++i) {
        int b[16];
        load_start16(p, idx, ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5), b);
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = b[e];
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      int b[16];
      load_bias16(p, ch0 + (wave_c * TC + i) * 32 + 16 * (lane >> 5), b);
#pragma unroll
      for (int j = 0; j < TP; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = b[e];
    }
  }
  if constexpr (SPLIT) {
    if (part != 0) {                    // the bias is part 0's
#pragma unroll
      for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
    }
  }
  // Pair build: bias and residual codes of the second layer's first channel tile, requested
  // ahead of the ring like the first layer's bias; double-buffered over its channel tiles.
  v16i bias2[TC];
  int res2[2][TC][TP][4];
  ConvParams p2 = p;
  if constexpr (PAIR) {
    p2.K = p.K2; p2.bias = p.bias2; p2.res = p.res2; p2.y = p.y2;
    p2.out_cs = p.out_cs2; p2.out_off = p.out_off2; p2.res_cs = p.res_cs2; p2.res_off = p.res_off2;
    p2.m = p.m2; p2.m_r = p.m_r2; p2.relu = p.relu2; p2.vec4 = p.vec4_2; p2.vec16 = p.vec16_2;
    p2.acc_dump = nullptr; p2.y_f32 = nullptr; p2.m_vec = nullptr;
  }
  auto fetch_bias2 = [&](int t) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      int b[16];
      load_bias16(p2, t * BC + (wave_c * TC + i) * 32 + 16 * (lane >> 5), b);
#pragma unroll
      for (int e = 0; e < 16; ++e) bias2[i][e] = b[e];
    }
  };
  auto fetch_second = [&](int t, auto buf_c) __attribute__((always_inline)) {
    constexpr int BUF = decltype(buf_c)::value;
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      const int ch = t * BC + (wave_c * TC + i) * 32 + 16 * (lane >> 5);
#pragma unroll
      for (int j = 0; j < TP; ++j)
        load_res16(p2, pix0 + (wave_p * TP + j) * 32 + (lane & 31), ch, res2[BUF][i][j]);
    }
  };
  // ... and ALL its filters, into LDS behind the ring: [K2 / BC tiles][KS2 steps][BC rows][BK]
  constexpr int KS2 = BC / BK;          // reduction steps of the second layer (C2 = BC)
  const int n_pass = PAIR ? p.K2 / BC : 0;
  const int8_t* w2_lds = lds + STAGES * STAGE_BYTES;
  if constexpr (PAIR) {
    fetch_bias2(0);
    fetch_second(0, std::integral_constant<int, 0>{});
    const __amdgpu_buffer_rsrc_t rsrc_w2 =
        __builtin_amdgcn_make_buffer_rsrc((void*)p.w2, 0, p.w2_bytes, 0x00020000);
    for (int t = 0; t < n_pass; ++t)
#pragma unroll
      for (int s2 = 0; s2 < KS2; ++s2)
#pragma unroll
        for (int j = 0; j < A_LOADS; ++j) {
          const int row = (wave + NW * j) * RPW + lrow;
          const int off = ((row & ~31) + row_to_channel(row & 31)) * BC + lchunk * 16;
          __builtin_amdgcn_raw_ptr_buffer_load_lds(
              rsrc_w2,
              (__attribute__((address_space(3))) void*)(lds + STAGES * STAGE_BYTES +
                                                         (t * KS2 + s2) * A_BYTES +
                                                         (wave + NW * j) * 1024),
              16, off, t * BC * BC + s2 * BK, 0, 0);
        }
  }
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
  // (split reduction: only the workgroup that finishes the tile needs them, see below)
  const bool early_residual = nk <= STAGES - 1;
  if (early_residual && !SPLIT) fetch_residual();

  // Operand fragments of the 32-byte sub-steps of a reduction step, double-buffered in
  // registers.  The loop is software-pipelined inside one wavefront: the LDS reads of a
  // sub-step are issued one phase before the MFMAs that consume them, and the MFMAs of the
  // last sub-step of step kt-1 run after the barrier of step kt, so LDS latency, the
  // barrier and the issue of the global loads all overlap matrix work.
  v4i af[2][TC], bf[2][TP];
  // LDS offsets inside a stage, per sub-step.  The swizzle term only looks at row bits below
  // 32, and sub-step h uses chunk 2h + half = (chunk of sub-step 0) ^ 2h: one offset is
  // computed in full, the others differ by a tile's row distance and one XOR.
  int a_foff[NH][TC], b_foff[NH][TP];
  const int foff0 = frag_row * BK + swz<CHUNKS>(frag_row, frag_half) * 16;
#pragma unroll
  for (int h = 0; h < NH; ++h) {
#pragma unroll
    for (int i = 0; i < TC; ++i) {
      a_foff[h][i] = (foff0 ^ (h * 32)) + (wave_c * TC + i) * 32 * BK;
      asm volatile("" : "+v"(a_foff[h][i]));     // keep in a register, do not recompute
    }
#pragma unroll
    for (int j = 0; j < TP; ++j) {
      b_foff[h][j] = (foff0 ^ (h * 32)) + A_BYTES + (wave_p * TP + j) * 32 * BK;
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

  // One reduction step.  LATER = steps issued after step kt that may still be in flight
  // when step kt must have landed; ISSUE = whether a further step is issued; LAST = whether
  // the residual codes are fetched (no stage load follows, so vmcnt bookkeeping is over).
  // STAGE = ring buffer of step kt when the caller knows it at compile time (the LDS reads
  // then need no address arithmetic: fixed per-lane offsets plus an immediate), else -1.
  auto step = [&](int kt, auto later_c, auto issue_c, auto last_c, auto stage_c) {
    constexpr int LATER = decltype(later_c)::value;
    constexpr int STAGE = decltype(stage_c)::value;
    wait_vmcnt<LATER * LOADS>();
    // Every LDS read this wave has issued (the last fragments of step kt-1) has returned:
    // behind the barrier the other waves request step kt+STAGES-1 into the buffer of step
    // kt-1, and a read still queued in the LDS could otherwise be overtaken by that data
    // (seen with several workgroups per CU and operands that come from a warm L2).
    __builtin_amdgcn_s_waitcnt(0xc07f);
    // Bare barrier (no fence: a fence would drain the loads of the later steps too).
    // Step kt is now visible to all waves, and everyone has read step kt-1 out of LDS.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int8_t* stage = lds + (STAGE >= 0 ? STAGE : kt % STAGES) * STAGE_BYTES;
    load_frags(stage, 0);
    if constexpr (decltype(issue_c)::value)
      issue_stage(STAGE >= 0 ? (STAGE + STAGES - 1) % STAGES : (kt + STAGES - 1) % STAGES);
    if constexpr (decltype(last_c)::value) {
      if (!early_residual && !SPLIT) fetch_residual();
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
    if constexpr (UNIFORM == 1 && decltype(issue_c)::value) {
      if (tap_changed) refresh_taps();
    }
  };
  using std::integral_constant;
  constexpr integral_constant<int, -1> any_stage{};

  // prologue: up to STAGES-1 reduction steps in flight
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nk) {
      issue_stage(s);
      if constexpr (UNIFORM == 1) {
        if (tap_changed) refresh_taps();
      }
    }
  // Scalar loads still outstanding here would make every LDS wait inside the loop a full
  // one (scalar and LDS results share a counter but return in no fixed order): settle them
  // now, so the loop waits for exactly the fragments it needs.
  __builtin_amdgcn_s_waitcnt(0xc07f);            // lgkmcnt(0), other counters untouched
  // steady state: every step finds STAGES-2 later steps in flight and issues one more
  int kt = 0;
  // passes over the ring: STAGES steps whose buffers are known at compile time
  for (; kt + 2 * STAGES - 2 < nk; kt += STAGES) {
    auto ring_pass = [&](auto self, auto s_c) __attribute__((always_inline)) -> void {
      constexpr int S = decltype(s_c)::value;
      if constexpr (S < STAGES) {
        step(kt + S, integral_constant<int, STAGES - 2>{}, integral_constant<bool, true>{},
             integral_constant<bool, false>{}, integral_constant<int, S>{});
        self(self, integral_constant<int, S + 1>{});
      }
    };
    ring_pass(ring_pass, integral_constant<int, 0>{});
  }
  for (; kt + STAGES - 1 < nk; ++kt)
    step(kt, integral_constant<int, STAGES - 2>{}, integral_constant<bool, true>{},
         integral_constant<bool, false>{}, any_stage);
  // drain: the last min(STAGES-1, nk) steps, with fewer and fewer loads behind them
#define Q8_DRAIN_STEP(L)                                                              \
  if constexpr (STAGES >= (L) + 2) {                                                  \
    if (nk - kt == (L) + 1) {                                                         \
      step(kt, integral_constant<int, (L)>{}, integral_constant<bool, false>{},       \
           integral_constant<bool, false>{}, any_stage);                              \
      ++kt;                                                                           \
    }                                                                                 \
  }
  Q8_DRAIN_STEP(6)
  Q8_DRAIN_STEP(5)
  Q8_DRAIN_STEP(4)
  Q8_DRAIN_STEP(3)
  Q8_DRAIN_STEP(2)
  Q8_DRAIN_STEP(1)
#undef Q8_DRAIN_STEP
  step(kt, integral_constant<int, 0>{}, integral_constant<bool, false>{},
       integral_constant<bool, true>{}, any_stage);
  mma(NH - 1);
  fold_sums();

  if constexpr (PAIR) {
    static_assert(UNIFORM == 1 && !U8, "pair build: plain uniform-tap kernel only");
    // every wave has read its last operands of the first layer out of LDS
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // The first layer's codes become the second layer's activation operand: the pixel rows
    // of stages 0 .. KS2-1 (step s = channels 64s .. 64s+63), in the loader's swizzle.
    {
      const float no_scales[16] = {};
      const int no_res[4] = {0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j) {
          int v[16];
#pragma unroll
          for (int e = 0; e < 16; ++e) v[e] = acc[i][j][e];
          const v4i codes = codes16_fast<false>(p, v, no_res, no_scales);
          const int chl = (wave_c * TC + i) * 32 + 16 * (lane >> 5);   // channel inside the tile
          const int row = (wave_p * TP + j) * 32 + (lane & 31);        // pixel inside the tile
          const int s2 = chl / BK, c = (chl % BK) / 16;
          *reinterpret_cast<v4i*>(lds + s2 * STAGE_BYTES + A_BYTES + row * BK +
                                  swz<CHUNKS>(row, c) * 16) = codes;
        }
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);            // the code writes
    wait_vmcnt<0>();                               // the second layer's filters (long landed)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // the tile's activations stay in registers for every channel tile
    v4i bfr[KS2][NH][TP];
#pragma unroll
    for (int s2 = 0; s2 < KS2; ++s2)
#pragma unroll
      for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int j = 0; j < TP; ++j)
          bfr[s2][h][j] = *reinterpret_cast<const v4i*>(lds + s2 * STAGE_BYTES + b_foff[h][j]);

    // No synchronisation from here on: filters and activations are in place, a wave walks
    // the channel tiles on its own; bias and residual codes are requested one tile ahead.
    const bool fast2 = p2.vec16 && pix0 + BP <= p.M;
    auto pass = [&](int t, auto buf_c) __attribute__((always_inline)) {
      constexpr int BUF = decltype(buf_c)::value;
      if (t + 1 < n_pass) fetch_second(t + 1, std::integral_constant<int, BUF ^ 1>{});
      const int8_t* wt = w2_lds + t * KS2 * A_BYTES;
#pragma unroll
      for (int s2 = 0; s2 < KS2; ++s2)
#pragma unroll
        for (int h = 0; h < NH; ++h) {
          v4i afr[TC];
#pragma unroll
          for (int i = 0; i < TC; ++i)
            afr[i] = *reinterpret_cast<const v4i*>(wt + s2 * A_BYTES + a_foff[h][i]);
#pragma unroll
          for (int i = 0; i < TC; ++i)
#pragma unroll
            for (int j = 0; j < TP; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                  afr[i], bfr[s2][h][j], (s2 == 0 && h == 0) ? bias2[i] : acc[i][j], 0, 0, 0);
        }
      if (t + 1 < n_pass) fetch_bias2(t + 1);      // the MFMAs above have consumed this tile's
      const float no_scales[16] = {};
#pragma unroll
      for (int i = 0; i < TC; ++i) {
        const int ch = t * BC + (wave_c * TC + i) * 32 + 16 * (lane >> 5);
#pragma unroll
        for (int j = 0; j < TP; ++j) {
          const int pix = pix0 + (wave_p * TP + j) * 32 + (lane & 31);
          int v[16];
#pragma unroll
          for (int e = 0; e < 16; ++e) v[e] = acc[i][j][e];
          if (fast2) {
            if (p2.res) finish16_fast<true>(p2, pix, ch, v, res2[BUF][i][j], no_scales);
            else finish16_fast<false>(p2, pix, ch, v, res2[BUF][i][j], no_scales);
          } else if (pix < p.M) {
            finish16(p2, pix, ch, v, res2[BUF][i][j]);
          }
        }
      }
    };
    for (int t = 0; t < n_pass; t += 2) {
      pass(t, std::integral_constant<int, 0>{});
      if (t + 1 < n_pass) pass(t + 1, std::integral_constant<int, 1>{});
    }
    return;
  }

  if constexpr (SPLIT) {
    // The parts of a tile may run on different XCDs, whose L2 caches do not see each other's
    // lines.  Slabs and counters are therefore written and read past the caches (relaxed
    // atomics of system scope: write-through stores, loads that miss on purpose), which
    // costs a trip to the memory side but no cache-wide write-back or invalidate.
    // Slab layout: register pair h of MFMA tile (i, j) of lane tid at 8-byte word
    // ((i TP + j) 8 + h) NW 64 + tid: every wave-wide access is 512 bytes in one piece.
    using word_t = unsigned long long;
    constexpr int kWords = BP * BC / 2;                       // 8-byte words per slab
    const int tile = ptile * p.n_ctiles + ctile;
    word_t* const slabs = reinterpret_cast<word_t*>(p.ws_slabs) + (size_t)tile * p.n_split * kWords;
    {
      word_t* const mine = slabs + (size_t)part * kWords + tid;
#pragma unroll
      for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
          for (int h = 0; h < 8; ++h)
            __hip_atomic_store(mine + ((i * TP + j) * 8 + h) * (NW * 64),
                               (word_t)(unsigned)acc[i][j][2 * h] |
                                   ((word_t)(unsigned)acc[i][j][2 * h + 1] << 32),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    // every store of this wave has been acknowledged by the memory side ...
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();                     // ... and so have the other waves'; LDS is free
    int* const word = reinterpret_cast<int*>(lds);
    if (wave == 0) {
      int before = 0;
      if (lane == 0)
        before = __hip_atomic_fetch_add(p.ws_counters + tile, 1, __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_SYSTEM);
      before = __builtin_amdgcn_readfirstlane(before);
      if (lane == 0) word[0] = before;
    }
    __syncthreads();
    if (word[0] != p.n_split - 1) return;           // someone else finishes the tile
    fetch_residual();
    for (int other = 0; other < p.n_split; ++other) {
      if (other == part) continue;
      word_t* const theirs = slabs + (size_t)other * kWords + tid;
#pragma unroll
      for (int i = 0; i < TC; ++i)
#pragma unroll
        for (int j = 0; j < TP; ++j)
#pragma unroll
          for (int h = 0; h < 8; ++h) {
            const word_t v = __hip_atomic_load(theirs + ((i * TP + j) * 8 + h) * (NW * 64),
                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            acc[i][j][2 * h] += (int)(unsigned)v;
            acc[i][j][2 * h + 1] += (int)(unsigned)(v >> 32);
          }
    }
    if (wave == 0 && lane == 0)
      __hip_atomic_store(p.ws_counters + tile, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  }
  finish_tile<TP, TC, U8>(p, acc, res_w, pix0, ch0, BP, BC, wave_p, wave_c, lane);
#endif  // __HIP_DEVICE_COMPILE__
}

// One workgroup per output tile.  Workgroup id -> tile: each XCD (workgroups are dealt to
// the XCDs round-robin) gets a contiguous run of tiles, channel tile fastest, so tiles that
// share activations share an L2.
template <int WP, int WC, int TP, int TC, int BK, int STAGES, int UNIFORM, int U8, int PAIR = 0,
          int SPLIT = 0>
__global__ __launch_bounds__(WP * WC * 64) void conv_i8_ring_kernel(const ConvParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];   // the operand ring
  // units of work: tiles, or (tile, part) with the parts of a tile next to each other
  const int nblk = p.n_ptiles * p.n_ctiles * (SPLIT ? p.n_split : 1);
  int bid = blockIdx.x;
  {
    const int xcd = bid % kNumXcd, idx = bid / kNumXcd;
    const int base = nblk / kNumXcd, rem = nblk % kNumXcd;
    bid = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
#ifdef Q8_TRACE
  const unsigned long long q8_t0 = __builtin_amdgcn_s_memrealtime();
#endif
  if constexpr (SPLIT) {
    const int tile = bid / p.n_split;
    conv_tile_ring<WP, WC, TP, TC, BK, STAGES, UNIFORM, U8, PAIR, 1>(
        p, tile / p.n_ctiles, tile % p.n_ctiles, lds, bid - tile * p.n_split);
  } else {
    const int ptile = p.ptile_fastest ? bid % p.n_ptiles : bid / p.n_ctiles;
    const int ctile = p.ptile_fastest ? bid / p.n_ptiles : bid % p.n_ctiles;
    conv_tile_ring<WP, WC, TP, TC, BK, STAGES, UNIFORM, U8, PAIR>(p, ptile, ctile, lds);
  }
#ifdef Q8_TRACE
  q8_trace_record(p, q8_t0);
#endif
#endif
}

template <int WP, int WC, int TP, int TC, int BK, int STAGES, int UNIFORM, int U8, int PAIR = 0>
int launch_ring_grid(const ConvParams& p, dim3 grid, hipStream_t stream) {
  constexpr int kRingBytes = STAGES * (WP * TP + WC * TC) * 32 * BK;
  auto kernel = conv_i8_ring_kernel<WP, WC, TP, TC, BK, STAGES, UNIFORM, U8, PAIR>;
  if constexpr (PAIR) {
    // the ring plus every filter of the second layer
    constexpr int kMaxLds = 160 * 1024;
    const long bytes = kRingBytes + (long)p.K2 * (WC * TC * 32);
    if (bytes > kMaxLds) return Q8_EUNSUPPORTED;
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLds);
    if (attr != hipSuccess) return Q8_EHIP;
    hipLaunchKernelGGL(kernel, grid, dim3(WP * WC * 64), (unsigned)bytes, stream, p);
    return q8_launch_status();
  }
  constexpr int kLdsBytes = kRingBytes;
  if constexpr (kLdsBytes > 65536) {
    // more than 64 KB of LDS per workgroup has to be requested once per kernel
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr != hipSuccess) return Q8_EHIP;
  }
  hipLaunchKernelGGL(kernel, grid, dim3(WP * WC * 64), kLdsBytes, stream, p);
  return q8_launch_status();
}

// Split-reduction launch of a plain uniform-tap build: p.n_split workgroups per output tile.
// The caller has checked split_applicable and set p.n_split, p.ws_counters and p.ws_slabs.
inline bool split_applicable(const ConvParams& p) {
  return p.S4 == 0 && p.C % 64 == 0 && !p.in_u8 && !p.out_u8 && !p.res_u8 && !p.m_vec && !p.w2 &&
         !p.tap_sums;
}
template <int WP, int WC, int TP, int TC, int BK, int STAGES>
int launch_ring_split(ConvParams& p, hipStream_t stream) {
  constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
  constexpr int kLdsBytes = STAGES * (BP + BC) * BK;
  p.n_ptiles = (p.M + BP - 1) / BP;
  p.n_ctiles = (p.K + BC - 1) / BC;
  const long nblk = (long)p.n_ptiles * p.n_ctiles * p.n_split;
  if (nblk > 0x7fffffffL || p.C % BK != 0) return Q8_EUNSUPPORTED;
  auto kernel = conv_i8_ring_kernel<WP, WC, TP, TC, BK, STAGES, 1, 0, 0, 1>;
  if constexpr (kLdsBytes > 65536) {
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (attr != hipSuccess) return Q8_EHIP;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)nblk), dim3(WP * WC * 64), kLdsBytes, stream, p);
  return q8_launch_status();
}

template <int WP, int WC, int TP, int TC, int BK, int STAGES, int U8>
int launch_ring(ConvParams& p, hipStream_t stream) {
  constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
  p.n_ptiles = (p.M + BP - 1) / BP;
  p.n_ctiles = (p.K + BC - 1) / BC;
  long nblk = (long)p.n_ptiles * p.n_ctiles;
  if (nblk > 0x7fffffffL) return Q8_EUNSUPPORTED;
  if (p.C % BK == 0)
    return launch_ring_grid<WP, WC, TP, TC, BK, STAGES, 1, U8>(p, dim3((unsigned)nblk), stream);
  if constexpr (WP * TP * 32 == 128 && WC * TC * 32 == 64 && STAGES == 2 && !U8) {
    // the tile the first (image) layers use also has the column-filter build
    if (p.S == 1 && BK % p.C == 0)
      return launch_ring_grid<WP, WC, TP, TC, BK, STAGES, 2, U8>(p, dim3((unsigned)nblk), stream);
  }
  return launch_ring_grid<WP, WC, TP, TC, BK, STAGES, 0, U8>(p, dim3((unsigned)nblk), stream);
}

// The pair build: tile of WP*TP*32 pixels x all K = WC*TC*32 channels of the first layer.
template <int WP, int WC, int TP, int TC, int BK, int STAGES>
int launch_pair(ConvParams& p, hipStream_t stream) {
  constexpr int BP = WP * TP * 32, BC = WC * TC * 32;
  if (p.K != BC || p.C % BK != 0 || p.K2 % BC != 0 || !p.w2) return Q8_EUNSUPPORTED;
  p.n_ptiles = (p.M + BP - 1) / BP;
  p.n_ctiles = 1;
  return launch_ring_grid<WP, WC, TP, TC, BK, STAGES, 1, 0, 1>(p, dim3((unsigned)p.n_ptiles), stream);
}

// The variants that also exist in the extended build (index, WP, WC, TP, TC, BK, STAGES);
// pixels x channels per tile = (WP*TP*32) x (WC*TC*32); BK bytes per step; ring depth.
#define Q8_RING_EXT_LIST(X)                                                   \
  X(0, 2, 2, 2, 2, 64, 2)   /* 128 x 128 */                                  \
  X(1, 2, 2, 2, 2, 64, 3)                                                     \
  X(2, 2, 2, 2, 2, 64, 4)                                                     \
  X(3, 4, 1, 2, 2, 64, 3)   /* 256 x 64 */                                   \
  X(4, 2, 2, 1, 2, 64, 2)   /* 64 x 128 */                                   \
  X(5, 2, 2, 1, 2, 64, 4)                                                     \
  X(6, 2, 2, 1, 1, 64, 2)   /* 64 x 64 */                                    \
  X(7, 2, 2, 1, 1, 64, 4)                                                     \
  X(8, 2, 2, 2, 1, 64, 2)   /* 128 x 64 */                                   \
  X(9, 2, 2, 2, 1, 64, 4)                                                     \
  X(10, 2, 4, 2, 1, 64, 3)  /* 128 x 128, eight wavefronts of 64 x 32 */     \
  X(11, 2, 4, 2, 1, 64, 4)
constexpr int kNumRingExtVariants = 12;

}  // namespace
}  // namespace q8
