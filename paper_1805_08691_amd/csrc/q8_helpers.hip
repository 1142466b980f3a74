// Helpers that only chain layers or feed calibration; none of them is part of the
// quantised arithmetic of arxiv 1805.08691.  The fp32 convolution produces the
// real-valued activations whose max-abs the calibration step measures.
#include "q8_common.h"

namespace {

constexpr int kThreads = 256;

// fp32 NHWC direct convolution, 64 pixels x 64 channels per block, 4 x 4 outputs per
// thread, reduction staged through LDS 16 values at a time.
constexpr int TP = 64, TCN = 64, TK = 16;

__global__ __launch_bounds__(kThreads) void conv_f32_kernel(
    const float* __restrict__ x, const float* __restrict__ w, const float* __restrict__ b,
    const float* __restrict__ res, float* __restrict__ y, int N, int H, int W, int C, int K,
    int R, int S, int sh, int sw, int ph, int pw, int dh, int dw, int Ho, int Wo, int relu) {
  __shared__ float xs[TK][TP + 1];
  __shared__ float ws[TK][TCN + 1];
  const long M = (long)N * Ho * Wo;
  const long pix0 = (long)blockIdx.x * TP;
  const int ch0 = blockIdx.y * TCN;
  const int tx = threadIdx.x % 16;   // channel group
  const int ty = threadIdx.x / 16;   // pixel group
  float acc[4][4] = {};
  const int RSC = R * S * C;
  // loader: thread moves element (row = tid / 16 + 16*j, kk = tid % 16)
  const int lk = threadIdx.x % TK;
  const int lr = threadIdx.x / TK;
  for (int k0 = 0; k0 < RSC; k0 += TK) {
    const int kidx = k0 + lk;
    int r = 0, s = 0, c = 0;
    const bool kok = kidx < RSC;
    if (kok) {
      int tap = kidx / C;
      c = kidx - tap * C;
      r = tap / S;
      s = tap - r * S;
    }
#pragma unroll
    for (int j = 0; j < TP / 16; ++j) {
      int row = lr + 16 * j;
      long pix = pix0 + row;
      float v = 0.f;
      if (kok && pix < M) {
        int n = (int)(pix / ((long)Ho * Wo));
        int rem = (int)(pix - (long)n * Ho * Wo);
        int ho = rem / Wo, wo = rem - ho * Wo;
        int hi = ho * sh - ph + r * dh, wi = wo * sw - pw + s * dw;
        if ((unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W)
          v = x[(((long)n * H + hi) * W + wi) * C + c];
      }
      xs[lk][row] = v;
    }
#pragma unroll
    for (int j = 0; j < TCN / 16; ++j) {
      int row = lr + 16 * j;
      int ch = ch0 + row;
      ws[lk][row] = (kok && ch < K) ? w[(long)ch * RSC + kidx] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float xv[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) xv[i] = xs[kk][ty * 4 + i];
#pragma unroll
      for (int i = 0; i < 4; ++i) wv[i] = ws[kk][tx * 4 + i];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    long pix = pix0 + ty * 4 + i;
    if (pix >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int ch = ch0 + tx * 4 + j;
      if (ch >= K) continue;
      float v = acc[i][j];
      if (b) v += b[ch];
      if (res) v += res[pix * K + ch];
      if (relu) v = fmaxf(v, 0.f);
      y[pix * K + ch] = v;
    }
  }
}

template <typename T>
__device__ __forceinline__ T lowest();
template <>
__device__ __forceinline__ int8_t lowest<int8_t>() { return -128; }
template <>
__device__ __forceinline__ float lowest<float>() { return -3.402823466e38f; }

template <typename T>
__global__ __launch_bounds__(kThreads) void maxpool_kernel(const T* __restrict__ x, int N, int H,
                                                           int W, int C, int R, int S, int stride,
                                                           int pad, int Ho, int Wo,
                                                           T* __restrict__ y) {
  const size_t total = (size_t)N * Ho * Wo * C;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (size_t)gridDim.x * kThreads) {
    int c = (int)(i % C);
    size_t t = i / C;
    int wo = (int)(t % Wo); t /= Wo;
    int ho = (int)(t % Ho);
    int n = (int)(t / Ho);
    T best = lowest<T>();
    for (int r = 0; r < R; ++r) {
      int hi = ho * stride - pad + r;
      if ((unsigned)hi >= (unsigned)H) continue;
      for (int s = 0; s < S; ++s) {
        int wi = wo * stride - pad + s;
        if ((unsigned)wi >= (unsigned)W) continue;
        T v = x[(((size_t)n * H + hi) * W + wi) * C + c];
        best = v > best ? v : best;
      }
    }
    y[i] = best;
  }
}

// int8 max-pool, 16 channels per thread (C % 16 == 0): 16-byte loads and stores.
typedef int v4i __attribute__((ext_vector_type(4)));
// WIN = 3: a 3 x 3 window, unrolled, all nine taps loaded at once from clamped addresses.
template <int WIN>
__global__ __launch_bounds__(kThreads) void maxpool_i8_vec_kernel(const int8_t* __restrict__ x, int N,
                                                                  int H, int W, int C16, int R, int S,
                                                                  int stride, int pad, int Ho, int Wo,
                                                                  int8_t* __restrict__ y) {
  // 32-bit index arithmetic: the host takes this kernel only below 2^31 items
  const unsigned total = (unsigned)N * Ho * Wo * C16;
  // Workgroups go to the 8 XCDs round robin: renumber them so that each XCD owns one
  // contiguous run of outputs.  Neighbouring output rows share input rows; with this they
  // find them in their own L2 instead of fetching them once per XCD.
  unsigned bid = blockIdx.x;
  {
    const unsigned xcd = bid % 8, idx = bid / 8;
    const unsigned base = gridDim.x / 8, rem = gridDim.x % 8;
    bid = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  for (unsigned i = bid * kThreads + threadIdx.x; i < total; i += gridDim.x * kThreads) {
    int c = (int)(i % (unsigned)C16);
    unsigned t = i / (unsigned)C16;
    int wo = (int)(t % (unsigned)Wo); t /= (unsigned)Wo;
    int ho = (int)(t % (unsigned)Ho);
    int n = (int)(t / (unsigned)Ho);
    // A byte in the high half of a 16-bit lane (low half zero) orders like the int8 it
    // is: odd bytes are masked in place, even bytes shifted up, and each set takes a packed
    // 16-bit max per tap.
    typedef short v2s __attribute__((ext_vector_type(2)));
    unsigned best_odd[4], best_even[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) best_odd[q] = best_even[q] = 0x80008000u;     // -128, -128
    auto take = [&](const v4i& v, bool in) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const unsigned odd = in ? ((unsigned)v[q] & 0xff00ff00u) : 0x80008000u;
        const unsigned even = in ? (((unsigned)v[q] << 8) & 0xff00ff00u) : 0x80008000u;
        const v2s mo = __builtin_elementwise_max(__builtin_bit_cast(v2s, best_odd[q]),
                                                 __builtin_bit_cast(v2s, odd));
        const v2s me = __builtin_elementwise_max(__builtin_bit_cast(v2s, best_even[q]),
                                                 __builtin_bit_cast(v2s, even));
        best_odd[q] = __builtin_bit_cast(unsigned, mo);
        best_even[q] = __builtin_bit_cast(unsigned, me);
      }
    };
    if constexpr (WIN == 3) {
      v4i taps[9];
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
          const int hi = ho * stride - pad + r, wi = wo * stride - pad + s;
          const int hc = min(max(hi, 0), H - 1), wc = min(max(wi, 0), W - 1);
          taps[3 * r + s] =
              *reinterpret_cast<const v4i*>(x + ((((size_t)n * H + hc) * W + wc) * C16 + c) * 16);
        }
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
          const int hi = ho * stride - pad + r, wi = wo * stride - pad + s;
          take(taps[3 * r + s], (unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W);
        }
    } else {
      for (int r = 0; r < R; ++r) {
        int hi = ho * stride - pad + r;
        if ((unsigned)hi >= (unsigned)H) continue;
        for (int s = 0; s < S; ++s) {
          int wi = wo * stride - pad + s;
          if ((unsigned)wi >= (unsigned)W) continue;
          take(*reinterpret_cast<const v4i*>(x + ((((size_t)n * H + hi) * W + wi) * C16 + c) * 16),
               true);
        }
      }
    }
    v4i o;
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = (int)(best_odd[q] | (best_even[q] >> 8));
    *reinterpret_cast<v4i*>(y + (size_t)i * 16) = o;
  }
}

// General int8 pooling into a channel slice with a change of factor (see q8_pool_i8).
#pragma clang fp contract(off)
__global__ __launch_bounds__(kThreads) void pool_i8_kernel(const int8_t* __restrict__ x, int N, int H,
                                                           int W, int C, int mode, int R, int S,
                                                           int stride, int pad, int Ho, int Wo,
                                                           float m, float inv_count,
                                                           int8_t* __restrict__ y, int out_cs,
                                                           int out_off) {
  const size_t total = (size_t)N * Ho * Wo * C;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (size_t)gridDim.x * kThreads) {
    int c = (int)(i % C);
    size_t t = i / C;
    int wo = (int)(t % Wo); t /= Wo;
    int ho = (int)(t % Ho);
    int n = (int)(t / Ho);
    int best = -128, sum = 0;
    for (int r = 0; r < R; ++r) {
      int hi = ho * stride - pad + r;
      if ((unsigned)hi >= (unsigned)H) continue;
      for (int s2 = 0; s2 < S; ++s2) {
        int wi = wo * stride - pad + s2;
        if ((unsigned)wi >= (unsigned)W) continue;
        int v = x[(((size_t)n * H + hi) * W + wi) * C + c];
        best = v > best ? v : best;
        sum += v;
      }
    }
    float f = mode == 0 ? (float)best : (float)sum * inv_count;
    f = f * m;
    f = fminf(fmaxf(f, -128.0f), 127.0f);
    y[(((size_t)n * Ho + ho) * Wo + wo) * out_cs + out_off + c] = (int8_t)(int)rintf(f);
  }
}

// The same with 16 channels per lane (C, out_cs and out_off multiples of 16, 16-byte aligned
// tensors): 16-byte loads and one 16-byte store; workgroups renumbered so that each XCD owns
// a contiguous run of outputs (neighbouring outputs share input rows).
// WIN = 3: a 3 x 3 window, unrolled, every tap loaded unconditionally from a clamped address
// (nine loads in flight per lane) and neutralised afterwards if it lies outside the image;
// WIN = 0: any window, taps outside skipped.
template <int WIN, int MODE>
__global__ __launch_bounds__(kThreads) void pool_i8_vec_kernel(const int8_t* __restrict__ x, int N,
                                                               int H, int W, int C16, int, int R,
                                                               int S, int stride, int pad, int Ho,
                                                               int Wo, float m, float inv_count,
                                                               int8_t* __restrict__ y, int out_cs,
                                                               int out_off) {
  // 32-bit index arithmetic: the host takes this kernel only below 2^31 items
  const unsigned total = (unsigned)N * Ho * Wo * C16;
  unsigned bid = blockIdx.x;
  {
    const unsigned xcd = bid % 8, idx = bid / 8;
    const unsigned base = gridDim.x / 8, rem = gridDim.x % 8;
    bid = xcd * base + (xcd < rem ? xcd : rem) + idx;
  }
  for (unsigned i = bid * kThreads + threadIdx.x; i < total; i += gridDim.x * kThreads) {
    int c = (int)(i % (unsigned)C16);
    unsigned t = i / (unsigned)C16;
    int wo = (int)(t % (unsigned)Wo); t /= (unsigned)Wo;
    int ho = (int)(t % (unsigned)Ho);
    int n = (int)(t / (unsigned)Ho);
    // Two bytes per 32-bit word at a time, as 16-bit lanes: the odd bytes and the even
    // bytes of a word, each sign-extended by a packed arithmetic shift, take a packed max
    // or a packed add per tap (a window of at most 128 taps cannot overflow 16 bits).
    typedef short v2s __attribute__((ext_vector_type(2)));
    v2s acc_odd[4], acc_even[4];
    const short init = MODE == 0 ? (short)-128 : (short)0;
#pragma unroll
    for (int q = 0; q < 4; ++q) acc_odd[q] = acc_even[q] = v2s{init, init};
    auto take = [&](const v4i& v) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int w = v[q], w8 = w << 8;
        const v2s odd = __builtin_bit_cast(v2s, w) >> 8;               // bytes 1 and 3
        const v2s even = __builtin_bit_cast(v2s, w8) >> 8;             // bytes 0 and 2
        if (MODE == 0) {
          acc_odd[q] = __builtin_elementwise_max(acc_odd[q], odd);
          acc_even[q] = __builtin_elementwise_max(acc_even[q], even);
        } else {
          acc_odd[q] += odd;
          acc_even[q] += even;
        }
      }
    };
    if constexpr (WIN == 3) {
      // a tap outside the image reads as the neutral element: -128 in every byte for the
      // maximum, 0 for the sum
      const int neutral = MODE == 0 ? (int)0x80808080 : 0;
      v4i taps[9];
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s2 = 0; s2 < 3; ++s2) {
          const int hi = ho * stride - pad + r, wi = wo * stride - pad + s2;
          const int hc = min(max(hi, 0), H - 1), wc = min(max(wi, 0), W - 1);
          taps[3 * r + s2] =
              *reinterpret_cast<const v4i*>(x + ((((size_t)n * H + hc) * W + wc) * C16 + c) * 16);
        }
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s2 = 0; s2 < 3; ++s2) {
          const int hi = ho * stride - pad + r, wi = wo * stride - pad + s2;
          const bool in = (unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W;
          v4i v = taps[3 * r + s2];
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = in ? v[q] : neutral;
          take(v);
        }
    } else {
      for (int r = 0; r < R; ++r) {
        int hi = ho * stride - pad + r;
        if ((unsigned)hi >= (unsigned)H) continue;
        for (int s2 = 0; s2 < S; ++s2) {
          int wi = wo * stride - pad + s2;
          if ((unsigned)wi >= (unsigned)W) continue;
          take(*reinterpret_cast<const v4i*>(x + ((((size_t)n * H + hi) * W + wi) * C16 + c) * 16));
        }
      }
    }
    // scale, clamp, Round by adding 1.5 * 2^23 (for |t| <= 128 the fp32 sum is the
    // round-half-to-even integer, its low byte the int8 code), byte permutes to pack
    unsigned rr[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int val = (e & 1) ? acc_odd[e >> 2][(e >> 1) & 1] : acc_even[e >> 2][(e >> 1) & 1];
      float f = MODE == 0 ? (float)val : (float)val * inv_count;
      f = f * m;
      f = __builtin_amdgcn_fmed3f(f, -128.0f, 127.0f);
      rr[e] = __float_as_uint(f + 12582912.0f);
    }
    v4i o;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const unsigned w01 = __builtin_amdgcn_perm(rr[4 * a + 1], rr[4 * a], 0x0c0c0400u);
      const unsigned w23 = __builtin_amdgcn_perm(rr[4 * a + 3], rr[4 * a + 2], 0x0c0c0400u);
      o[a] = (int)__builtin_amdgcn_perm(w23, w01, 0x05040100u);
    }
    *reinterpret_cast<v4i*>(y + (((size_t)n * Ho + ho) * Wo + wo) * out_cs + out_off + c * 16) = o;
  }
}

// fp32 twin for the calibration forward (max, or mean with padding counted as zeros).
__global__ __launch_bounds__(kThreads) void pool_f32_kernel(const float* __restrict__ x, int N, int H,
                                                            int W, int C, int mode, int R, int S,
                                                            int stride, int pad, int Ho, int Wo,
                                                            float* __restrict__ y, int out_cs,
                                                            int out_off) {
  const size_t total = (size_t)N * Ho * Wo * C;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total;
       i += (size_t)gridDim.x * kThreads) {
    int c = (int)(i % C);
    size_t t = i / C;
    int wo = (int)(t % Wo); t /= Wo;
    int ho = (int)(t % Ho);
    int n = (int)(t / Ho);
    float best = -3.402823466e38f, sum = 0.f;
    for (int r = 0; r < R; ++r) {
      int hi = ho * stride - pad + r;
      if ((unsigned)hi >= (unsigned)H) continue;
      for (int s2 = 0; s2 < S; ++s2) {
        int wi = wo * stride - pad + s2;
        if ((unsigned)wi >= (unsigned)W) continue;
        float v = x[(((size_t)n * H + hi) * W + wi) * C + c];
        best = fmaxf(best, v);
        sum += v;
      }
    }
    y[(((size_t)n * Ho + ho) * Wo + wo) * out_cs + out_off + c] =
        mode == 0 ? best : sum / (float)(R * S);
  }
}

template <typename T>
int maxpool_launch(const T* x, int N, int H, int W, int C, int R, int S, int stride, int pad,
                   int Ho, int Wo, T* y, void* stream) {
  Q8_REQUIRE(N >= 0 && H >= 1 && W >= 1 && C >= 1 && R >= 1 && S >= 1 && stride >= 1 && pad >= 0 &&
                 Ho >= 0 && Wo >= 0, Q8_EINVAL);
  // every window must hold at least one in-image tap
  Q8_REQUIRE(pad < R && pad < S, Q8_EINVAL);
  Q8_REQUIRE(Ho == 0 || (long)(Ho - 1) * stride - pad < H, Q8_EINVAL);
  Q8_REQUIRE(Wo == 0 || (long)(Wo - 1) * stride - pad < W, Q8_EINVAL);
  size_t total = (size_t)N * Ho * Wo * C;
  if (total == 0) return Q8_OK;
  Q8_REQUIRE(x && y, Q8_EINVAL);
  if constexpr (sizeof(T) == 1) {
    if (C % 16 == 0 && q8_aligned(x, 16) && q8_aligned(y, 16) && total / 16 < 0x7fffffffUL) {
      size_t items = total / 16;
      size_t vb = (items + kThreads - 1) / kThreads;
      if (vb > 65536) vb = 65536;
      if (R == 3 && S == 3)
        hipLaunchKernelGGL(maxpool_i8_vec_kernel<3>, dim3((unsigned)vb), dim3(kThreads), 0,
                           (hipStream_t)stream, (const int8_t*)x, N, H, W, C / 16, R, S, stride, pad,
                           Ho, Wo, (int8_t*)y);
      else
        hipLaunchKernelGGL(maxpool_i8_vec_kernel<0>, dim3((unsigned)vb), dim3(kThreads), 0,
                           (hipStream_t)stream, (const int8_t*)x, N, H, W, C / 16, R, S, stride, pad,
                           Ho, Wo, (int8_t*)y);
      return q8_launch_status();
    }
  }
  size_t blocks = (total + kThreads - 1) / kThreads;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(maxpool_kernel<T>, dim3((unsigned)blocks), dim3(kThreads), 0,
                     (hipStream_t)stream, x, N, H, W, C, R, S, stride, pad, Ho, Wo, y);
  return q8_launch_status();
}

// Register-resident i8 MFMA loop: what the matrix cores sustain with no operand traffic
// (four independent accumulator chains per wave, four waves per block).
typedef int probe_v4i __attribute__((ext_vector_type(4)));
typedef int probe_v16i __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void mfma_i8_probe_kernel(int iters, int32_t* sink) {
  probe_v4i a = {(int)threadIdx.x, 1, 2, 3}, b = {4, 5, 6, (int)blockIdx.x};
  probe_v16i c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int i = 0; i < iters; ++i) {
    c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
  }
  int s = 0;
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == 0x12345678) sink[0] = s;      // keeps the loop alive; practically never taken
}

}  // namespace

extern "C" {

int q8_conv_f32_ref(const q8_conv_desc* d, const float* x_dev, const float* w_dev,
                    const float* b_dev, const float* res_dev, float* y_dev, void* stream) {
  Q8_REQUIRE(d && d->N >= 0 && d->H >= 1 && d->W >= 1 && d->C >= 1 && d->K >= 1 && d->R >= 1 &&
                 d->S >= 1 && d->stride_h >= 1 && d->stride_w >= 1 && d->pad_h >= 0 &&
                 d->pad_w >= 0 && d->dil_h >= 1 && d->dil_w >= 1, Q8_EINVAL);
  const int Ho = q8_conv_out_h(d), Wo = q8_conv_out_w(d);
  const long M = (long)d->N * Ho * Wo;
  if (M == 0) return Q8_OK;
  Q8_REQUIRE(x_dev && w_dev && y_dev, Q8_EINVAL);
  const long bx = (M + TP - 1) / TP;
  const int by = (d->K + TCN - 1) / TCN;
  Q8_REQUIRE(bx <= 0x7fffffffL && by <= 65535, Q8_EUNSUPPORTED);
  hipLaunchKernelGGL(conv_f32_kernel, dim3((unsigned)bx, by), dim3(kThreads), 0, (hipStream_t)stream,
                     x_dev, w_dev, b_dev, res_dev, y_dev, d->N, d->H, d->W, d->C, d->K, d->R, d->S,
                     d->stride_h, d->stride_w, d->pad_h, d->pad_w, d->dil_h, d->dil_w, Ho, Wo,
                     d->relu ? 1 : 0);
  return q8_launch_status();
}

int q8_maxpool_i8(const int8_t* x_dev, int N, int H, int W, int C, int R, int S, int stride, int pad,
                  int Ho, int Wo, int8_t* y_dev, void* stream) {
  return maxpool_launch<int8_t>(x_dev, N, H, W, C, R, S, stride, pad, Ho, Wo, y_dev, stream);
}
int q8_pool_i8(const int8_t* x_dev, int N, int H, int W, int C, int mode, int R, int S, int stride,
               int pad, int Ho, int Wo, float q_in, float q_out, int8_t* y_dev, int out_c_stride,
               int out_c_off, void* stream) {
  Q8_REQUIRE(q8_finite_pos(q_in) && q8_finite_pos(q_out), Q8_EINVAL);
  const float m = q_in / q_out;        // the rescale of Eq. A' between two factors, one fp32 division
  Q8_REQUIRE(N >= 0 && H >= 1 && W >= 1 && C >= 1 && R >= 1 && S >= 1 && stride >= 1 && pad >= 0 &&
                 Ho >= 0 && Wo >= 0 && (mode == 0 || mode == 1), Q8_EINVAL);
  Q8_REQUIRE(pad < R && pad < S && q8_finite_pos(m), Q8_EINVAL);
  Q8_REQUIRE(Ho == 0 || (long)(Ho - 1) * stride - pad < H, Q8_EINVAL);
  Q8_REQUIRE(Wo == 0 || (long)(Wo - 1) * stride - pad < W, Q8_EINVAL);
  Q8_REQUIRE(out_c_off >= 0 && out_c_stride >= out_c_off + C, Q8_EINVAL);
  size_t total = (size_t)N * Ho * Wo * C;
  if (total == 0) return Q8_OK;
  Q8_REQUIRE(x_dev && y_dev, Q8_EINVAL);
  const float inv_count = 1.0f / (float)(R * S);
  if (C % 16 == 0 && out_c_stride % 16 == 0 && out_c_off % 16 == 0 && q8_aligned(x_dev, 16) &&
      q8_aligned(y_dev, 16) && R * S <= 128 && total / 16 < 0x7fffffffUL) {
    size_t vb = (total / 16 + kThreads - 1) / kThreads;
    if (vb > 65536) vb = 65536;
    auto kernel = R == 3 && S == 3 ? (mode == 0 ? pool_i8_vec_kernel<3, 0> : pool_i8_vec_kernel<3, 1>)
                                   : (mode == 0 ? pool_i8_vec_kernel<0, 0> : pool_i8_vec_kernel<0, 1>);
    hipLaunchKernelGGL(kernel, dim3((unsigned)vb), dim3(kThreads), 0, (hipStream_t)stream, x_dev, N, H,
                       W, C / 16, mode, R, S, stride, pad, Ho, Wo, m, inv_count, y_dev, out_c_stride,
                       out_c_off);
    return q8_launch_status();
  }
  size_t blocks = (total + kThreads - 1) / kThreads;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(pool_i8_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                     x_dev, N, H, W, C, mode, R, S, stride, pad, Ho, Wo, m, inv_count, y_dev,
                     out_c_stride, out_c_off);
  return q8_launch_status();
}

int q8_pool_f32(const float* x_dev, int N, int H, int W, int C, int mode, int R, int S, int stride,
                int pad, int Ho, int Wo, float* y_dev, int out_c_stride, int out_c_off, void* stream) {
  Q8_REQUIRE(N >= 0 && H >= 1 && W >= 1 && C >= 1 && R >= 1 && S >= 1 && stride >= 1 && pad >= 0 &&
                 Ho >= 0 && Wo >= 0 && (mode == 0 || mode == 1), Q8_EINVAL);
  Q8_REQUIRE(pad < R && pad < S, Q8_EINVAL);
  Q8_REQUIRE(Ho == 0 || (long)(Ho - 1) * stride - pad < H, Q8_EINVAL);
  Q8_REQUIRE(Wo == 0 || (long)(Wo - 1) * stride - pad < W, Q8_EINVAL);
  Q8_REQUIRE(out_c_off >= 0 && out_c_stride >= out_c_off + C, Q8_EINVAL);
  size_t total = (size_t)N * Ho * Wo * C;
  if (total == 0) return Q8_OK;
  Q8_REQUIRE(x_dev && y_dev, Q8_EINVAL);
  size_t blocks = (total + kThreads - 1) / kThreads;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(pool_f32_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, (hipStream_t)stream,
                     x_dev, N, H, W, C, mode, R, S, stride, pad, Ho, Wo, y_dev, out_c_stride,
                     out_c_off);
  return q8_launch_status();
}

int q8_maxpool_f32(const float* x_dev, int N, int H, int W, int C, int R, int S, int stride, int pad,
                   int Ho, int Wo, float* y_dev, void* stream) {
  return maxpool_launch<float>(x_dev, N, H, W, C, R, S, stride, pad, Ho, Wo, y_dev, stream);
}

int q8_probe_mfma_i8(int blocks, int iters, int32_t* sink_dev, void* stream) {
  Q8_REQUIRE(blocks >= 1 && blocks <= 65536 && iters >= 1 && iters <= (1 << 22) && sink_dev,
             Q8_EINVAL);
  hipLaunchKernelGGL(mfma_i8_probe_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     (hipStream_t)stream, iters, sink_dev);
  return q8_launch_status();
}

}  // extern "C"
