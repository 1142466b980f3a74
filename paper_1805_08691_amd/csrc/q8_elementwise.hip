// HBM-bound passes of the quantised-convolution path: max-abs calibration, the
// quantiser Q, the dequantiser D, batch-norm folding and the p = 31 bias quantiser
// (Eq. Q, Eq. D, Eq. BN and the calibration text of arxiv 1805.08691).
//
// Every floating-point step is one IEEE binary32 (or binary64) operation: contraction
// into fused multiply-adds is switched off for this file, and division and square root
// are the correctly rounded ones (hipcc -fhip-fp32-correctly-rounded-divide-sqrt, the
// default).  __fsqrt_rn is NOT used: without OCML_BASIC_ROUNDED_OPERATIONS it maps to the
// approximate native square root.
#include "q8_common.h"
#include "q8_quant.h"
#pragma clang fp contract(off)

namespace {

using q8::pack4;
using q8::quant1;
using q8::quant1_fast;

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 256 * 8;   // 256 CUs x 8 resident blocks

inline int blocks_for(size_t work_items) {
  size_t b = (work_items + kThreads - 1) / kThreads;
  if (b < 1) b = 1;
  if (b > (size_t)kMaxBlocks) b = kMaxBlocks;
  return (int)b;
}

// ---------------------------------------------------------------- max-abs ----------
// One running maximum per tensor.  Every block owns one contiguous run of 16-byte vectors
// and walks it with sixteen independent non-temporal loads in flight per lane (measured on
// 205 MB and on 1 GiB: 7.0 TB/s this way against 5.3 - 6.3 TB/s when all blocks sweep the
// tensor together in grid-sized strides); a wavefront folds with lane shuffles, the four
// wavefronts of a block fold through LDS, and one atomic per block updates the result.
// |x| >= 0, so the IEEE bit pattern orders like an unsigned integer.
typedef float f4_nt __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float abs4max(f4_nt v) {
  return fmaxf(fmaxf(fabsf(v[0]), fabsf(v[1])), fmaxf(fabsf(v[2]), fabsf(v[3])));
}
__global__ __launch_bounds__(kThreads) void maxabs_kernel(const float* __restrict__ x,
                                                          size_t n, size_t head,
                                                          unsigned* __restrict__ out) {
  constexpr int U = 16;
  float m = 0.0f;
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  // scalar head (until 16-byte alignment) and tail
  const size_t body = (n - head) / 4;
  const size_t tail0 = head + body * 4;
  if (tid < head) m = fabsf(x[tid]);
  if (tid < n - tail0) m = fmaxf(m, fabsf(x[tail0 + tid]));
  const f4_nt* __restrict__ x4 = reinterpret_cast<const f4_nt*>(x + head);
  const size_t per = (body + gridDim.x - 1) / gridDim.x;
  const size_t lo = (size_t)blockIdx.x * per;
  const size_t hi = lo + per < body ? lo + per : body;
  size_t i = lo + threadIdx.x;
  for (; i + (U - 1) * kThreads < hi; i += U * kThreads) {
    f4_nt v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(x4 + i + u * kThreads);
#pragma unroll
    for (int u = 0; u < U; ++u) m = fmaxf(m, abs4max(v[u]));
  }
  for (; i < hi; i += kThreads) m = fmaxf(m, abs4max(__builtin_nontemporal_load(x4 + i)));

  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  __shared__ float wave_max[kThreads / 64];
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float b = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
    // The result only grows, so a block whose maximum is not above what is already there
    // has nothing to add: most blocks skip the atomic (2048 of them on one address cost
    // 15 us of a 45 us launch).  The check reads past the caches.
    const unsigned bits = __float_as_uint(b);
    if (bits > __hip_atomic_load(out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
      atomicMax(out, bits);
  }
}

// ---------------------------------------------------------------- Q ---------------
__global__ __launch_bounds__(kThreads) void quantize_kernel(const float* __restrict__ r,
                                                            size_t n, size_t head, float q,
                                                            float lo, float hi,
                                                            int8_t* __restrict__ z) {
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  const size_t body = (n - head) / 4;
  const size_t tail0 = head + body * 4;
  if (tid < head) z[tid] = (int8_t)quant1(r[tid], q, lo, hi);
  if (tid < n - tail0) z[tail0 + tid] = (int8_t)quant1(r[tail0 + tid], q, lo, hi);
  const float4* __restrict__ r4 = reinterpret_cast<const float4*>(r + head);
  unsigned* __restrict__ z4 = reinterpret_cast<unsigned*>(z + head);
  size_t i = tid;
  for (; i + 3 * nthreads < body; i += 4 * nthreads) {
    float4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = r4[i + j * nthreads];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      z4[i + j * nthreads] = pack4(quant1(v[j].x, q, lo, hi), quant1(v[j].y, q, lo, hi),
                                   quant1(v[j].z, q, lo, hi), quant1(v[j].w, q, lo, hi));
  }
  for (; i < body; i += nthreads) {
    float4 v = r4[i];
    z4[i] = pack4(quant1(v.x, q, lo, hi), quant1(v.y, q, lo, hi), quant1(v.z, q, lo, hi),
                  quant1(v.w, q, lo, hi));
  }
}

// NHWC with the channel count padded from C to Cp (Cp == 4 and C <= 4): one thread
// per pixel, one packed 4-byte store.
__global__ __launch_bounds__(kThreads) void quantize_pad4_kernel(const float* __restrict__ r,
                                                                 size_t npix, int C, float q,
                                                                 float lo, float hi,
                                                                 unsigned* __restrict__ z) {
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  for (size_t p = (size_t)blockIdx.x * kThreads + threadIdx.x; p < npix; p += nthreads) {
    int v[4] = {0, 0, 0, 0};
    for (int c = 0; c < C; ++c) v[c] = quant1(r[p * C + c], q, lo, hi);
    z[p] = pack4(v[0], v[1], v[2], v[3]);
  }
}

// Image with a zero border: pixel (n, h, w) of an [N][H][W][C] fp32 tensor (C <= 4) goes to
// pixel (n, top + h, left + w) of an [N][Hs][Ws][4] int8 tensor.  blockIdx.y = n * H + h;
// a thread takes GROUP consecutive pixels of the row.  GROUP = 4 is the 3-channel case:
// three 16-byte loads (12 floats) and one 16-byte store, both only 4-byte aligned (the
// frame shifts the row start); the border is never written.
typedef float f4_a4 __attribute__((ext_vector_type(4), aligned(4)));
typedef unsigned u4_a4 __attribute__((ext_vector_type(4), aligned(4)));

template <int GROUP>
__global__ __launch_bounds__(kThreads) void quantize_image_kernel(const float* __restrict__ r,
                                                                  int n_rows, int H, int W, int C, int Hs,
                                                                  int Ws, int top, int left,
                                                                  float q, float lo, float hi,
                                                                  unsigned* __restrict__ z) {
  // one item = GROUP consecutive pixels of one image row; items are numbered through the
  // whole batch so that every wave is full whatever the row length
  const unsigned per_row = (unsigned)(W + GROUP - 1) / GROUP;
  const unsigned item = blockIdx.x * blockDim.x + threadIdx.x;
  const unsigned row = item / per_row;        // n * H + h
  if (row >= (unsigned)n_rows) return;
  const int w = (int)(item - row * per_row) * GROUP;
  const int n = (int)(row / (unsigned)H), h = (int)row - n * H;
  const float* src = r + ((size_t)row * W + w) * C;
  unsigned* dst = z + ((size_t)n * Hs + top + h) * Ws + left + w;
  if (GROUP == 4 && w + 4 <= W) {             // C == 3
    const f4_a4 a = *reinterpret_cast<const f4_a4*>(src);
    const f4_a4 b = *reinterpret_cast<const f4_a4*>(src + 4);
    const f4_a4 c = *reinterpret_cast<const f4_a4*>(src + 8);
    const float iq = __fdiv_rn(1.0f, q);
    auto Q = [&](float v) { return quant1_fast(v, q, iq, lo, hi); };
    u4_a4 o;
    o[0] = pack4(Q(a[0]), Q(a[1]), Q(a[2]), 0);
    o[1] = pack4(Q(a[3]), Q(b[0]), Q(b[1]), 0);
    o[2] = pack4(Q(b[2]), Q(b[3]), Q(c[0]), 0);
    o[3] = pack4(Q(c[1]), Q(c[2]), Q(c[3]), 0);
    *reinterpret_cast<u4_a4*>(dst) = o;
    return;
  }
  for (int g = 0; g < GROUP && w + g < W; ++g) {
    int v[4] = {0, 0, 0, 0};
    for (int c = 0; c < C; ++c) v[c] = quant1(src[g * C + c], q, lo, hi);
    dst[g] = pack4(v[0], v[1], v[2], v[3]);
  }
}

// The 3-channel image case: four pixels per thread = three aligned 16-byte loads (12
// floats) and one 16-byte store.  r 16-byte aligned, z 16-byte aligned, npix4 = npix / 4.
__global__ __launch_bounds__(kThreads) void quantize_rgb_pad4_kernel(const float4* __restrict__ r,
                                                                     size_t npix4, float q, float lo,
                                                                     float hi, uint4* __restrict__ z) {
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  for (size_t g = (size_t)blockIdx.x * kThreads + threadIdx.x; g < npix4; g += nthreads) {
    const float4 a = r[3 * g], b = r[3 * g + 1], c = r[3 * g + 2];
    uint4 o;
    o.x = pack4(quant1(a.x, q, lo, hi), quant1(a.y, q, lo, hi), quant1(a.z, q, lo, hi), 0);
    o.y = pack4(quant1(a.w, q, lo, hi), quant1(b.x, q, lo, hi), quant1(b.y, q, lo, hi), 0);
    o.z = pack4(quant1(b.z, q, lo, hi), quant1(b.w, q, lo, hi), quant1(c.x, q, lo, hi), 0);
    o.w = pack4(quant1(c.y, q, lo, hi), quant1(c.z, q, lo, hi), quant1(c.w, q, lo, hi), 0);
    z[g] = o;
  }
}

// General channel padding (any C <= Cp): one thread per output element.
__global__ __launch_bounds__(kThreads) void quantize_padc_kernel(const float* __restrict__ r,
                                                                 size_t npix, int C, int Cp,
                                                                 float q, float lo, float hi,
                                                                 int8_t* __restrict__ z) {
  const size_t total = npix * (size_t)Cp;
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += nthreads) {
    size_t p = i / Cp;
    int c = (int)(i - p * Cp);
    z[i] = c < C ? (int8_t)quant1(r[p * C + c], q, lo, hi) : (int8_t)0;
  }
}

// Eq. Q with p = 31 in fp64; the factor is the exact-in-fp64 product q_x * q_w.
__global__ __launch_bounds__(kThreads) void quantize_bias_kernel(const float* __restrict__ b,
                                                                 size_t n, double q,
                                                                 int32_t* __restrict__ z) {
  size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= n) return;
  double t = __ddiv_rn((double)b[i], q);
  t = rint(t);
  t = fmin(fmax(t, -2147483648.0), 2147483647.0);
  z[i] = (int32_t)t;
}

// ---------------------------------------------------------------- D ---------------
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const int8_t* __restrict__ z,
                                                              size_t n, size_t head, float q,
                                                              float* __restrict__ r) {
  const size_t tid = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  const size_t body = (n - head) / 4;
  const size_t tail0 = head + body * 4;
  if (tid < head) r[tid] = __fmul_rn(q, (float)z[tid]);
  if (tid < n - tail0) r[tail0 + tid] = __fmul_rn(q, (float)z[tail0 + tid]);
  const unsigned* __restrict__ z4 = reinterpret_cast<const unsigned*>(z + head);
  for (size_t i = tid; i < body; i += nthreads) {
    unsigned w = z4[i];
    float4 o;
    o.x = __fmul_rn(q, (float)(int8_t)(w & 0xff));
    o.y = __fmul_rn(q, (float)(int8_t)((w >> 8) & 0xff));
    o.z = __fmul_rn(q, (float)(int8_t)((w >> 16) & 0xff));
    o.w = __fmul_rn(q, (float)(int8_t)(w >> 24));
    // r + head need not be 16-byte aligned when z + head is 4-byte aligned: scalar stores
    float* dst = r + head + 4 * i;
    dst[0] = o.x; dst[1] = o.y; dst[2] = o.z; dst[3] = o.w;
  }
}

// One filter per workgroup: max |w| over the row, q = max / (2^p - 1) (1 for an all-zero
// row), then Eq. Q on the row with that factor.
__global__ __launch_bounds__(kThreads) void quantize_rows_kernel(const float* __restrict__ w,
                                                                 size_t row_len, float hi, float lo,
                                                                 float* __restrict__ q_out,
                                                                 int8_t* __restrict__ z) {
  const float* row = w + (size_t)blockIdx.x * row_len;
  float m = 0.0f;
  for (size_t i = threadIdx.x; i < row_len; i += kThreads) m = fmaxf(m, fabsf(row[i]));
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  __shared__ float wave_max[kThreads / 64];
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
  const float q = m > 0.0f ? __fdiv_rn(m, hi) : 1.0f;
  if (threadIdx.x == 0) q_out[blockIdx.x] = q;
  int8_t* zr = z + (size_t)blockIdx.x * row_len;
  for (size_t i = threadIdx.x; i < row_len; i += kThreads) zr[i] = (int8_t)quant1(row[i], q, lo, hi);
}

__global__ void quantize_bias_pc_kernel(const float* __restrict__ b, int K, double q_x,
                                        const float* __restrict__ q_w, int32_t* __restrict__ z) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= K) return;
  const double q = q_x * (double)q_w[k];
  double t = rint(__ddiv_rn((double)b[k], q));
  t = fmin(fmax(t, -2147483648.0), 2147483647.0);
  z[k] = (int32_t)t;
}

__global__ void requant_scales_kernel(float q_x, const float* __restrict__ q_w, int K, float q_out,
                                      float* __restrict__ m) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= K) return;
  const float prod = __fmul_rn(q_x, q_w[k]);      // the x rule: factor of the accumulator
  m[k] = __fdiv_rn(prod, q_out);
}

// Unsigned p = 8 codes (0..255) are kept as code - 128 in an int8 byte.
__global__ __launch_bounds__(kThreads) void quantize_u8_kernel(const float* __restrict__ r,
                                                               size_t n, float q,
                                                               int8_t* __restrict__ z) {
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += nthreads)
    z[i] = (int8_t)(quant1(r[i], q, 0.0f, 255.0f) - 128);
}

__global__ __launch_bounds__(kThreads) void dequantize_u8_kernel(const int8_t* __restrict__ z,
                                                                 size_t n, float q,
                                                                 float* __restrict__ r) {
  const size_t nthreads = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += nthreads)
    r[i] = __fmul_rn(q, (float)((int)z[i] + 128));
}

__global__ __launch_bounds__(kThreads) void dequantize_vec_kernel(const int8_t* __restrict__ z,
                                                                  size_t n4, float q,
                                                                  float4* __restrict__ r) {
  // every block owns one contiguous run of 4-code groups (see maxabs_kernel), four groups
  // per lane in flight
  constexpr int U = 4;
  const unsigned* __restrict__ z4 = reinterpret_cast<const unsigned*>(z);
  const size_t per = (n4 + gridDim.x - 1) / gridDim.x;
  const size_t lo = (size_t)blockIdx.x * per;
  const size_t hi = lo + per < n4 ? lo + per : n4;
  auto one = [&](size_t i, unsigned w) {
    float4 o;
    o.x = __fmul_rn(q, (float)(int8_t)(w & 0xff));
    o.y = __fmul_rn(q, (float)(int8_t)((w >> 8) & 0xff));
    o.z = __fmul_rn(q, (float)(int8_t)((w >> 16) & 0xff));
    o.w = __fmul_rn(q, (float)(int8_t)(w >> 24));
    r[i] = o;
  };
  size_t i = lo + threadIdx.x;
  for (; i + (U - 1) * kThreads < hi; i += U * kThreads) {
    unsigned w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) w[u] = z4[i + u * kThreads];
#pragma unroll
    for (int u = 0; u < U; ++u) one(i + u * kThreads, w[u]);
  }
  for (; i < hi; i += kThreads) one(i, z4[i]);
}

// ---------------------------------------------------------------- Eq. BN ----------
__global__ __launch_bounds__(kThreads) void fold_bn_kernel(
    const float* __restrict__ W, const float* __restrict__ b, const float* __restrict__ gamma,
    const float* __restrict__ beta, const float* __restrict__ mu, const float* __restrict__ var,
    float eps, int K, int RSC, float* __restrict__ W_out, float* __restrict__ b_out) {
  const int k = blockIdx.y;
  const float s = __fdiv_rn(gamma[k], sqrtf(__fadd_rn(var[k], eps)));
  const size_t row = (size_t)k * RSC;
  for (int j = blockIdx.x * kThreads + threadIdx.x; j < RSC; j += gridDim.x * kThreads)
    W_out[row + j] = __fmul_rn(s, W[row + j]);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    float bk = b ? b[k] : 0.0f;
    b_out[k] = __fadd_rn(__fmul_rn(s, __fsub_rn(bk, mu[k])), beta[k]);
  }
}

inline size_t head_elems(const void* p, size_t elem, size_t n) {
  size_t mis = reinterpret_cast<uintptr_t>(p) & 15;
  size_t h = mis ? (16 - mis) / elem : 0;
  return h < n ? h : n;
}

}  // namespace

extern "C" {

const char* q8_strerror(int code) {
  switch (code) {
    case Q8_OK: return "ok";
    case Q8_EINVAL: return "invalid argument (null pointer, bad size, q <= 0 or not finite, bad p)";
    case Q8_EUNSUPPORTED: return "shape not supported by the kernels";
    case Q8_EALIGN: return "pointer or channel stride not aligned as the call requires";
    case Q8_EHIP: return "HIP launch failed";
    case Q8_EWORKSPACE: return "workspace too small for this call";
    default: return "unknown q8conv error code";
  }
}

float q8_qfactor(float maxabs, int p) {
  if (!(maxabs > 0.0f) || p < 1 || p > 31) return 1.0f;
  volatile float levels = (float)(((int64_t)1 << p) - 1);
  volatile float q = maxabs / levels;
  return q;
}

float q8_sum_factor(float q1, float q2) { return q1 > q2 ? q1 : q2; }

int q8_calibrate_maxabs(const float* x_dev, size_t n, float* maxabs_dev, void* stream) {
  Q8_REQUIRE(maxabs_dev != nullptr, Q8_EINVAL);
  if (n == 0) return Q8_OK;
  Q8_REQUIRE(x_dev != nullptr, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(x_dev, 4) && q8_aligned(maxabs_dev, 4), Q8_EALIGN);
  size_t head = head_elems(x_dev, 4, n);
  int blocks = blocks_for((n + 15) / 16);
  hipLaunchKernelGGL(maxabs_kernel, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, x_dev, n,
                     head, reinterpret_cast<unsigned*>(maxabs_dev));
  return q8_launch_status();
}

int q8_quantize(const float* r_dev, size_t n, float q, int p, int8_t* z_dev, void* stream) {
  Q8_REQUIRE(p >= 1 && p <= 7 && q8_finite_pos(q), Q8_EINVAL);
  if (n == 0) return Q8_OK;
  Q8_REQUIRE(r_dev != nullptr && z_dev != nullptr, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(r_dev, 4), Q8_EALIGN);
  const float hi = (float)((1 << p) - 1), lo = -(float)(1 << p);
  // the vector body needs r 16-byte and z 4-byte aligned at the same element
  size_t head = head_elems(r_dev, 4, n);
  if (!q8_aligned(z_dev + head, 4)) head = n;   // fully scalar via the head/tail path
  if (head == n) {
    hipLaunchKernelGGL(quantize_padc_kernel, dim3(blocks_for(n)), dim3(kThreads), 0,
                       (hipStream_t)stream, r_dev, n, 1, 1, q, lo, hi, z_dev);
    return q8_launch_status();
  }
  int blocks = blocks_for((n + 15) / 16);
  hipLaunchKernelGGL(quantize_kernel, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, r_dev, n,
                     head, q, lo, hi, z_dev);
  return q8_launch_status();
}

int q8_quantize_pad_channels(const float* r_dev, size_t npix, int C, int C_pad, float q, int p,
                             int8_t* z_dev, void* stream) {
  Q8_REQUIRE(p >= 1 && p <= 7 && q8_finite_pos(q), Q8_EINVAL);
  Q8_REQUIRE(C >= 1 && C_pad >= C, Q8_EINVAL);
  if (npix == 0) return Q8_OK;
  Q8_REQUIRE(r_dev != nullptr && z_dev != nullptr, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(r_dev, 4), Q8_EALIGN);
  const float hi = (float)((1 << p) - 1), lo = -(float)(1 << p);
  if (C_pad == 4 && C == 3 && q8_aligned(z_dev, 16) && q8_aligned(r_dev, 16)) {
    const size_t npix4 = npix / 4, tail = npix - 4 * npix4;
    if (npix4)
      hipLaunchKernelGGL(quantize_rgb_pad4_kernel, dim3(blocks_for(npix4)), dim3(kThreads), 0,
                         (hipStream_t)stream, reinterpret_cast<const float4*>(r_dev), npix4, q, lo,
                         hi, reinterpret_cast<uint4*>(z_dev));
    if (tail)
      hipLaunchKernelGGL(quantize_pad4_kernel, dim3(1), dim3(kThreads), 0, (hipStream_t)stream,
                         r_dev + 12 * npix4, tail, C, q, lo, hi,
                         reinterpret_cast<unsigned*>(z_dev) + 4 * npix4);
  } else if (C_pad == 4 && q8_aligned(z_dev, 4)) {
    hipLaunchKernelGGL(quantize_pad4_kernel, dim3(blocks_for(npix)), dim3(kThreads), 0,
                       (hipStream_t)stream, r_dev, npix, C, q, lo, hi,
                       reinterpret_cast<unsigned*>(z_dev));
  } else {
    hipLaunchKernelGGL(quantize_padc_kernel, dim3(blocks_for(npix * (size_t)C_pad)), dim3(kThreads),
                       0, (hipStream_t)stream, r_dev, npix, C, C_pad, q, lo, hi, z_dev);
  }
  return q8_launch_status();
}

int q8_quantize_image(const float* r_dev, int N, int H, int W, int C, float q, int p,
                      int8_t* z_dev, int Hs, int Ws, int top, int left, void* stream) {
  Q8_REQUIRE(p >= 1 && p <= 7 && q8_finite_pos(q), Q8_EINVAL);
  Q8_REQUIRE(N >= 0 && H >= 1 && W >= 1 && C >= 1 && C <= 4, Q8_EINVAL);
  Q8_REQUIRE(top >= 0 && left >= 0 && Hs >= top + H && Ws >= left + W, Q8_EINVAL);
  if (N == 0) return Q8_OK;
  Q8_REQUIRE(r_dev != nullptr && z_dev != nullptr, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(r_dev, 4) && q8_aligned(z_dev, 4), Q8_EALIGN);
  const float hi = (float)((1 << p) - 1), lo = -(float)(1 << p);
  const int group = C == 3 ? 4 : 1;
  const long items = (long)N * H * ((W + group - 1) / group);
  Q8_REQUIRE(items < 0x7fffffffL, Q8_EUNSUPPORTED);             // 32-bit item numbers
  const dim3 grid((unsigned)((items + kThreads - 1) / kThreads));
  if (C == 3)
    hipLaunchKernelGGL(quantize_image_kernel<4>, grid, dim3(kThreads), 0, (hipStream_t)stream, r_dev,
                       N * H, H, W, C, Hs, Ws, top, left, q, lo, hi,
                       reinterpret_cast<unsigned*>(z_dev));
  else
    hipLaunchKernelGGL(quantize_image_kernel<1>, grid, dim3(kThreads), 0, (hipStream_t)stream, r_dev,
                       N * H, H, W, C, Hs, Ws, top, left, q, lo, hi,
                       reinterpret_cast<unsigned*>(z_dev));
  return q8_launch_status();
}

int q8_quantize_bias(const float* b_dev, size_t n, float q_x, float q_w, int32_t* z_b_dev,
                     void* stream) {
  Q8_REQUIRE(q8_finite_pos(q_x) && q8_finite_pos(q_w), Q8_EINVAL);
  if (n == 0) return Q8_OK;
  Q8_REQUIRE(b_dev != nullptr && z_b_dev != nullptr, Q8_EINVAL);
  const double q = (double)q_x * (double)q_w;
  Q8_REQUIRE(q > 0.0, Q8_EINVAL);
  hipLaunchKernelGGL(quantize_bias_kernel, dim3((unsigned)((n + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, (hipStream_t)stream, b_dev, n, q, z_b_dev);
  return q8_launch_status();
}

int q8_dequantize(const int8_t* z_dev, size_t n, float q, float* r_dev, void* stream) {
  Q8_REQUIRE(q8_finite_pos(q), Q8_EINVAL);
  if (n == 0) return Q8_OK;
  Q8_REQUIRE(z_dev != nullptr && r_dev != nullptr, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(r_dev, 4), Q8_EALIGN);
  if (q8_aligned(z_dev, 4) && q8_aligned(r_dev, 16)) {
    size_t n4 = n / 4;
    if (n4)
      hipLaunchKernelGGL(dequantize_vec_kernel, dim3(blocks_for(n4 / 2 + 1)), dim3(kThreads), 0,
                         (hipStream_t)stream, z_dev, n4, q, reinterpret_cast<float4*>(r_dev));
    if (n & 3)   // ragged tail: the scalar path of the generic kernel (head = all)
      hipLaunchKernelGGL(dequantize_kernel, dim3(1), dim3(kThreads), 0, (hipStream_t)stream,
                         z_dev + 4 * n4, n & 3, n & 3, q, r_dev + 4 * n4);
    return q8_launch_status();
  }
  size_t mis = reinterpret_cast<uintptr_t>(z_dev) & 3;
  size_t head = mis ? 4 - mis : 0;
  if (head > n) head = n;
  hipLaunchKernelGGL(dequantize_kernel, dim3(blocks_for((n + 3) / 4)), dim3(kThreads), 0,
                     (hipStream_t)stream, z_dev, n, head, q, r_dev);
  return q8_launch_status();
}

int q8_quantize_weights_per_channel(const float* w_dev, int K, size_t row_len, int p,
                                    float* q_w_dev, int8_t* z_w_dev, void* stream) {
  Q8_REQUIRE(p >= 1 && p <= 7 && K >= 0, Q8_EINVAL);
  if (K == 0 || row_len == 0) return Q8_OK;
  Q8_REQUIRE(w_dev != nullptr && q_w_dev != nullptr && z_w_dev != nullptr, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(w_dev, 4) && q8_aligned(q_w_dev, 4), Q8_EALIGN);
  hipLaunchKernelGGL(quantize_rows_kernel, dim3(K), dim3(kThreads), 0, (hipStream_t)stream, w_dev,
                     row_len, (float)((1 << p) - 1), -(float)(1 << p), q_w_dev, z_w_dev);
  return q8_launch_status();
}

int q8_quantize_bias_per_channel(const float* b_dev, int K, float q_x, const float* q_w_dev,
                                 int32_t* z_b_dev, void* stream) {
  Q8_REQUIRE(q8_finite_pos(q_x) && K >= 0, Q8_EINVAL);
  if (K == 0) return Q8_OK;
  Q8_REQUIRE(b_dev != nullptr && q_w_dev != nullptr && z_b_dev != nullptr, Q8_EINVAL);
  hipLaunchKernelGGL(quantize_bias_pc_kernel, dim3((K + kThreads - 1) / kThreads), dim3(kThreads), 0,
                     (hipStream_t)stream, b_dev, K, (double)q_x, q_w_dev, z_b_dev);
  return q8_launch_status();
}

int q8_requant_scales(float q_x, const float* q_w_dev, int K, float q_out, float* m_dev,
                      void* stream) {
  Q8_REQUIRE(q8_finite_pos(q_x) && q8_finite_pos(q_out) && K >= 0, Q8_EINVAL);
  if (K == 0) return Q8_OK;
  Q8_REQUIRE(q_w_dev != nullptr && m_dev != nullptr, Q8_EINVAL);
  hipLaunchKernelGGL(requant_scales_kernel, dim3((K + kThreads - 1) / kThreads), dim3(kThreads), 0,
                     (hipStream_t)stream, q_x, q_w_dev, K, q_out, m_dev);
  return q8_launch_status();
}

int q8_quantize_u8(const float* r_dev, size_t n, float q, int8_t* z_dev, void* stream) {
  Q8_REQUIRE(q8_finite_pos(q), Q8_EINVAL);
  if (n == 0) return Q8_OK;
  Q8_REQUIRE(r_dev != nullptr && z_dev != nullptr, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(r_dev, 4), Q8_EALIGN);
  hipLaunchKernelGGL(quantize_u8_kernel, dim3(blocks_for(n)), dim3(kThreads), 0,
                     (hipStream_t)stream, r_dev, n, q, z_dev);
  return q8_launch_status();
}

int q8_dequantize_u8(const int8_t* z_dev, size_t n, float q, float* r_dev, void* stream) {
  Q8_REQUIRE(q8_finite_pos(q), Q8_EINVAL);
  if (n == 0) return Q8_OK;
  Q8_REQUIRE(z_dev != nullptr && r_dev != nullptr, Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(r_dev, 4), Q8_EALIGN);
  hipLaunchKernelGGL(dequantize_u8_kernel, dim3(blocks_for(n)), dim3(kThreads), 0,
                     (hipStream_t)stream, z_dev, n, q, r_dev);
  return q8_launch_status();
}

int q8_fold_bn(const float* W_dev, const float* b_dev, const float* gamma_dev,
               const float* beta_dev, const float* mu_dev, const float* var_dev, float eps, int K,
               int RSC, float* W_out_dev, float* b_out_dev, void* stream) {
  Q8_REQUIRE(K >= 0 && RSC >= 0 && eps >= 0.0f, Q8_EINVAL);
  if (K == 0) return Q8_OK;
  Q8_REQUIRE(K <= 65535, Q8_EUNSUPPORTED);
  Q8_REQUIRE(gamma_dev && beta_dev && mu_dev && var_dev && b_out_dev, Q8_EINVAL);
  Q8_REQUIRE(RSC == 0 || (W_dev && W_out_dev), Q8_EINVAL);
  int bx = (RSC + kThreads * 4 - 1) / (kThreads * 4);
  if (bx < 1) bx = 1;
  hipLaunchKernelGGL(fold_bn_kernel, dim3(bx, K), dim3(kThreads), 0, (hipStream_t)stream, W_dev,
                     b_dev, gamma_dev, beta_dev, mu_dev, var_dev, eps, K, RSC, W_out_dev, b_out_dev);
  return q8_launch_status();
}

}  // extern "C"
