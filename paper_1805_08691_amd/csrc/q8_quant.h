// Eq. Q of arxiv 1805.08691 on one value, as device code: z = clamp(Round(r / q), lo, hi) with a
// true fp32 division and round-half-to-even.  Shared by the stand-alone quantisation kernels
// and the first-layer kernel that quantises the image while it loads it.
#pragma once
#include <hip/hip_runtime.h>

namespace q8 {

__device__ __forceinline__ int quant1(float r, float q, float lo, float hi) {
  float t = __fdiv_rn(r, q);
  t = rintf(t);                       // round-half-to-even
  t = fminf(fmaxf(t, lo), hi);
  return (int)t;
}

// The same code as quant1 for less arithmetic: Round(r/q) only depends on the correctly rounded
// quotient when r/q lies next to a tie k + 1/2.  t = r * inv_q (inv_q = fl(1/q)) is within
// 1.2e-7 |t| of r/q and fl(r/q) within 6e-8 |t|; if t is further than 4.8e-7 |t| from every
// tie, Round(t) = Round(fl(r/q)).  Otherwise (a few elements in 10^5) the division is done.
__device__ __forceinline__ int quant1_fast(float r, float q, float inv_q, float lo, float hi) {
  const float t = __fmul_rn(r, inv_q);
  float k = rintf(t);
  const float d = fabsf(__fsub_rn(t, k));                 // distance to the nearest integer
  if (fabsf(__fsub_rn(d, 0.5f)) <= __fmul_rn(fabsf(t), 4.8e-7f)) k = rintf(__fdiv_rn(r, q));
  return (int)fminf(fmaxf(k, lo), hi);
}

__device__ __forceinline__ unsigned pack4(int a, int b, int c, int d) {
  return (unsigned)(a & 0xff) | ((unsigned)(b & 0xff) << 8) | ((unsigned)(c & 0xff) << 16) |
         ((unsigned)(d & 0xff) << 24);
}

}  // namespace q8
