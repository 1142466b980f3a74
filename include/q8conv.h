/*
 * q8conv -- int8 quantised convolution for MI355X (gfx950), C ABI.
 *
 * The calls follow the statement of 8-bit inference in arxiv 1805.08691
 * ("8-bit Low Precision Inference" and "Model Optimization" sections):
 *   Eq. Q   z = max(min(Round(r/q), 2^p-1), -2^p), Round = round-half-to-even
 *   Eq. D   r' = q z
 *   Eq. x   (z1 x z2, q1 q2): integer contraction, the factor is the product
 *   Eq. +   Q_p(D(z1) + D(z2), max(q1, q2))
 *   Eq. A'  y_q = Q(ReLU(D(Q(W) x z + Q_31(b)))) -- the quantised layer
 *   Eq. BN  w' = gamma/sqrt(var+eps) w,  b' = gamma/sqrt(var+eps) (b - mu) + beta
 *   calibration: q = max|tensor| / (2^p - 1), one factor per tensor.
 *
 * Conventions common to every call
 *   - Every pointer named *_dev, z_*, residual, acc_dump, packed is DEVICE memory
 *     owned by the caller.  The library never allocates, frees or keeps pointers,
 *     and holds no state between calls, so calls on different streams are
 *     independent.  (One exception, stated where it is declared: the fixed workspace
 *     of q8_conv_chain_int8_static.)
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on that stream and return at once.
 *   - Descriptors (q8_conv_desc) are HOST memory and are read before return.
 *   - Activations are NHWC, weights KRSC (K output channels, R x S taps, C input
 *     channels), both dense unless a *_c_stride says otherwise.
 *   - Return value: Q8_OK (0) or a negative Q8_E* code; q8_strerror names it.
 *     All argument checks run on the host before anything is launched, so a
 *     rejected call has touched no device memory.
 *   - Floating point is IEEE binary32 round-to-nearest-even with no fused
 *     multiply-add; the int8 results are therefore a pure function of the inputs.
 */
#ifndef Q8CONV_H
#define Q8CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  Q8_OK = 0,
  Q8_EINVAL = -1,       /* null pointer, negative size, q <= 0 or not finite, bad p   */
  Q8_EUNSUPPORTED = -2, /* a shape the kernels cannot take (see q8_conv_int8)         */
  Q8_EALIGN = -3,       /* pointer or channel-stride alignment (see each call)        */
  Q8_EHIP = -4,         /* the HIP runtime refused a launch                            */
  Q8_EWORKSPACE = -5    /* the workspace passed in is smaller than the call needs      */
};

const char *q8_strerror(int code);

/* Geometry of one convolution layer and of the tensors it touches. */
typedef struct q8_conv_desc {
  int32_t N, H, W, C;     /* input: batch, height, width, channels                   */
  int32_t K, R, S;        /* output channels, filter height, filter width            */
  int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
  int32_t relu;           /* 0/1: max(.,0) after the residual sum, before Round      */
  int32_t in_c_stride;    /* elements between pixels of z_x   (>= C; 0 means C)      */
  int32_t out_c_stride;   /* elements between pixels of z_y   (>= K; 0 means K)      */
  int32_t out_c_off;      /* first channel written inside a wider (concat) tensor    */
  int32_t res_c_stride;   /* same two for the residual tensor (0 means K)            */
  int32_t res_c_off;
} q8_conv_desc;

/* Output extent floor((in + 2 pad - dil (k-1) - 1) / stride) + 1, 0 if negative. */
int q8_conv_out_h(const q8_conv_desc *d);
int q8_conv_out_w(const q8_conv_desc *d);

/* Calibration (text after Eq. +/x): *maxabs_dev = max(*maxabs_dev, max_i |x_i|).
 * The caller zeroes *maxabs_dev once; calling it for every calibration batch leaves
 * the running maximum.  NaNs are ignored.  n may be 0.  x_dev 4-byte aligned.      */
int q8_calibrate_maxabs(const float *x_dev, size_t n, float *maxabs_dev, void *stream);

/* Host helper: q = maxabs / (2^p - 1) in fp32; an all-zero tensor gets q = 1.      */
float q8_qfactor(float maxabs, int p);

/* Host helper, Eq. +: the factor of the sum of two quantised tensors, max(q1, q2).
 * For a sum fused into a convolution q1 is the factor of the branch's own output
 * before the sum and q2 that of the residual; the result is the layer's q_out.    */
float q8_sum_factor(float q1, float q2);

/* Eq. Q for 1 <= p <= 7: n fp32 values -> n int8 codes.  True fp32 division.       */
int q8_quantize(const float *r_dev, size_t n, float q, int p, int8_t *z_dev,
                void *stream);

/* Eq. Q on an NHWC tensor whose channel count grows from C to C_pad (zeros in the
 * added channels): npix*C fp32 -> npix*C_pad int8.  Used for the 3-channel image.  */
int q8_quantize_pad_channels(const float *r_dev, size_t npix, int C, int C_pad,
                             float q, int p, int8_t *z_dev, void *stream);

/* Eq. Q on an image of C <= 4 channels, stored as 4 int8 channels (zeros in the added
 * ones) inside a larger zero frame: pixel (n, h, w) of the [N][H][W][C] fp32 tensor goes
 * to pixel (n, top + h, left + w) of the [N][Hs][Ws][4] int8 tensor z_dev.  Only the
 * H x W interior is written: the caller zeroes z_dev once and the frame stays zero.  With
 * the padding of the first convolution stored in the frame, that layer runs without
 * padding (the zeros Eq. A' reads outside the image are then real bytes).
 * Q8_EINVAL if the interior does not fit the frame.                                      */
int q8_quantize_image(const float *r_dev, int N, int H, int W, int C, float q, int p,
                      int8_t *z_dev, int Hs, int Ws, int top, int left, void *stream);

/* Eq. Q with p = 31 for the bias of Eq. A': z_b = clamp(Round(b / (q_x q_w))), the
 * factor being that of the accumulator (Eq. x).  Evaluated in fp64.               */
int q8_quantize_bias(const float *b_dev, size_t n, float q_x, float q_w,
                     int32_t *z_b_dev, void *stream);

/* Eq. D: n int8 codes -> n fp32 values q*z.                                        */
int q8_dequantize(const int8_t *z_dev, size_t n, float q, float *r_dev, void *stream);

/* Eq. BN.  W_dev is [K][RSC]; b_dev may be NULL (zero bias); var is the variance.
 * W_out_dev may alias W_dev.  Op order: s = gamma / sqrt(var + eps); w' = s*w;
 * b' = (s * (b - mu)) + beta.                                                      */
int q8_fold_bn(const float *W_dev, const float *b_dev, const float *gamma_dev,
               const float *beta_dev, const float *mu_dev, const float *var_dev,
               float eps, int K, int RSC, float *W_out_dev, float *b_out_dev,
               void *stream);

/* Filter pre-pack.  q8_conv_int8 reads its filters in a layout private to the
 * library; q8_pack_weights converts dense KRSC int8 into it (d->C, K, R, S are
 * used).  q8_packed_weight_bytes gives the size of `packed_dev` (16-byte aligned). */
size_t q8_packed_weight_bytes(const q8_conv_desc *d);
int q8_pack_weights(const q8_conv_desc *d, const int8_t *z_w_krsc_dev, void *packed_dev,
                    void *stream);

/* Eq. A' with the fused element-wise sum of the "Model Optimization" section:
 *   acc[n,ho,wo,k] = bias_i32[k] + sum_{r,s,c} z_x[n,hi,wi,c] * z_w[k,r,s,c]
 *                    (hi = ho*stride_h - pad_h + r*dil_h, zero outside the image)
 *   t = fp32(acc) * m                         m   = (q_x * q_w) / q_out
 *   t = t + fp32(residual) * m_r              m_r = q_res / q_out  (if residual)
 *   t = max(t, 0)                             (if d->relu)
 *   z_y = int8(Round(clamp(t, -128, 127)))
 * The caller passes q_out = max(q1, q_res) for a fused sum (Eq. +).
 *   z_x        int8 [N][H][W][in_c_stride]; in_c_stride % 4 == 0, 4-byte aligned;
 *              d->C must match the C the filters were packed with.  C % 16 == 0 and
 *              in_c_stride % 16 == 0 with a 16-byte aligned pointer take the fast
 *              path; C == 4 (a padded 3-channel image) is supported for any R, S.
 *   bias_i32   [K] or NULL.
 *   residual   int8 [N][Ho][Wo][res_c_stride] or NULL.
 *   z_y        int8 [N][Ho][Wo][out_c_stride], written at channel out_c_off.
 *   acc_dump   NULL, or dense int32 [N][Ho][Wo][K] that receives acc (tests).
 *   workspace  NULL, or device memory of at least q8_conv_workspace_bytes(d) bytes, 256-byte
 *              aligned, owned by the caller.  With a workspace the library may split the
 *              reduction over r, s, c of a layer with few output tiles among several
 *              workgroups (Eq. x: acc is an integer sum, so every grouping of its terms
 *              gives the same bits; the results do not depend on whether, or how, the
 *              reduction is split).  The caller zeroes the workspace once after allocating
 *              it; every call leaves its counters zero again, so one workspace serves any
 *              number of calls that do not overlap in time.  Q8_EWORKSPACE if it is
 *              smaller than q8_conv_workspace_bytes(d); without one nothing is split.
 * Accumulation wraps modulo 2^32 (cannot happen below R*S*C = 130 000).           */
int q8_conv_int8(const q8_conv_desc *d, const int8_t *z_x, const void *z_w_packed,
                 const int32_t *bias_i32, float q_x, float q_w, float q_out,
                 const int8_t *residual, float q_res, int8_t *z_y, int32_t *acc_dump,
                 void *workspace, size_t workspace_bytes, void *stream);

/* Bytes of workspace with which q8_conv_int8 splits this layer's reduction; 0 for a layer it
 * would not split (then the workspace argument is ignored).                              */
size_t q8_conv_workspace_bytes(const q8_conv_desc *d);

/* ---- unsigned activations: the calibration paragraph's p = 8 for non-negative tensors --
 * An unsigned tensor (the output of a ReLU layer) holds codes 0..255 with q = max/255, one
 * more bit than the signed p = 7 form.  The matrix instruction multiplies signed bytes, so
 * a code is STORED as code - 128 (= code XOR 0x80) in an int8 byte; everything below
 * reads and writes that form.
 *
 * q8_quantize_u8 / q8_dequantize_u8: Eq. Q with p = 8 clamped to [0, 255] (the tensor is
 * non-negative) and Eq. D, on the stored form.
 *
 * q8_u8_prepare: for a layer that READS an unsigned tensor, from the dense KRSC int8
 * filters and the int32 bias (or NULL).  Since sum z_x z_w = sum (z_x - 128) z_w
 * + 128 * sum z_w, the signed contraction of the stored bytes started at
 * bias_eff[k] = bias[k] + 128 * (sum of filter k) equals Eq. A' on the codes wherever every
 * tap reads inside the image.  Near the border the taps inside the image are a rectangle
 * [r_lo, r_hi) x [s_lo, s_hi) of the filter, and the accumulator has to start at the bias
 * plus 128 times the sum over that rectangle only: start_dev, int32
 * [((R+1)*(S+1))^2][K], holds that value for every rectangle,
 *   start[idx*K + k], idx = ((r_lo*(R+1) + r_hi)*(S+1) + s_lo)*(S+1) + s_hi,
 * and the kernel loads a pixel's accumulators from its rectangle's row.  16-byte aligned.
 *
 * q8_conv_u8: q8_conv_int8 where the input, the output and the residual may each be an
 * unsigned tensor (flags).  in_unsigned: pass bias_eff as the bias, and the start table if
 * the layer has padding (else it may be NULL).  out_unsigned needs d->relu; the output is
 * clamped to [0, 255].  acc_dump receives the accumulators of Eq. A' on the codes.
 * Main-kernel geometries only (C % 16 == 0, K > 32, R*S <= 32): Q8_EUNSUPPORTED otherwise. */
int q8_quantize_u8(const float *r_dev, size_t n, float q, int8_t *z_dev, void *stream);
int q8_dequantize_u8(const int8_t *z_dev, size_t n, float q, float *r_dev, void *stream);
int q8_u8_prepare(const q8_conv_desc *d, const int8_t *z_w_krsc_dev, const int32_t *bias_i32,
                  int32_t *start_dev, int32_t *bias_eff_dev, void *stream);
int q8_conv_u8(const q8_conv_desc *d, int in_unsigned, int out_unsigned, int res_unsigned,
               const int8_t *z_x, const void *z_w_packed, const int32_t *bias_eff,
               const int32_t *start_table, float q_x, float q_w, float q_out,
               const int8_t *residual, float q_res, int8_t *z_y, int32_t *acc_dump,
               void *stream);

/* ---- per-output-channel weight factors ------------------------------------------------
 * A finer granularity than the calibration paragraph's one factor per tensor: filter k gets
 * q_w[k] = max|w'[k]| / (2^p - 1).  By Eq. x the accumulator of channel k then carries
 * q_x * q_w[k], the bias is Q_31(b[k], q_x q_w[k]) and the tail of Eq. A' uses the scale
 * m[k] = (q_x * q_w[k]) / q_out (two fp32 operations, as for the single scale).
 *
 * q8_quantize_weights_per_channel: W fp32 [K][row_len] (KRSC) -> q_w_dev fp32 [K] and int8
 *   codes of the same shape (Eq. Q per row; an all-zero row gets q = 1).
 * q8_quantize_bias_per_channel: z_b[k] = Q_31(b[k], q_x * q_w[k]) in fp64.
 * q8_requant_scales: m_dev[k] = (q_x * q_w[k]) / q_out.
 * q8_conv_int8_per_channel: q8_conv_int8 with m_dev (fp32 [K], 16-byte aligned) in place of
 *   q_x and q_w.  Main-kernel geometries only; not combined with unsigned activations.   */
int q8_quantize_weights_per_channel(const float *w_dev, int K, size_t row_len, int p,
                                    float *q_w_dev, int8_t *z_w_dev, void *stream);
int q8_quantize_bias_per_channel(const float *b_dev, int K, float q_x, const float *q_w_dev,
                                 int32_t *z_b_dev, void *stream);
int q8_requant_scales(float q_x, const float *q_w_dev, int K, float q_out, float *m_dev,
                      void *stream);
int q8_conv_int8_per_channel(const q8_conv_desc *d, const int8_t *z_x, const void *z_w_packed,
                             const int32_t *bias_i32, const float *m_dev, float q_out,
                             const int8_t *residual, float q_res, int8_t *z_y,
                             int32_t *acc_dump, void *stream);

/* A layer whose output leaves the quantised domain (the last layer before a
 * floating-point consumer, a detection head): the first half of Eq. A' only,
 *   y' = ReLU(D(acc) [+ D(z_res)])   (Eq. D at the accumulator's factor q_x*q_w of Eq. x),
 * written as fp32 with no Q afterwards, which saves the separate q8_dequantize pass and the
 * rounding to 8 bits.  Fixed fp32 order: s = q_x*q_w; t = fp32(acc)*s; with a residual
 * t = t + fp32(z_res)*q_res (separate multiply and add); ReLU if d->relu.
 * y_dev: fp32 [N][Ho][Wo][out_c_stride] (0 = K), channels [out_c_off, out_c_off + K),
 * 4-byte aligned (16-byte aligned with strides % 4 == 0 for vector stores).  Other
 * arguments, layouts and error codes as q8_conv_int8.                                   */
int q8_conv_int8_real_output(const q8_conv_desc *d, const int8_t *z_x, const void *z_w_packed,
                             const int32_t *bias_i32, float q_x, float q_w,
                             const int8_t *residual, float q_res, float *y_dev, void *stream);

/* Two layers in one launch: a convolution (d1; ReLU per d1->relu, no residual) whose output
 * is read by one 1x1 layer (d2: stride 1, no padding, C = d1->K) and by nothing else -- the
 * 3x3 -> 1x1 tail of a bottleneck block.  Each layer is Eq. A' as in q8_conv_int8 (the
 * second may carry the fused sum and ReLU of the "Model Optimization" section); the
 * intermediate int8 codes at factor q_mid never leave the chip.  Results are bit-identical
 * to two q8_conv_int8 calls with the same factors.
 * Supported (q8_conv_pair_supported returns 1): d1 takes the main kernel with C % 64 == 0,
 * d1->K is 64 or 128, d2->K % d1->K == 0, d2 spans exactly d1's output.  d1's out_* / res_*
 * fields are ignored; d2's describe z_y and the residual.  w2_packed: [K2][K1] int8
 * (q8_pack_weights of d2), bias2 at q_mid*q_w2.  Otherwise Q8_EUNSUPPORTED: call the two
 * layers one after the other.                                                           */
int q8_conv_pair_supported(const q8_conv_desc *d1, const q8_conv_desc *d2);
int q8_conv_pair_int8(const q8_conv_desc *d1, const int8_t *z_x, const void *w1_packed,
                      const int32_t *bias1, float q_x, float q_w1, float q_mid,
                      const q8_conv_desc *d2, const void *w2_packed, const int32_t *bias2,
                      float q_w2, float q_out, const int8_t *residual, float q_res,
                      int8_t *z_y, void *stream);

/* Two layers that do not depend on each other (typically the projection branch and the first
 * 1x1 of a residual stage, which read the same tensor) in ONE launch: each is Eq. A' exactly
 * as q8_conv_int8 computes it, arguments as there, results bit-identical to two calls.  Saves
 * one launch boundary on the critical path.  Supported (q8_conv_dual_supported returns 1):
 * both layers have C % 64 == 0, K > 32 and at most 32 taps, and their sizes map to one of
 * the tile-shape pairs the library was built with; otherwise Q8_EUNSUPPORTED (call the two
 * layers one after the other).  The outputs must be distinct tensors that neither layer
 * reads.                                                                                  */
int q8_conv_dual_supported(const q8_conv_desc *d1, const q8_conv_desc *d2);
int q8_conv_dual_int8(const q8_conv_desc *d1, const int8_t *z_x1, const void *w1_packed,
                      const int32_t *bias1, float q_x1, float q_w1, float q_out1,
                      const int8_t *residual1, float q_res1, int8_t *z_y1,
                      const q8_conv_desc *d2, const int8_t *z_x2, const void *w2_packed,
                      const int32_t *bias2, float q_x2, float q_w2, float q_out2,
                      const int8_t *residual2, float q_res2, int8_t *z_y2, void *stream);

/* ---- a list of layers in one launch (cross-layer fusion, "Model Optimization" section) --
 * q8_conv_chain_int8 runs a list of convolution layers, each one Eq. A' exactly as
 * q8_conv_int8 computes it (bias, scale, fused residual sum of Eq. +, ReLU, Round, clamp, one
 * int8 store), as ONE persistent launch instead of one launch per layer; the results are
 * bit-identical to calling q8_conv_int8 layer by layer.  The batch is split into eight groups
 * of images, one per XCD of the chip; output tiles are queued per XCD in layer order and a
 * tile starts as soon as the tiles producing the pixels it reads have finished, so there is
 * no launch boundary and no chip-wide barrier between layers.
 *
 * q8_chain_layer (HOST memory): the arguments of q8_conv_int8 for one layer, plus
 *   src_layer / res_layer   index (smaller than the layer's own) of the layer of this list
 *                           whose z_y is this layer's z_x / residual, or -1 if that tensor
 *                           was written before the call;
 *   variant                 -1, or a tile variant 0..3 (128x128, 128x64, 64x128, 64x64
 *                           pixels x channels) to force for this layer (tests, tuning).
 * Supported layers (q8_conv_chain_supported): C % 64 == 0, K > 32, R*S <= 32, dense tensors
 * (no channel strides or offsets); every z_y of the list is a distinct tensor that no layer
 * reads from outside the list; all layers share N.  Otherwise Q8_EUNSUPPORTED / Q8_EINVAL.
 *
 * Use: plan_host = malloc(q8_conv_chain_plan_bytes(...)); q8_conv_chain_plan fills it (host
 * work only; it holds the device pointers and factors of the list, so it is rebuilt when
 * those change); the caller copies the same bytes to DEVICE memory (plan_dev, 256-byte
 * aligned) and provides q8_conv_chain_workspace_bytes(plan_host) bytes of device workspace
 * (16-byte aligned; completion counters and queue heads, cleared by the call itself).
 * q8_conv_chain_int8 then enqueues the clear and the launch on `stream`; it may be called any
 * number of times with the same plan (also inside a stream capture).  Two calls that share
 * a workspace must not overlap in time.
 * After the stream has drained, word 0 of the workspace (int32) is 0 if every tile found its
 * inputs; 1 means a tile gave up waiting (the outputs are then invalid; cannot happen
 * unless the launch was starved of its workgroups for about a second); 2 means the chip
 * reported an XCD number above 7.                                                      */
typedef struct q8_chain_layer {
  q8_conv_desc d;
  const int8_t *z_x;
  const void *z_w_packed;
  const int32_t *bias_i32;
  float q_x, q_w, q_out;
  const int8_t *residual;
  float q_res;
  int8_t *z_y;
  int32_t src_layer, res_layer, variant;
} q8_chain_layer;
int q8_conv_chain_supported(const q8_conv_desc *d);
size_t q8_conv_chain_plan_bytes(const q8_chain_layer *layers, int n_layers);
int q8_conv_chain_plan(const q8_chain_layer *layers, int n_layers, void *plan_host,
                       size_t plan_bytes);
size_t q8_conv_chain_workspace_bytes(const void *plan_host);
int q8_conv_chain_int8(const void *plan_host, const void *plan_dev, void *workspace_dev,
                       size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory for the workspace (code under HIP graph
 * capture that has nothing preallocated, tight serving loops, harnesses that forbid
 * hipMalloc): q8_conv_chain_int8 with the workspace taken from a fixed array inside the
 * library's own device image, q8_conv_chain_static_workspace_limit() bytes (1 MiB) per GPU,
 * held from the moment the library is loaded until the process ends.  The call allocates and
 * frees nothing; a plan whose workspace is larger is refused with Q8_EWORKSPACE (use
 * q8_conv_chain_int8).  Same results as q8_conv_chain_int8.  Every call on one GPU shares
 * that GPU's array (the call clears what it uses first): two such calls must not overlap in
 * time on one GPU, whatever their streams.  q8_conv_chain_static_status copies the status
 * word (see above) of the current device's array to host memory; it synchronises.       */
size_t q8_conv_chain_static_workspace_limit(void);
int q8_conv_chain_int8_static(const void *plan_host, const void *plan_dev, void *stream);
int q8_conv_chain_static_status(int32_t *status_host);

/* Name of the kernel variant (tile shape) q8_conv_int8 picks for this geometry, as it
 * appears in a profiler's kernel trace; "unsupported" if the call would be rejected.
 * For measurement code that groups launches by kernel.                              */
const char *q8_conv_variant(const q8_conv_desc *d);

/* q8_conv_int8 that also applies Eq. D to its own output in the same launch, for a layer whose
 * output leaves the quantised domain as fp32 AND is kept as codes: besides z_y it writes
 *   r_y[i] = q_out * fp32(z_y[i])      (one fp32 multiplication, the arithmetic of q8_dequantize)
 * for every element it writes of z_y, r_y being fp32 [N][Ho][Wo][out_c_stride] laid out like
 * z_y (4-byte aligned; 16-byte aligned with strides % 4 == 0 for vector stores).  Saves the
 * separate pass over the tensor.  Signed codes only; other arguments and errors as
 * q8_conv_int8 (no accumulator dump, no workspace).                                        */
int q8_conv_int8_dequantized(const q8_conv_desc *d, const int8_t *z_x, const void *z_w_packed,
                             const int32_t *bias_i32, float q_x, float q_w, float q_out,
                             const int8_t *residual, float q_res, int8_t *z_y, float *r_y,
                             void *stream);

/* The head of a network as ONE launch: Eq. Q on the real-valued image, the first layer on the
 * codes (Eq. x / Eq. A' with bias, ReLU and requantisation as q8_conv_int8) and, with pool = 1,
 * the 3x3 / stride 2 / padding 1 max-pool behind it (the maximum of codes, which keeps q_out).
 * The result is, bit for bit, that of q8_quantize_image into a zero frame, q8_conv_int8 on the
 * frame and q8_maxpool_i8 on its output; the int8 image and, with pool = 1, the layer's own
 * output are never written to memory.
 *   d      the layer over the zero frame, as it would be given to q8_conv_int8 after
 *          q8_quantize_image: d->H x d->W the frame, no padding, d->C = C <= 4,
 *          in_c_stride 4 (or 0); out_c_stride / out_c_off place the output channels;
 *   r_dev  device, fp32 [N][H][W][C], 4-byte aligned; pixel (n, h, w) lies at pixel
 *          (top + h, left + w) of the frame, whose other pixels are zeros;
 *   q_x, p Eq. Q's factor and bit count (1 <= p <= 7);  z_w_packed, bias_i32, q_w, q_out as
 *          q8_conv_int8 (filters packed by q8_pack_weights for d);
 *   z_y    device, int8 [N][Ho][Wo][out_c_stride], or with pool = 1
 *          [N][(Ho-1)/2+1][(Wo-1)/2+1][out_c_stride]; 16-byte aligned, strides % 16 == 0.
 * Layers taken: 5 .. 8 filter columns, at most 8 filter rows, stride 1 or 2 (pool: vertical
 * stride 2), K <= 64 with K % 16 == 0, output rows of at most 128 pixels, frames at most 240
 * pixels wide.  Q8_EUNSUPPORTED otherwise (q8_conv_image_f32_supported says so beforehand:
 * 1 / 0); the caller then makes the three calls.  Q8_EINVAL for an image that does not fit
 * the frame or C != d->C, Q8_EALIGN as q8_conv_int8.                                       */
int q8_conv_image_f32_supported(const q8_conv_desc *d, int H, int W, int C, int top, int left,
                                int pool);
int q8_conv_image_f32_int8(const q8_conv_desc *d, const float *r_dev, int H, int W, int C,
                           int top, int left, float q_x, int p, const void *z_w_packed,
                           const int32_t *bias_i32, float q_w, float q_out, int pool,
                           int8_t *z_y, void *stream);

/* Tests and tuning only: q8_conv_int8 with the tile / ring variant of the main kernel given
 * by the caller (0 .. q8_conv_num_variants() - 1, in the order of the library's variant
 * table; -1 = automatic choice, i.e. q8_conv_int8 itself).  The variant is used wherever the
 * main kernel can take the geometry (C % 16 == 0, R*S <= 32) and ignored otherwise.  With a
 * split-reduction variant, n_split >= 2 workgroups share each output tile (clipped to the
 * number of 64-byte reduction steps; the layer must have C % 64 == 0) and the workspace holds
 * at least q8_conv_workspace_bytes_variant(d, variant, n_split) bytes; n_split < 2, or a layer
 * such a variant cannot take, runs unsplit.  The results are identical for every variant
 * and every split factor.                                                                */
int q8_conv_num_variants(void);
const char *q8_conv_variant_name(int variant);   /* as in a profiler's kernel trace */
size_t q8_conv_workspace_bytes_variant(const q8_conv_desc *d, int variant, int n_split);
int q8_conv_int8_variant(const q8_conv_desc *d, const int8_t *z_x, const void *z_w_packed,
                         const int32_t *bias_i32, float q_x, float q_w, float q_out,
                         const int8_t *residual, float q_res, int8_t *z_y, int32_t *acc_dump,
                         int variant, int n_split, void *workspace, size_t workspace_bytes,
                         void *stream);

/* ---- helpers that only chain layers; not part of the paper's method ------------ */

/* fp32 NHWC convolution + bias (+ dense residual) (+ ReLU), used to produce the
 * real-valued activations that calibration measures.  Dense tensors, weights KRSC. */
int q8_conv_f32_ref(const q8_conv_desc *d, const float *x_dev, const float *w_dev,
                    const float *b_dev, const float *res_dev, float *y_dev,
                    void *stream);

/* int8 max-pool over an R x S window; taps outside the image are ignored.         */
int q8_maxpool_i8(const int8_t *x_dev, int N, int H, int W, int C, int R, int S,
                  int stride, int pad, int Ho, int Wo, int8_t *y_dev, void *stream);
/* The same on fp32 (calibration forward).                                          */
int q8_maxpool_f32(const float *x_dev, int N, int H, int W, int C, int R, int S,
                   int stride, int pad, int Ho, int Wo, float *y_dev, void *stream);

/* General int8 pooling into channels [out_c_off, out_c_off + C) of a tensor with pixel
 * stride out_c_stride, with a change of quantisation factor.  mode 0: v = max over the taps
 * inside the image, t = fp32(v).  mode 1: v = sum over the taps inside the image,
 * t = fp32(v) * (1 / fp32(R*S)) (padding counts as zeros).  Then t = t * m with
 * m = q_in / q_out (one fp32 division, formed here as q8_conv_int8 forms its scales: the
 * tail of Eq. A' between the input's factor and the output's), z = int8(Round(clamp(t,
 * -128, 127))).  With q_in == q_out max-pooling is exact.  x is dense [N][H][W][C].     */
int q8_pool_i8(const int8_t *x_dev, int N, int H, int W, int C, int mode, int R, int S,
               int stride, int pad, int Ho, int Wo, float q_in, float q_out, int8_t *y_dev,
               int out_c_stride, int out_c_off, void *stream);
/* fp32 twin for the calibration forward: max, or mean with padding counted as zeros.   */
int q8_pool_f32(const float *x_dev, int N, int H, int W, int C, int mode, int R, int S,
                int stride, int pad, int Ho, int Wo, float *y_dev, int out_c_stride,
                int out_c_off, void *stream);

/* Measurement only, not part of the method (no parity claim rests on it): `blocks` workgroups of four wavefronts each issue 4 * iters
 * register-resident v_mfma_i32_32x32x32_i8 (65536 int8 ops each), no memory traffic:
 * ops = blocks * 4 * 4 * iters * 65536.  The caller times the launch; the result is the
 * int8 matrix-core rate the chip sustains, to set beside the published peak.  sink_dev:
 * one int32 of device memory (practically never written).                             */
int q8_probe_mfma_i8(int blocks, int iters, int32_t *sink_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* Q8CONV_H */
