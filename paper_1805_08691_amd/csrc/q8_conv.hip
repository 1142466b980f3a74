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
// This file: host side of the convolution (argument checks, kernel choice, launch) and the
// filter pre-pack.  Kernels: q8_conv_ring_kernel.h (main), q8_conv_reg.hip (special shapes).
#include "q8_common.h"
#include "q8_conv_common.h"

namespace q8 {
int num_stream_variants();
int num_ring_variants();
int first_pw_variant();
int first_p3_variant();
int first_stem_variant();
int launch_stem_image(ConvParams& p, const StemImage& im, int pool, bool dry_run, hipStream_t stream);
int first_split_variant();
int num_split_variants();
void split_variant_tile(int variant, int* bp, int* bc);
int launch_dual_variant(ConvParams& p1, ConvParams& p2, hipStream_t stream);   // q8_conv_dual.hip
bool dual_shapes_supported(const ConvParams& p1, const ConvParams& p2);
}
#ifdef Q8_TRACE
namespace { unsigned long long* g_trace = nullptr; unsigned long long g_trace_cap = 0; }
#endif

namespace {

using q8::ConvParams;

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

// Kernel choice.  Stream variants (q8_conv_ring.hip) are numbered 0..; the register-staged
// kernel's variants (q8_conv_reg.hip) are offset by kRegBase.
constexpr int kRegBase = 100;

// A 4-channel image without padding: the S4 16-byte chunks (4 pixels each) of a filter row
// are contiguous bytes, i.e. the layer is an R x 1 convolution over 16*S4 "channels" whose
// pixels overlap, and the streaming kernel takes it as such (4-byte aligned loads, nothing
// needs a mask).  The pixels a row's last chunk reads beyond the last tap (next row, next
// image, or past the tensor, where the buffer range check returns zeros) meet the zero
// filter bytes that pad S to 4*S4 taps, so they add nothing.
bool image_rows_contiguous(const q8_conv_desc* d) {
  if (conv_mode(d) != 1 || d->pad_h || d->pad_w || d->dil_h != 1 || d->dil_w != 1) return false;
  if (d->in_c_stride != 0 && d->in_c_stride != 4) return false;
  return d->R <= 32 && d->H >= d->R && d->W >= d->S;
}

// The main kernel: 16-channel chunks and at most 32 taps (its in-image tap mask is 32 bits),
// any K (a channel tile is at least 64 wide; filter rows beyond K read as zeros), or an
// unpadded 4-channel image.
bool stream_capable(const q8_conv_desc* d) {
  return (conv_mode(d) == 0 && d->R * d->S <= 32) || image_rows_contiguous(d);
}
// Its extended build (unsigned codes, per-channel scales) is kept to K > 32.
bool ext_capable(const q8_conv_desc* d) { return stream_capable(d) && d->K > 32; }

// The 3x3 tile family (q8_conv_halo_kernel.h) for a padded 3x3 stride-1 layer over two or more
// 64-channel chunks (with one chunk the patch is not reused across chunks and the generic
// kernel is as fast): the largest tile that still gives every CU a tile and a half, else the
// smallest one the map's width allows.  -1: the generic kernel.  Fitted to a sweep over the
// 3x3 layers of the three benchmark networks.
int pick_halo3(const q8_conv_desc* d) {
  if (d->R != 3 || d->S != 3 || d->stride_h != 1 || d->stride_w != 1 || d->dil_h != 1 ||
      d->dil_w != 1 || d->pad_h != 1 || d->pad_w != 1 || d->C % 64 != 0 || d->C < 128 || d->K <= 32)
    return -1;
  struct Shape { int index, bp, bc, max_w; };
  // by falling tile size; the order of q8_conv_halo.hip's table is the index
  static const Shape shapes[] = {{2, 256, 128, 127}, {3, 256, 128, 383}, {1, 128, 128, 63},
                                 {0, 128, 64, 63},   {4, 128, 64, 191},  {6, 64, 64, 31}};
  const long M = (long)d->N * d->H * d->W;
  int smallest = -1;
  for (const Shape& s : shapes) {
    if (d->W > s.max_w || (s.bc == 128 && d->K <= 64)) continue;
    const long tiles = ((M + s.bp - 1) / s.bp) * ((d->K + s.bc - 1) / s.bc);
    // (the 64 x 64 tile inside a network, its filters coming from HBM: a ring of nine slabs)
    if (tiles >= 360) return s.index == 6 ? 11 : s.index;
    smallest = s.index;
  }
  // Down at the 64 x 64 tile there are at most a tile or two per CU and a tile's time is its
  // chain of reduction steps: with an even number of 64-channel chunks two groups of
  // wavefronts share the chain (builds 8 and 9 of the family's table), on 64 x 128 tiles
  // where those still give most CUs one.
  if (smallest == 6 && d->C % 128 == 0) {
    const long tiles_wide = ((M + 63) / 64) * ((d->K + 127) / 128);
    return d->K > 64 && tiles_wide >= 192 ? 9 : 12;
  }
  return smallest;
}

// `forced`: -1, or a variant of the main kernel to use where that kernel is applicable.
int pick_variant(const q8_conv_desc* d, int forced = -1) {
  const int mode = conv_mode(d);
  const int tile = d->K > 64 ? 0 : d->K > 32 ? 1 : 2;      // 128x128, 256x64, 256x32
  if (!stream_capable(d)) return kRegBase + 3 * mode + tile;
  if (forced >= 0) return forced;
  if (mode == 1) {
    // a first layer with up to eight taps per filter row, a stride and short output rows: the
    // image's rows are the operand as they lie in memory (q8_conv_stem_kernel.h)
    const int wo = out_extent(d->W, 0, 1, d->S, d->stride_w);
    const int ho = out_extent(d->H, 0, 1, d->R, d->stride_h);
    if (d->S > 4 && d->S <= 8 && d->R <= 8 && d->K <= 64 && (d->K & 15) == 0 && wo <= 128 &&
        d->W <= 240 && d->stride_h <= 2 && d->stride_w <= 2 &&
        (long)d->N * ho * wo >= 128L * 256 && wo >= 64)
      return q8::first_stem_variant();
    return d->K <= 64 ? 8 : 4;   // short reduction: small tiles, many per CU
  }
  // 3x3 / stride 1 / padding 1 on 64 channels with K <= 64 and many pixel tiles: persistent
  // workgroups with every filter resident, on 8 x 16 blocks of the map (any width; also a
  // little faster than the build on runs of 128 pixels where that one fits)
  if (d->R == 3 && d->S == 3 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 1 &&
      d->pad_w == 1 && d->dil_h == 1 && d->dil_w == 1 && d->C == 64 && d->K <= 64 &&
      (d->K & 15) == 0 && (long)d->N * d->H * d->W >= 128L * 256)
    return q8::first_p3_variant() + 2;
  const int halo = pick_halo3(d);
  if (halo >= 0) return q8::num_ring_variants() + halo;
  const int red = d->R * d->S * d->C;
  // pointwise layers on 64 channels with many pixel tiles: persistent workgroups (a layer the
  // build cannot take -- odd strides, a dump of the accumulators -- goes to the generic kernel)
  if (d->R * d->S == 1 && d->stride_h == 1 && d->stride_w == 1 && d->pad_h == 0 && d->pad_w == 0 &&
      d->C == 64 && (d->K & 15) == 0 && (long)d->N * d->H * d->W >= 128L * 512)
    return q8::first_pw_variant();
  const int nk = (red + 63) / 64;     // reduction steps of 64 bytes
  const long M = (long)d->N * out_extent(d->H, d->pad_h, d->dil_h, d->R, d->stride_h) *
                 out_extent(d->W, d->pad_w, d->dil_w, d->S, d->stride_w);
  const long tiles128 = ((M + 127) / 128) * ((d->K + 127) / 128);
  // Variant numbers: see kRingVariants.  Rules fitted to a sweep of every variant over the
  // ResNet-50 shapes at batch 64 (56x56 ... 7x7 maps, 64 ... 2048 channels):
  //  - few output channels: 128 pixels x 64 channels, more workgroups per CU;
  //  - very few tiles (the chip is not filled anyway, a workgroup's own chain of steps is
  //    what takes the time): smaller tiles with a deep ring, 64 x 64 at the smallest sizes;
  //  - short reductions (bound by memory latency and epilogue work per workgroup): ring of
  //    2, three or more workgroups per CU, 128 pixels x 64 channels on the large maps,
  //    64 pixels x 128 channels otherwise;
  //  - otherwise 128 x 128 with a ring of 3; when at most one workgroup per CU exists,
  //    eight wavefronts share the tile (more waves to hide LDS latency) with a ring of 4.
  //  - very large maps (hundreds of tiles per CU; the VGG-style layers of a detector at
  //    batch 64): 256 pixels per tile, which halves the filter reads per pixel.
  if (d->K <= 64) {
    if (tiles128 >= 16384) return 3;
    // a long reduction on a small map (a detector's box head): at most a workgroup or two
    // per CU, so the ring has to cover the memory latency by itself
    if (nk >= 16 && tiles128 <= 512) return tiles128 <= 128 ? (nk % 2 == 0 ? 21 : 7) : 9;
    return 8;
  }
  if (d->K >= 256 && tiles128 >= 1024 && nk > 4) return 13;
  // (layers with at most 128 such tiles: measured inside the networks, where their filters
  // come from HBM in every pass, 64 x 64 tiles with 128 reduction bytes per step beat the
  // 64-byte steps and the wider tiles that win on a warm cache)
  if (tiles128 <= 64) return nk % 2 == 0 ? 21 : 7;
  if (tiles128 <= 128) return d->R * d->S == 1 ? (nk % 2 == 0 ? 21 : 5) : 9;
  if (nk <= 4) return tiles128 >= 192 ? 8 : 4;
  // at most two 128 x 128 tiles per CU: eight wavefronts on such a tile with a ring of 4, or,
  // where those tiles would leave a third of the CUs idle (the 17 x 17 maps of an
  // Inception-shaped stack), 128 x 64 tiles with a ring of 4
  if (tiles128 <= 160) return 9;
  return tiles128 <= 512 ? 11 : 1;
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

}  // extern "C"

namespace {

// The 1x1 layer fused behind a convolution (see q8_conv_pair_int8).
struct PairArgs {
  const q8_conv_desc* d2;
  const void* w2;
  const int32_t* bias2;
  float q_w2, q_out;
  const int8_t* residual;
  float q_res;
  int8_t* z_y;
};

struct U8Flags {
  int in_u8, out_u8, res_u8;
  const int32_t* tap_sums;
  const float* m_vec = nullptr;     // per-output-channel scales (replace q_x * q_w / q_out)
  float* y_f32 = nullptr;           // real-valued output instead of int8 codes
  float* y_deq = nullptr;           // Eq. D of the output codes, written beside them
  const PairArgs* pair = nullptr;   // a second, 1x1 layer on the output while it is on chip
  int variant = -1;                 // tile variant of the main kernel to use (tests, tuning)
  int n_split = 0;                  // with a split-reduction variant: workgroups per tile
  void* workspace = nullptr;        // caller's device workspace: lets the reduction be split
  size_t workspace_bytes = 0;
};

// Checks the arguments of one layer and fills the kernels' parameter block.  *empty: the
// layer has no output pixel (nothing to launch).
int conv_fill(const q8_conv_desc* d, const U8Flags& u, const int8_t* z_x, const void* z_w_packed,
              const int32_t* bias_i32, float q_x, float q_w, float q_out,
              const int8_t* residual, float q_res, int8_t* z_y, int32_t* acc_dump,
              ConvParams& p, bool* empty) {
  *empty = false;
  Q8_REQUIRE(desc_sane(d), Q8_EINVAL);
  Q8_REQUIRE(q8_finite_pos(q_x) && q8_finite_pos(q_w) && q8_finite_pos(q_out), Q8_EINVAL);
  Q8_REQUIRE(residual == nullptr || q8_finite_pos(q_res), Q8_EINVAL);
  const int mode = conv_mode(d);
  Q8_REQUIRE(mode >= 0, Q8_EUNSUPPORTED);

  p = ConvParams{};
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
  if (M == 0) {
    *empty = true;
    return Q8_OK;
  }
  Q8_REQUIRE(M <= 0x7fffffffL, Q8_EUNSUPPORTED);
  Q8_REQUIRE((long)d->H * d->W * p.in_cs <= 0x7fffffffL, Q8_EUNSUPPORTED);
  Q8_REQUIRE(z_x && z_w_packed && (z_y || u.y_f32 || u.pair), Q8_EINVAL);
  Q8_REQUIRE(q8_aligned(z_w_packed, 16), Q8_EALIGN);
  if (u.y_f32) {
    Q8_REQUIRE(!(u.in_u8 || u.out_u8 || u.res_u8 || u.m_vec) && acc_dump == nullptr,
               Q8_EUNSUPPORTED);
    Q8_REQUIRE(q8_aligned(u.y_f32, 4), Q8_EALIGN);
  }
  if (mode == 0) {
    Q8_REQUIRE(p.in_cs % 16 == 0 && q8_aligned(z_x, 16), Q8_EALIGN);
    p.red_len = d->R * d->S * d->C;
    p.S4 = 0;
  } else {
    Q8_REQUIRE(p.in_cs == 4 && q8_aligned(z_x, 4), Q8_EALIGN);
    Q8_REQUIRE(d->dil_w == 1 && d->dil_h == 1, Q8_EUNSUPPORTED);
    p.S4 = (d->S + 3) / 4;
    p.red_len = d->R * p.S4 * 16;
    if (image_rows_contiguous(d)) {     // R x 1 taps over 16*S4 overlapping "channels"
      p.C = 16 * p.S4;
      p.S = 1;
    }
  }
  Q8_REQUIRE(bias_i32 == nullptr || q8_aligned(bias_i32, 16), Q8_EALIGN);
  Q8_REQUIRE(acc_dump == nullptr || q8_aligned(acc_dump, 16), Q8_EALIGN);

  {
    const long xb = (long)d->N * d->H * d->W * p.in_cs, wb = (long)d->K * p.red_len;
    // 32-bit buffer offsets; the activation descriptor also spans the first padding rows
    const long lead = ((long)d->pad_h * d->W + d->pad_w) * p.in_cs;
    Q8_REQUIRE(xb + lead < 0x7fffffffL && wb < 0x7fffffffL, Q8_EUNSUPPORTED);
    p.x_bytes = (int)xb;
    p.w_bytes = (int)wb;
    // tile order over the XCDs: filters larger than the activations the layer reads -> every
    // XCD keeps a slice of the filters and sees all pixels, else the other way round
    const long x_read = (d->R * d->S == 1) ? xb / ((long)d->stride_h * d->stride_w) : xb;
    p.ptile_fastest = x_read < wb ? 1 : 0;
  }
  p.x = z_x; p.w = (const int8_t*)z_w_packed; p.bias = bias_i32; p.res = residual; p.y = z_y;
  p.res_bytes = (residual && M * (long)p.res_cs < 0x7fffffffL) ? (int)(M * (long)p.res_cs) : 0;
  p.acc_dump = acc_dump;
  p.M = (int)M;
  p.in_u8 = u.in_u8; p.out_u8 = u.out_u8; p.res_u8 = u.res_u8;
  p.tap_sums = u.tap_sums;
  p.m_vec = u.m_vec;
  if (u.m_vec) {
    Q8_REQUIRE(ext_capable(d), Q8_EUNSUPPORTED);
    Q8_REQUIRE(!(u.in_u8 || u.out_u8 || u.res_u8), Q8_EUNSUPPORTED);
    Q8_REQUIRE(q8_aligned(u.m_vec, 16), Q8_EALIGN);
  }
  if (u.in_u8 || u.out_u8 || u.res_u8) {
    // unsigned codes: the streaming kernel only; an unsigned input whose taps can fall into
    // the padding needs the per-tap filter sums; an unsigned output is a ReLU output
    Q8_REQUIRE(ext_capable(d) && (mode == 0 || !u.in_u8), Q8_EUNSUPPORTED);
    Q8_REQUIRE(!u.out_u8 || d->relu, Q8_EINVAL);
    Q8_REQUIRE(!u.res_u8 || residual, Q8_EINVAL);
    if (u.in_u8 && (d->pad_h || d->pad_w)) {
      Q8_REQUIRE(u.tap_sums != nullptr, Q8_EINVAL);
      Q8_REQUIRE(q8_aligned(u.tap_sums, 16), Q8_EALIGN);
    } else {
      p.tap_sums = nullptr;          // every tap reads inside the image
    }
  }
  {
    const q8::FastDiv img = q8::make_fast_div((unsigned)(p.Ho * p.Wo));
    const q8::FastDiv row = q8::make_fast_div((unsigned)p.Wo);
    p.div_img_m = img.m; p.div_img_s = img.s;
    p.div_row_m = row.m; p.div_row_s = row.s;
  }
  p.relu = d->relu ? 1 : 0;
  {
    float prod = q_x * q_w;      // the x rule: factor of the accumulator
    if (u.y_f32) {               // Eq. D on the accumulator and on the residual, no Q
      p.m = prod;
      p.m_r = residual ? q_res : 0.0f;
    } else {
      p.m = prod / q_out;
      p.m_r = residual ? q_res / q_out : 0.0f;
    }
  }
  auto aligned_to = [&](int a) {
    return (u.y_f32 != nullptr ||
            (p.out_cs % a == 0 && p.out_off % a == 0 && q8_aligned(z_y, a))) &&
           (residual == nullptr ||
            (p.res_cs % a == 0 && p.res_off % a == 0 && q8_aligned(residual, a)));
  };
  p.vec4 = aligned_to(4) ? 1 : 0;
  p.vec16 = aligned_to(16) ? 1 : 0;
  p.y_f32 = u.y_f32;
  p.y_deq = u.y_deq;
  p.q_deq = q_out;
  if (u.y_deq) {
    Q8_REQUIRE(!(u.in_u8 || u.out_u8 || u.res_u8 || u.m_vec || u.y_f32 || u.pair) && z_y,
               Q8_EUNSUPPORTED);
    Q8_REQUIRE(q8_aligned(u.y_deq, 4), Q8_EALIGN);
  }
#ifdef Q8_TRACE
  p.trace = g_trace;
  p.trace_cap = g_trace_cap;
#endif
  p.f32_vec4 =
      ((u.y_f32 || u.y_deq) && p.out_cs % 4 == 0 && p.out_off % 4 == 0 &&
       q8_aligned(u.y_f32 ? u.y_f32 : u.y_deq, 16)) ? 1 : 0;

  return Q8_OK;
}

// Workspace of a split reduction: one int32 arrival counter per output tile (padded to 256
// bytes), then one int32 partial tile per (tile, part).
struct SplitLayout {
  int n_split;            // clipped to the number of reduction steps; < 2: no split
  size_t counter_bytes, bytes;
};
SplitLayout split_layout(const q8_conv_desc* d, int variant, int n_split) {
  SplitLayout l{1, 0, 0};
  if (variant < q8::first_split_variant() || conv_mode(d) != 0 || !stream_capable(d) ||
      d->C % 64 != 0)
    return l;
  int bp = 0, bc = 0;
  q8::split_variant_tile(variant - q8::first_split_variant(), &bp, &bc);
  const long M = (long)d->N * q8_conv_out_h(d) * q8_conv_out_w(d);
  const long tiles = ((M + bp - 1) / bp) * ((d->K + bc - 1) / bc);
  const int nk = d->R * d->S * d->C / 64;
  if (n_split > nk) n_split = nk;
  if (n_split < 2 || tiles <= 0) return l;
  l.n_split = n_split;
  l.counter_bytes = (size_t)((tiles * 4 + 255) / 256 * 256);
  l.bytes = l.counter_bytes + (size_t)tiles * n_split * bp * bc * 4;
  return l;
}

// Whether the layer's reduction is split when the caller provides a workspace, and how.
// No layer is: the partial tiles have to pass through memory (the parts of a tile may sit on
// different XCDs), and on every ResNet-50 / SSD shape tried that costs more than the shorter
// chain of reduction steps saves (7x7 512->512 3x3 at batch 32: 10.2 us unsplit, 12.2 us at
// best split in two).  The split builds stay reachable through q8_conv_int8_variant.
void split_plan(const q8_conv_desc*, int*, int*) {}

int conv_launch(const q8_conv_desc* d, const U8Flags& u, const int8_t* z_x, const void* z_w_packed,
                const int32_t* bias_i32, float q_x, float q_w, float q_out,
                const int8_t* residual, float q_res, int8_t* z_y, int32_t* acc_dump,
                void* stream) {
  ConvParams p;
  bool empty = false;
  const int rc = conv_fill(d, u, z_x, z_w_packed, bias_i32, q_x, q_w, q_out, residual, q_res, z_y,
                           acc_dump, p, &empty);
  if (rc != Q8_OK || empty) return rc;
  const int mode = conv_mode(d);
  hipStream_t s = (hipStream_t)stream;
  if (u.pair) {
    // q_out of this call is the intermediate tensor's factor; the second layer reads it
    const PairArgs& a = *u.pair;
    const q8_conv_desc* d2 = a.d2;
    Q8_REQUIRE(!(u.in_u8 || u.out_u8 || u.res_u8 || u.m_vec || u.y_f32) && !acc_dump && !residual,
               Q8_EUNSUPPORTED);
    Q8_REQUIRE(desc_sane(d2) && a.w2 && a.z_y, Q8_EINVAL);
    Q8_REQUIRE(q8_finite_pos(a.q_w2) && q8_finite_pos(a.q_out), Q8_EINVAL);
    Q8_REQUIRE(a.residual == nullptr || q8_finite_pos(a.q_res), Q8_EINVAL);
    // the second layer: 1x1, stride 1, no padding, over exactly the first layer's output
    Q8_REQUIRE(d2->N == d->N && d2->H == p.Ho && d2->W == p.Wo && d2->C == d->K, Q8_EINVAL);
    Q8_REQUIRE(d2->R == 1 && d2->S == 1 && d2->stride_h == 1 && d2->stride_w == 1 &&
                   d2->pad_h == 0 && d2->pad_w == 0 &&
                   (d2->in_c_stride == 0 || d2->in_c_stride == d->K), Q8_EUNSUPPORTED);
    Q8_REQUIRE(mode == 0 && stream_capable(d) && d->C % 64 == 0 && (d->K == 64 || d->K == 128) &&
                   d2->K % d->K == 0, Q8_EUNSUPPORTED);
    Q8_REQUIRE(q8_aligned(a.w2, 16) && (a.bias2 == nullptr || q8_aligned(a.bias2, 16)), Q8_EALIGN);
    p.w2 = (const int8_t*)a.w2; p.bias2 = a.bias2; p.res2 = a.residual; p.y2 = a.z_y;
    p.K2 = d2->K;
    p.w2_bytes = d2->K * d->K;
    p.out_cs2 = d2->out_c_stride ? d2->out_c_stride : d2->K;
    p.out_off2 = d2->out_c_off;
    p.res_cs2 = d2->res_c_stride ? d2->res_c_stride : d2->K;
    p.res_off2 = d2->res_c_off;
    Q8_REQUIRE(p.out_off2 >= 0 && p.res_off2 >= 0 && p.out_cs2 >= p.out_off2 + d2->K, Q8_EINVAL);
    Q8_REQUIRE(a.residual == nullptr || p.res_cs2 >= p.res_off2 + d2->K, Q8_EINVAL);
    {
      float prod = q_out * a.q_w2;      // the intermediate's factor times the filters'
      p.m2 = prod / a.q_out;
      p.m_r2 = a.residual ? a.q_res / a.q_out : 0.0f;
    }
    p.relu2 = d2->relu ? 1 : 0;
    auto aligned2 = [&](int al) {
      return p.out_cs2 % al == 0 && p.out_off2 % al == 0 && q8_aligned(a.z_y, al) &&
             (a.residual == nullptr ||
              (p.res_cs2 % al == 0 && p.res_off2 % al == 0 && q8_aligned(a.residual, al)));
    };
    p.vec4_2 = aligned2(4) ? 1 : 0;
    p.vec16_2 = aligned2(16) ? 1 : 0;
    return q8::launch_pair_variant(p, s);
  }
  int variant = pick_variant(d, u.variant);
  p.n_split = 1;
  p.ws_counters = nullptr;
  p.ws_slabs = nullptr;
  if (variant >= kRegBase) return q8::launch_reg_variant(variant - kRegBase, p, s);
  int n_split = u.n_split;
  if (u.variant < 0 && u.workspace && !(u.in_u8 || u.out_u8 || u.res_u8 || u.m_vec || u.y_f32))
    split_plan(d, &variant, &n_split);
  if (variant >= q8::first_split_variant() && n_split >= 2) {
    const SplitLayout l = split_layout(d, variant, n_split);
    if (l.n_split >= 2) {       // (a reduction of one step is not split)
      Q8_REQUIRE(u.workspace != nullptr, Q8_EINVAL);
      Q8_REQUIRE(q8_aligned(u.workspace, 256), Q8_EALIGN);
      Q8_REQUIRE(u.workspace_bytes >= l.bytes, Q8_EWORKSPACE);
      p.n_split = l.n_split;
      p.ws_counters = (int*)u.workspace;
      p.ws_slabs = (int*)((char*)u.workspace + l.counter_bytes);
    }
  }
  return q8::launch_stream_variant(variant, p, s);
}

}  // namespace

namespace q8 {
int conv_fill_plain(const q8_conv_desc* d, const int8_t* z_x, const void* z_w_packed,
                    const int32_t* bias_i32, float q_x, float q_w, float q_out,
                    const int8_t* residual, float q_res, int8_t* z_y, ConvParams& p, bool* empty) {
  return conv_fill(d, U8Flags{0, 0, 0, nullptr}, z_x, z_w_packed, bias_i32, q_x, q_w, q_out,
                   residual, q_res, z_y, nullptr, p, empty);
}
}  // namespace q8

namespace {

// start[idx*K + k] = bias[k] + 128 * (sum of filter k over the taps of rectangle idx), for
// every rectangle [r_lo, r_hi) x [s_lo, s_hi) of the filter (see u8_start_index; an empty or
// inverted rectangle gets the bare bias); bias_eff[k] = the whole filter's row.
constexpr int kMaxPrefix = 128;      // (R+1)*(S+1) with R*S <= 32 is at most 66
__global__ void u8_prepare_kernel(const int8_t* __restrict__ w, const int32_t* __restrict__ bias,
                                  int K, int R, int S, int C, int32_t* __restrict__ start,
                                  int32_t* __restrict__ bias_eff) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= K) return;
  const int w1 = S + 1;
  int pre[kMaxPrefix];               // 2-D prefix sums of the per-tap filter sums
  for (int s = 0; s <= S; ++s) pre[s] = 0;
  for (int r = 1; r <= R; ++r) {
    pre[r * w1] = 0;
    int row = 0;                                   // sum of filter row r-1 up to column s
    for (int s = 1; s <= S; ++s) {
      const int8_t* tap = w + (((size_t)k * R + (r - 1)) * S + (s - 1)) * C;
      int sum = 0;
      for (int c = 0; c < C; ++c) sum += tap[c];
      row += sum;
      pre[r * w1 + s] = pre[(r - 1) * w1 + s] + row;
    }
  }
  const int b = bias ? bias[k] : 0;
  for (int r_lo = 0; r_lo <= R; ++r_lo)
    for (int r_hi = 0; r_hi <= R; ++r_hi)
      for (int s_lo = 0; s_lo <= S; ++s_lo)
        for (int s_hi = 0; s_hi <= S; ++s_hi) {
          int sum = 0;
          if (r_hi > r_lo && s_hi > s_lo)
            sum = pre[r_hi * w1 + s_hi] - pre[r_lo * w1 + s_hi] - pre[r_hi * w1 + s_lo] +
                  pre[r_lo * w1 + s_lo];
          const size_t idx = ((size_t)(r_lo * (R + 1) + r_hi) * w1 + s_lo) * w1 + s_hi;
          start[idx * K + k] = b + 128 * sum;
        }
  bias_eff[k] = b + 128 * pre[R * w1 + S];
}

}  // namespace

extern "C" {

int q8_conv_int8(const q8_conv_desc* d, const int8_t* z_x, const void* z_w_packed,
                 const int32_t* bias_i32, float q_x, float q_w, float q_out,
                 const int8_t* residual, float q_res, int8_t* z_y, int32_t* acc_dump,
                 void* workspace, size_t workspace_bytes, void* stream) {
  U8Flags u{0, 0, 0, nullptr};
  u.workspace = workspace;
  u.workspace_bytes = workspace_bytes;
  return conv_launch(d, u, z_x, z_w_packed, bias_i32, q_x, q_w, q_out, residual, q_res, z_y,
                     acc_dump, stream);
}

// Eq. Q on the image + its first layer (+ max-pool): see include/q8conv.h.  dry_run: checks only.
static int conv_image_f32(const q8_conv_desc* d, const float* r_dev, int H, int W, int C, int top,
                          int left, float q_x, int p_bits, const void* z_w_packed,
                          const int32_t* bias_i32, float q_w, float q_out, int pool, int8_t* z_y,
                          bool dry_run, void* stream) {
  Q8_REQUIRE(desc_sane(d) && p_bits >= 1 && p_bits <= 7 && (pool == 0 || pool == 1), Q8_EINVAL);
  Q8_REQUIRE(H >= 1 && W >= 1 && C >= 1 && C <= 4 && C == d->C && top >= 0 && left >= 0 &&
                 d->H >= top + H && d->W >= left + W, Q8_EINVAL);
  if (!image_rows_contiguous(d)) return Q8_EUNSUPPORTED;
  Q8_REQUIRE(r_dev != nullptr && q8_aligned(r_dev, 4), r_dev ? Q8_EALIGN : Q8_EINVAL);
  q8::ConvParams p;
  bool empty = false;
  // the layer over the zero frame; its int8 input pointer only stands in (never read)
  const int rc = conv_fill(d, U8Flags{0, 0, 0, nullptr}, reinterpret_cast<const int8_t*>(r_dev),
                           z_w_packed, bias_i32, q_x, q_w, q_out, nullptr, 0.0f, z_y, nullptr, p,
                           &empty);
  if (rc != Q8_OK || empty) return rc;
  q8::StemImage im;
  im.r = r_dev; im.H = H; im.W = W; im.C = C; im.top = top; im.left = left;
  im.q = q_x;
  im.hi = (float)((1 << p_bits) - 1);
  im.lo = -(float)(1 << p_bits);
  im.Hp = (p.Ho - 1) / 2 + 1;
  im.Wp = (p.Wo - 1) / 2 + 1;
  return q8::launch_stem_image(p, im, pool, dry_run, (hipStream_t)stream);
}

int q8_conv_image_f32_int8(const q8_conv_desc* d, const float* r_dev, int H, int W, int C, int top,
                           int left, float q_x, int p, const void* z_w_packed,
                           const int32_t* bias_i32, float q_w, float q_out, int pool, int8_t* z_y,
                           void* stream) {
  return conv_image_f32(d, r_dev, H, W, C, top, left, q_x, p, z_w_packed, bias_i32, q_w, q_out,
                        pool, z_y, false, stream);
}

int q8_conv_image_f32_supported(const q8_conv_desc* d, int H, int W, int C, int top, int left,
                                int pool) {
  // stand-in pointers with the alignment a caller's buffers must have
  const auto fake = [](uintptr_t a) { return reinterpret_cast<void*>(a); };
  return conv_image_f32(d, static_cast<const float*>(fake(256)), H, W, C, top, left, 1.0f, 7,
                        fake(512), nullptr, 1.0f, 1.0f, pool, static_cast<int8_t*>(fake(768)), true,
                        nullptr) == Q8_OK ? 1 : 0;
}

size_t q8_conv_workspace_bytes(const q8_conv_desc* d) {
  if (!desc_sane(d)) return 0;
  int variant = -1, n_split = 1;
  split_plan(d, &variant, &n_split);
  return variant < 0 ? 0 : split_layout(d, variant, n_split).bytes;
}

size_t q8_conv_workspace_bytes_variant(const q8_conv_desc* d, int variant, int n_split) {
  if (!desc_sane(d) || variant < 0 || variant >= q8::num_stream_variants()) return 0;
  return split_layout(d, variant, n_split).bytes;
}

int q8_conv_u8(const q8_conv_desc* d, int in_unsigned, int out_unsigned, int res_unsigned,
               const int8_t* z_x, const void* z_w_packed, const int32_t* bias_eff,
               const int32_t* tap_sums, float q_x, float q_w, float q_out,
               const int8_t* residual, float q_res, int8_t* z_y, int32_t* acc_dump,
               void* stream) {
  Q8_REQUIRE(!in_unsigned || bias_eff != nullptr, Q8_EINVAL);
  return conv_launch(d, U8Flags{in_unsigned ? 1 : 0, out_unsigned ? 1 : 0, res_unsigned ? 1 : 0,
                                tap_sums},
                     z_x, z_w_packed, bias_eff, q_x, q_w, q_out, residual, q_res, z_y, acc_dump,
                     stream);
}

int q8_conv_int8_per_channel(const q8_conv_desc* d, const int8_t* z_x, const void* z_w_packed,
                             const int32_t* bias_i32, const float* m_dev, float q_out,
                             const int8_t* residual, float q_res, int8_t* z_y,
                             int32_t* acc_dump, void* stream) {
  Q8_REQUIRE(m_dev != nullptr, Q8_EINVAL);
  U8Flags u{0, 0, 0, nullptr};
  u.m_vec = m_dev;
  // q_x and q_w only enter through m_dev here: pass neutral factors to the shared checks
  return conv_launch(d, u, z_x, z_w_packed, bias_i32, 1.0f, 1.0f, q_out, residual, q_res, z_y,
                     acc_dump, stream);
}

int q8_conv_int8_real_output(const q8_conv_desc* d, const int8_t* z_x, const void* z_w_packed,
                             const int32_t* bias_i32, float q_x, float q_w,
                             const int8_t* residual, float q_res, float* y_dev, void* stream) {
  U8Flags u{0, 0, 0, nullptr};
  u.y_f32 = y_dev;            // null: rejected by the shared checks unless the output is empty
  return conv_launch(d, u, z_x, z_w_packed, bias_i32, q_x, q_w, 1.0f, residual, q_res, nullptr,
                     nullptr, stream);
}

int q8_conv_int8_dequantized(const q8_conv_desc* d, const int8_t* z_x, const void* z_w_packed,
                             const int32_t* bias_i32, float q_x, float q_w, float q_out,
                             const int8_t* residual, float q_res, int8_t* z_y, float* r_y,
                             void* stream) {
  Q8_REQUIRE(r_y != nullptr || (d && d->N == 0), Q8_EINVAL);
  U8Flags u{0, 0, 0, nullptr};
  u.y_deq = r_y;
  return conv_launch(d, u, z_x, z_w_packed, bias_i32, q_x, q_w, q_out, residual, q_res, z_y,
                     nullptr, stream);
}

int q8_conv_pair_int8(const q8_conv_desc* d1, const int8_t* z_x, const void* w1_packed,
                      const int32_t* bias1, float q_x, float q_w1, float q_mid,
                      const q8_conv_desc* d2, const void* w2_packed, const int32_t* bias2,
                      float q_w2, float q_out, const int8_t* residual, float q_res, int8_t* z_y,
                      void* stream) {
  PairArgs a{d2, w2_packed, bias2, q_w2, q_out, residual, q_res, z_y};
  U8Flags u{0, 0, 0, nullptr};
  u.pair = &a;
  return conv_launch(d1, u, z_x, w1_packed, bias1, q_x, q_w1, q_mid, nullptr, 0.0f, nullptr, nullptr,
                     stream);
}

// Both layers must take the uniform-tap build of the main kernel (C % 64 == 0, at most 32
// taps, K > 32) and a supported pair of tile shapes; the library tries and reports.
int q8_conv_dual_int8(const q8_conv_desc* d1, const int8_t* z_x1, const void* w1_packed,
                      const int32_t* bias1, float q_x1, float q_w1, float q_out1,
                      const int8_t* residual1, float q_res1, int8_t* z_y1,
                      const q8_conv_desc* d2, const int8_t* z_x2, const void* w2_packed,
                      const int32_t* bias2, float q_x2, float q_w2, float q_out2,
                      const int8_t* residual2, float q_res2, int8_t* z_y2, void* stream) {
  Q8_REQUIRE(q8_conv_dual_supported(d1, d2), Q8_EUNSUPPORTED);
  ConvParams p1, p2;
  bool e1 = false, e2 = false;
  int rc = conv_fill(d1, U8Flags{0, 0, 0, nullptr}, z_x1, w1_packed, bias1, q_x1, q_w1, q_out1,
                     residual1, q_res1, z_y1, nullptr, p1, &e1);
  if (rc != Q8_OK) return rc;
  rc = conv_fill(d2, U8Flags{0, 0, 0, nullptr}, z_x2, w2_packed, bias2, q_x2, q_w2, q_out2,
                 residual2, q_res2, z_y2, nullptr, p2, &e2);
  if (rc != Q8_OK) return rc;
  if (e1 || e2) return Q8_EUNSUPPORTED;
  // the outputs must not overlap each other nor an input of the other layer
  Q8_REQUIRE(z_y1 != z_y2 && (const int8_t*)z_y1 != z_x2 && (const int8_t*)z_y2 != z_x1 &&
                 (const int8_t*)z_y1 != residual2 && (const int8_t*)z_y2 != residual1, Q8_EINVAL);
  return q8::launch_dual_variant(p1, p2, (hipStream_t)stream);
}

int q8_conv_dual_supported(const q8_conv_desc* d1, const q8_conv_desc* d2) {
  for (const q8_conv_desc* d : {d1, d2}) {
    if (!desc_sane(d) || conv_mode(d) != 0 || d->C % 64 != 0 || d->R * d->S > 32 || d->K <= 32) return 0;
  }
  // probe the shape table with the two layers' sizes (no launch)
  ConvParams p1{}, p2{};
  const q8_conv_desc* ds[2] = {d1, d2};
  ConvParams* ps[2] = {&p1, &p2};
  for (int i = 0; i < 2; ++i) {
    ps[i]->M = (int)((long)ds[i]->N * q8_conv_out_h(ds[i]) * q8_conv_out_w(ds[i]));
    ps[i]->K = ds[i]->K;
    ps[i]->red_len = ds[i]->R * ds[i]->S * ds[i]->C;
  }
  return q8::dual_shapes_supported(p1, p2) ? 1 : 0;
}

int q8_conv_pair_supported(const q8_conv_desc* d1, const q8_conv_desc* d2) {
  if (!desc_sane(d1) || !desc_sane(d2) || conv_mode(d1) != 0 || !stream_capable(d1)) return 0;
  if (d1->C % 64 != 0 || (d1->K != 64 && d1->K != 128) || d2->K % d1->K != 0) return 0;
  if (d2->N != d1->N || d2->H != q8_conv_out_h(d1) || d2->W != q8_conv_out_w(d1) || d2->C != d1->K)
    return 0;
  if (d2->R != 1 || d2->S != 1 || d2->stride_h != 1 || d2->stride_w != 1 || d2->pad_h || d2->pad_w)
    return 0;
  if (d2->in_c_stride != 0 && d2->in_c_stride != d1->K) return 0;
  // the operand ring and every filter of the second layer share the 160 KB of LDS
  const long ring = d1->K == 64 ? 2L * (128 + 64) * 64 : 4L * (128 + 128) * 64;
  if (ring + (long)d2->K * d1->K > 160 * 1024) return 0;
  return 1;
}

int q8_u8_prepare(const q8_conv_desc* d, const int8_t* z_w_krsc_dev, const int32_t* bias_i32,
                  int32_t* tap_sums_dev, int32_t* bias_eff_dev, void* stream) {
  Q8_REQUIRE(desc_sane(d) && z_w_krsc_dev && tap_sums_dev && bias_eff_dev, Q8_EINVAL);
  Q8_REQUIRE(conv_mode(d) == 0 && (d->R + 1) * (d->S + 1) <= kMaxPrefix, Q8_EUNSUPPORTED);
  hipLaunchKernelGGL(u8_prepare_kernel, dim3((d->K + 63) / 64), dim3(64), 0, (hipStream_t)stream,
                     z_w_krsc_dev, bias_i32, d->K, d->R, d->S, d->C, tap_sums_dev, bias_eff_dev);
  return q8_launch_status();
}

int q8_conv_num_variants(void) { return q8::num_stream_variants(); }
const char* q8_conv_variant_name(int variant) { return q8::stream_variant_name(variant); }

int q8_conv_int8_variant(const q8_conv_desc* d, const int8_t* z_x, const void* z_w_packed,
                         const int32_t* bias_i32, float q_x, float q_w, float q_out,
                         const int8_t* residual, float q_res, int8_t* z_y, int32_t* acc_dump,
                         int variant, int n_split, void* workspace, size_t workspace_bytes,
                         void* stream) {
  Q8_REQUIRE(variant >= -1 && variant < q8::num_stream_variants(), Q8_EINVAL);
  Q8_REQUIRE(n_split >= 0 && n_split <= 64, Q8_EINVAL);
  U8Flags u{0, 0, 0, nullptr};
  u.variant = variant;
  u.n_split = n_split;
  u.workspace = workspace;
  u.workspace_bytes = workspace_bytes;
  return conv_launch(d, u, z_x, z_w_packed, bias_i32, q_x, q_w, q_out, residual, q_res, z_y,
                     acc_dump, stream);
}

const char* q8_conv_variant(const q8_conv_desc* d) {
  if (!desc_sane(d) || conv_mode(d) < 0) return "unsupported";
  const int variant = pick_variant(d);
  return variant >= kRegBase ? q8::reg_variant_name(variant - kRegBase)
                             : q8::stream_variant_name(variant);
}

}  // extern "C"

#ifdef Q8_TRACE
// Measurement build only (never part of the product library): where the workgroups log.
extern "C" void q8_trace_set(unsigned long long* buf_dev, unsigned long long cap) {
  g_trace = buf_dev;
  g_trace_cap = cap;
}
#endif
