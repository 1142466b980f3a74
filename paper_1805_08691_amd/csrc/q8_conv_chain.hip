// A list of convolution layers (Eq. A' of arxiv 1805.08691 with the fused ReLU / element-wise
// sum of its "Model Optimization" section, each layer exactly as q8_conv_int8 computes it) run
// by ONE persistent launch, built around how an MI355X is put together:
//
//  * The chip is eight XCDs of 32 compute units, each XCD with an L2 of its own.  The batch is
//    split into eight groups of images and XCD x computes every layer for group x only.
//    Images are independent, so a tile's operands and results are only ever touched by
//    workgroups of one XCD: that XCD's L2 is the point of coherence, with plain loads and
//    stores, and nothing has to be written back or invalidated between layers.  A workgroup
//    learns which XCD it runs on from the XCC_ID hardware register and takes its work from
//    that XCD's queue, so the affinity holds by construction, not by a launch-order guess.
//  * Work items are output tiles, queued per XCD in layer order.  A tile waits until the
//    tiles that produce the input pixels it reads (and its residual pixels) have finished:
//    one completion counter per pixel tile of every layer, bumped through the L2 after the
//    tile's stores have been acknowledged (s_waitcnt vmcnt(0)).  There is no grid-wide
//    barrier and no launch boundary between layers: the head of layer l+1 overlaps the tail
//    of layer l, and a layer too small to fill the chip shares it with its neighbours.
//  * Every wait is bounded.  A tile that gives up raises a status word that ends every other
//    wait at once, so the launch always drains; the host can read the status afterwards.
//    Queue order = layer order and a tile only waits for earlier queue entries, which are
//    finished or in the hands of a running workgroup, so a healthy launch cannot deadlock
//    whatever number of workgroups is resident.
//
// The tile itself is conv_tile_ring of q8_conv_ring_kernel.h, unchanged.
#include "q8_conv_ring_kernel.h"

#include <stdlib.h>
#include <string.h>
#include <mutex>
#include <vector>

namespace q8 {
int conv_fill_plain(const q8_conv_desc* d, const int8_t* z_x, const void* z_w_packed,
                    const int32_t* bias_i32, float q_x, float q_w, float q_out,
                    const int8_t* residual, float q_res, int8_t* z_y, ConvParams& p, bool* empty);
}

namespace {

using q8::ConvParams;
using q8::kNumXcd;

constexpr unsigned kPlanMagic = 0x51384348u;      // "Q8CH"
constexpr int kChainThreads = 256;
constexpr int kWgPerCu = 3;
constexpr int kSpinLimit = 1 << 19;               // polls (about 0.4 s) before a waiting tile gives up

// Workspace layout (int32 words): word 0 = status (0 ok; 1 a wait gave up; 2 unexpected
// XCC_ID); from word 32 on one region per XCD, 32-word aligned so that no two XCDs ever
// touch the same 128-byte line: the queue head, then that XCD's completion counters.
constexpr int kWsStatus = 0;
constexpr int kWsRegions = 32;
constexpr int kRegionHead = 0;                    // first word of a region: next queue entry
constexpr int kRegionDone = 32;                   // completion counters from here on

// tile variants of the chain kernel (four wavefronts each): pixels x channels, ring depth
struct ChainVariant { int bp, bc, stages; };
constexpr ChainVariant kVariants[] = {{128, 128, 3}, {128, 64, 4}, {64, 128, 4}, {64, 64, 4}};
constexpr int kNumVariants = 4;
constexpr int kChainLds = 48 * 1024;              // the largest ring of the four

struct ChainLayerDev {
  int variant;
  int n_ctiles;               // channel tiles per pixel tile = completion target of a counter
  int bp;                     // pixels per tile
  int src_layer, res_layer;   // producer of z_x / of the residual inside the chain, or -1
  int pad_;
  int done_off[kNumXcd];      // word offset of this layer's counters in the workspace, per XCD
                              // (absolute: inside XCD x's region)
  int n_ptiles[kNumXcd];
};

struct ChainHeader {
  unsigned magic;
  int n_layers;
  int total_bytes;
  int ws_words;
  int grid;
  int layers_off, params_off, items_off;   // byte offsets inside the plan
  int n_items[kNumXcd];
  int item_off[kNumXcd];                   // first entry of XCD x in the item array
  int head_off[kNumXcd];                   // word of XCD x's queue head in the workspace
};

// item: layer << 24 | ctile << 16 | ptile
__host__ __device__ inline int pack_item(int layer, int ptile, int ctile) {
  return (layer << 24) | (ctile << 16) | ptile;
}

__device__ __forceinline__ int xcc_id() {
  // hwreg(HW_REG_XCC_ID = 20), bits 3:0: the XCD this wavefront runs on
  return __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & 15;
}

// Index (in the input tensor's pixel order n, h, w) of the first / last input pixel that
// output pixel `pix` reads; the taps outside the image are clipped away.
__device__ __forceinline__ int input_pixel(const ConvParams& p, int pix, bool last) {
  const int n = q8::fast_div(pix, p.div_img_m, p.div_img_s);
  const int rem = pix - n * (p.Ho * p.Wo);
  const int ho = q8::fast_div(rem, p.div_row_m, p.div_row_s);
  const int wo = rem - ho * p.Wo;
  int hi = ho * p.stride_h - p.pad_h, wi = wo * p.stride_w - p.pad_w;
  if (last) {
    hi += (p.R - 1) * p.dil_h;
    wi += (p.S - 1) * p.dil_w;
  }
  hi = min(max(hi, 0), p.H - 1);
  wi = min(max(wi, 0), p.W - 1);
  return (n * p.H + hi) * p.W + wi;
}

// Wave 0 waits until counters [j0, j1] of `done` have reached `target`.
__device__ __forceinline__ bool wait_counters(int* done, int j0, int j1, int target, int* status,
                                              int zero, int lane) {
  bool ok = true;
  for (int j = j0 + lane; j <= j1; j += 64) {
    int n = 0;
    // an atomic add of a run-time zero: executed by the L2, never answered by the L1
    while (__hip_atomic_fetch_add(done + j, zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) <
           target) {
      __builtin_amdgcn_s_sleep(12);      // about 0.4 us between polls: the L2 serves the producers first
      ++n;
      if (n > kSpinLimit ||
          ((n & 63) == 0 && __hip_atomic_fetch_add(status, zero, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT) != 0)) {
        ok = false;
        break;
      }
    }
  }
  return ok;
}

__global__ __launch_bounds__(kChainThreads, kWgPerCu) void conv_chain_kernel(
    const unsigned char* __restrict__ plan, int* ws, const int zero) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(1024))) int8_t lds[];
  int* const s_word = reinterpret_cast<int*>(lds + kChainLds);     // [0]: the claimed queue entry
  const ChainHeader& hd = *reinterpret_cast<const ChainHeader*>(plan);
  const ChainLayerDev* const layers = reinterpret_cast<const ChainLayerDev*>(plan + hd.layers_off);
  const ConvParams* const params = reinterpret_cast<const ConvParams*>(plan + hd.params_off);
  const int* const items = reinterpret_cast<const int*>(plan + hd.items_off);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int x = xcc_id();
  if (x >= kNumXcd) {           // not a chip this code knows: touch nothing but the status
    __hip_atomic_fetch_max(ws + kWsStatus, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }
  const int n_items = hd.n_items[x];
  const int* const my_items = items + hd.item_off[x];
  // Control flow around the barriers below is kept wave-uniform: the branches are on `wave`
  // (a scalar), and what one lane alone does sits in a small lane-0 region nested inside, closed
  // again before the barrier.  A divergent "if (tid == 0)" on both sides of the loop's back
  // edge lets the compiler send the other lanes round the loop, barrier included, ahead of
  // lane 0.
  // (a workgroup cannot take more entries than its queue holds: the loop is bounded even if
  // the claimed index were misread)
  for (int taken = 0; taken <= n_items; ++taken) {
    if (wave == 0) {
      int got = 0;
      if (lane == 0)
        got = __hip_atomic_fetch_add(ws + hd.head_off[x], 1, __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_WORKGROUP);
      s_word[0] = __builtin_amdgcn_readfirstlane(got);     // every lane writes the same word
    }
    __syncthreads();
    const int idx = __builtin_amdgcn_readfirstlane(s_word[0]);
    if (idx >= n_items) break;
    const int item = my_items[idx];
    const int li = item >> 24, ctile = (item >> 16) & 255, ptile = item & 0xffff;
    const ChainLayerDev& L = layers[li];
    const ConvParams& p = params[li * kNumXcd + x];
    if (wave == 0) {
      const int pix0 = ptile * L.bp;
      const int pix1 = min(pix0 + L.bp, p.M) - 1;
      bool ok = true;
      if (L.src_layer >= 0) {
        const ChainLayerDev& S = layers[L.src_layer];
        const int a = input_pixel(p, pix0, false), b = input_pixel(p, pix1, true);
        ok = wait_counters(ws + S.done_off[x], a / S.bp, b / S.bp, S.n_ctiles, ws + kWsStatus, zero,
                           lane);
      }
      if (L.res_layer >= 0) {
        const ChainLayerDev& R = layers[L.res_layer];
        ok = wait_counters(ws + R.done_off[x], pix0 / R.bp, pix1 / R.bp, R.n_ctiles,
                           ws + kWsStatus, zero, lane) && ok;
      }
      // any lane that gave up raises the status (max with 0 from the others)
      if (!ok) __hip_atomic_fetch_max(ws + kWsStatus, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();      // the producers' results are in the L2; nothing of them is in this L1
    switch (L.variant) {
      case 0: q8::conv_tile_ring<2, 2, 2, 2, 64, 3, 1, 0>(p, ptile, ctile, lds); break;
      case 1: q8::conv_tile_ring<2, 2, 2, 1, 64, 4, 1, 0>(p, ptile, ctile, lds); break;
      case 2: q8::conv_tile_ring<2, 2, 1, 2, 64, 4, 1, 0>(p, ptile, ctile, lds); break;
      default: q8::conv_tile_ring<2, 2, 1, 1, 64, 4, 1, 0>(p, ptile, ctile, lds); break;
    }
    // the tile's stores have reached the L2 (the counter below is what a consumer sees)
    q8::wait_vmcnt<0>();
    __syncthreads();
    if (wave == 0) {
      if (lane == 0)
        __hip_atomic_fetch_add(ws + L.done_off[x] + ptile, 1, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_WORKGROUP);
    }
  }
#endif
}

__global__ void chain_clear_kernel(int* ws, int n) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) ws[i] = 0;
}

// images [n0, n0 + nx) of XCD x
void xcd_share(int N, int x, int* n0, int* nx) {
  const int base = N / kNumXcd, rem = N % kNumXcd;
  *nx = base + (x < rem ? 1 : 0);
  *n0 = x * base + (x < rem ? x : rem);
}

bool chain_capable(const q8_conv_desc& d) {
  // the uniform-tap build of the main kernel, whole dense tensors
  return d.C % 64 == 0 && d.R * d.S <= 32 && d.K > 32 &&
         (d.in_c_stride == 0 || d.in_c_stride == d.C) &&
         (d.out_c_stride == 0 || d.out_c_stride == d.K) && d.out_c_off == 0 &&
         (d.res_c_stride == 0 || d.res_c_stride == d.K) && d.res_c_off == 0;
}

// Tile variant for a layer whose XCD share has Mx output pixels: a model of the time one
// compute unit needs (tiles it gets in turn x steps x the larger of operand-fill and matrix
// clocks per step, plus a fixed cost per tile).
int pick_chain_variant(long Mx, int K, int red_len, int forced) {
  if (forced >= 0 && forced < kNumVariants) return forced;
  const int nk = (red_len + 63) / 64;
  int best = 0;
  double best_cost = 1e30;
  for (int v = 0; v < kNumVariants; ++v) {
    const int P = kVariants[v].bp, Q = kVariants[v].bc;
    const long tiles = ((Mx + P - 1) / P) * ((K + Q - 1) / Q);
    // clocks of one CU per reduction step: operand fill (64 B/clk) or matrix issue at the
    // rate the ring sustains; a tile alone on its CU cannot go faster than its own chain
    // of steps (about 350 clocks each: memory latency over the ring depth)
    const double fill = P + Q, mat = P * Q / 64 * 1.5;
    const double thr = fill > mat ? fill : mat;
    const double work = (double)tiles / 32.0 * (nk * thr + 1500.0);   // throughput: 32 CUs share
    const double lat = nk * (thr > 350.0 ? thr : 350.0) + 4000.0;      // latency of one tile
    const double cost = work > lat ? work : lat;
    if (cost < best_cost) { best_cost = cost; best = v; }
  }
  return best;
}

int out_extent(int in, int pad, int dil, int k, int stride) {
  long span = (long)dil * (k - 1) + 1;
  long t = (long)in + 2L * pad - span;
  if (t < 0) return 0;
  return (int)(t / stride) + 1;
}

struct PlanSizes {
  size_t layers_off, params_off, items_off, total;
  long n_items_total;
};

// per-layer, per-XCD tile counts; -1 on an unsupported list
int chain_layout(const q8_chain_layer* layers, int n, std::vector<ChainLayerDev>& L, PlanSizes* sz,
                 ChainHeader* hd) {
  Q8_REQUIRE(layers && n >= 1 && n <= 127, Q8_EINVAL);
  L.assign(n, ChainLayerDev{});
  const int N = layers[0].d.N;
  long n_items[kNumXcd] = {0};
  long region_words[kNumXcd];
  for (int x = 0; x < kNumXcd; ++x) region_words[x] = kRegionDone;
  for (int i = 0; i < n; ++i) {
    const q8_conv_desc& d = layers[i].d;
    Q8_REQUIRE(d.N == N && d.N >= 0 && d.H >= 1 && d.W >= 1 && d.C >= 1 && d.K >= 1 && d.R >= 1 &&
                   d.S >= 1 && d.stride_h >= 1 && d.stride_w >= 1 && d.pad_h >= 0 && d.pad_w >= 0 &&
                   d.dil_h >= 1 && d.dil_w >= 1, Q8_EINVAL);
    Q8_REQUIRE(chain_capable(d), Q8_EUNSUPPORTED);
    const int Ho = out_extent(d.H, d.pad_h, d.dil_h, d.R, d.stride_h);
    const int Wo = out_extent(d.W, d.pad_w, d.dil_w, d.S, d.stride_w);
    Q8_REQUIRE(Ho >= 1 && Wo >= 1, Q8_EUNSUPPORTED);
    const int s = layers[i].src_layer, r = layers[i].res_layer;
    Q8_REQUIRE(s >= -1 && s < i && r >= -1 && r < i, Q8_EINVAL);
    if (s >= 0) {     // reads exactly what layer s writes
      const q8_conv_desc& ds = layers[s].d;
      Q8_REQUIRE(layers[s].z_y == layers[i].z_x && ds.K == d.C &&
                     out_extent(ds.H, ds.pad_h, ds.dil_h, ds.R, ds.stride_h) == d.H &&
                     out_extent(ds.W, ds.pad_w, ds.dil_w, ds.S, ds.stride_w) == d.W, Q8_EINVAL);
    }
    Q8_REQUIRE((r >= 0) <= (layers[i].residual != nullptr), Q8_EINVAL);
    if (r >= 0) {
      const q8_conv_desc& dr = layers[r].d;
      Q8_REQUIRE(layers[r].z_y == layers[i].residual && dr.K == d.K &&
                     out_extent(dr.H, dr.pad_h, dr.dil_h, dr.R, dr.stride_h) == Ho &&
                     out_extent(dr.W, dr.pad_w, dr.dil_w, dr.S, dr.stride_w) == Wo, Q8_EINVAL);
    }
    // a tensor written in the chain is written once, and never one the chain reads from outside
    for (int j = 0; j < n; ++j) {
      Q8_REQUIRE(j == i || layers[j].z_y != layers[i].z_y, Q8_EINVAL);
      if (layers[j].src_layer < 0) Q8_REQUIRE((const int8_t*)layers[i].z_y != layers[j].z_x, Q8_EINVAL);
      if (layers[j].res_layer < 0 && layers[j].residual)
        Q8_REQUIRE((const int8_t*)layers[i].z_y != layers[j].residual, Q8_EINVAL);
    }
    int n0, nx;
    xcd_share(N, 0, &n0, &nx);                      // the largest share decides the tile
    const long Mx = (long)nx * Ho * Wo;
    Q8_REQUIRE(Mx <= 0xffffL * 64, Q8_EUNSUPPORTED);
    L[i].variant = pick_chain_variant(Mx, d.K, d.R * d.S * d.C, layers[i].variant);
    L[i].bp = kVariants[L[i].variant].bp;
    L[i].n_ctiles = (d.K + kVariants[L[i].variant].bc - 1) / kVariants[L[i].variant].bc;
    Q8_REQUIRE(L[i].n_ctiles <= 255, Q8_EUNSUPPORTED);
    L[i].src_layer = s;
    L[i].res_layer = r;
    for (int x = 0; x < kNumXcd; ++x) {
      xcd_share(N, x, &n0, &nx);
      const long m = (long)nx * Ho * Wo;
      L[i].n_ptiles[x] = (int)((m + L[i].bp - 1) / L[i].bp);
      Q8_REQUIRE(L[i].n_ptiles[x] <= 0xffff, Q8_EUNSUPPORTED);
      L[i].done_off[x] = (int)region_words[x];         // relative for now
      region_words[x] += L[i].n_ptiles[x];
      n_items[x] += (long)L[i].n_ptiles[x] * L[i].n_ctiles;
    }
  }
  long ws_words = kWsRegions;
  for (int x = 0; x < kNumXcd; ++x) {
    hd->head_off[x] = (int)ws_words + kRegionHead;
    for (int i = 0; i < n; ++i) L[i].done_off[x] += (int)ws_words;
    ws_words += (region_words[x] + 31) & ~31L;
    Q8_REQUIRE(ws_words < 0x3fffffffL, Q8_EUNSUPPORTED);
  }
  long total_items = 0;
  for (int x = 0; x < kNumXcd; ++x) {
    Q8_REQUIRE(n_items[x] < 0x7fffffffL, Q8_EUNSUPPORTED);
    hd->n_items[x] = (int)n_items[x];
    hd->item_off[x] = (int)total_items;
    total_items += n_items[x];
  }
  sz->layers_off = (sizeof(ChainHeader) + 255) & ~(size_t)255;
  sz->params_off = (sz->layers_off + (size_t)n * sizeof(ChainLayerDev) + 255) & ~(size_t)255;
  sz->items_off = (sz->params_off + (size_t)n * kNumXcd * sizeof(ConvParams) + 255) & ~(size_t)255;
  sz->total = (sz->items_off + (size_t)total_items * 4 + 255) & ~(size_t)255;
  sz->n_items_total = total_items;
  Q8_REQUIRE(sz->total < 0x7fffffffL, Q8_EUNSUPPORTED);
  hd->magic = kPlanMagic;
  hd->n_layers = n;
  hd->total_bytes = (int)sz->total;
  hd->ws_words = (int)ws_words;
  hd->layers_off = (int)sz->layers_off;
  hd->params_off = (int)sz->params_off;
  hd->items_off = (int)sz->items_off;
  return Q8_OK;
}

int chain_launch(const ChainHeader* hd, const void* plan_dev, int* ws, hipStream_t s) {
  static const hipError_t attr =
      hipFuncSetAttribute(reinterpret_cast<const void*>(conv_chain_kernel),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kChainLds + 64);
  if (attr != hipSuccess) return Q8_EHIP;
  const int words = hd->ws_words;
  // (a fill kernel, not a memset: the call may be recorded into a HIP graph)
  hipLaunchKernelGGL(chain_clear_kernel, dim3((words + 1023) / 1024), dim3(256), 0, s, ws, words);
  hipLaunchKernelGGL(conv_chain_kernel, dim3(hd->grid), dim3(kChainThreads), kChainLds + 64, s,
                     (const unsigned char*)plan_dev, ws, 0);
  return q8_launch_status();
}

// The workspace of q8_conv_chain_int8_static: device memory that belongs to the library's
// code object, one copy per GPU, never allocated or freed by a call.  In host code the
// array's name only stands for the symbol; its device address is looked up once per device.
constexpr size_t kStaticWsBytes = 1u << 20;
constexpr int kMaxDevices = 64;
__device__ __align__(256) int g_chain_scratch[kStaticWsBytes / 4];

int static_scratch(int** ws) {
  static std::mutex mu;
  static int* addr[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return Q8_EHIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_chain_scratch)) != hipSuccess || !p) return Q8_EHIP;
    addr[dev] = (int*)p;
  }
  *ws = addr[dev];
  return Q8_OK;
}

}  // namespace

extern "C" {

size_t q8_conv_chain_plan_bytes(const q8_chain_layer* layers, int n_layers) {
  std::vector<ChainLayerDev> L;
  PlanSizes sz;
  ChainHeader hd{};
  if (chain_layout(layers, n_layers, L, &sz, &hd) != Q8_OK) return 0;
  return sz.total;
}

int q8_conv_chain_plan(const q8_chain_layer* layers, int n_layers, void* plan_host,
                       size_t plan_bytes) {
  std::vector<ChainLayerDev> L;
  PlanSizes sz;
  ChainHeader hd{};
  const int rc = chain_layout(layers, n_layers, L, &sz, &hd);
  if (rc != Q8_OK) return rc;
  Q8_REQUIRE(plan_host && plan_bytes >= sz.total, Q8_EINVAL);
  unsigned char* out = (unsigned char*)plan_host;
  memset(out, 0, sz.total);
  int n_cu = 256;
  {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
      n_cu = prop.multiProcessorCount;
  }
  hd.grid = n_cu * kWgPerCu;
  memcpy(out, &hd, sizeof(hd));
  memcpy(out + sz.layers_off, L.data(), L.size() * sizeof(ChainLayerDev));
  ConvParams* params = (ConvParams*)(out + sz.params_off);
  int* items = (int*)(out + sz.items_off);
  const int N = layers[0].d.N;
  for (int i = 0; i < n_layers; ++i) {
    const q8_chain_layer& a = layers[i];
    const int Ho = out_extent(a.d.H, a.d.pad_h, a.d.dil_h, a.d.R, a.d.stride_h);
    const int Wo = out_extent(a.d.W, a.d.pad_w, a.d.dil_w, a.d.S, a.d.stride_w);
    for (int x = 0; x < kNumXcd; ++x) {
      int n0, nx;
      xcd_share(N, x, &n0, &nx);
      ConvParams& p = params[i * kNumXcd + x];
      if (nx == 0) continue;
      q8_conv_desc d = a.d;
      d.N = nx;
      bool empty = false;
      const int rc2 = q8::conv_fill_plain(
          &d, a.z_x + (size_t)n0 * d.H * d.W * d.C, a.z_w_packed, a.bias_i32, a.q_x, a.q_w, a.q_out,
          a.residual ? a.residual + (size_t)n0 * Ho * Wo * d.K : nullptr, a.q_res,
          a.z_y + (size_t)n0 * Ho * Wo * d.K, p, &empty);
      if (rc2 != Q8_OK) return rc2;
      p.n_ptiles = L[i].n_ptiles[x];
      p.n_ctiles = L[i].n_ctiles;
    }
  }
  // queue of XCD x: layer by layer, channel tile fastest (a pixel tile completes early)
  for (int x = 0; x < kNumXcd; ++x) {
    int* q = items + hd.item_off[x];
    int k = 0;
    for (int i = 0; i < n_layers; ++i)
      for (int pt = 0; pt < L[i].n_ptiles[x]; ++pt)
        for (int ct = 0; ct < L[i].n_ctiles; ++ct) q[k++] = pack_item(i, pt, ct);
  }
  return Q8_OK;
}

size_t q8_conv_chain_workspace_bytes(const void* plan_host) {
  const ChainHeader* hd = (const ChainHeader*)plan_host;
  if (!hd || hd->magic != kPlanMagic) return 0;
  return (size_t)hd->ws_words * 4;
}

int q8_conv_chain_int8(const void* plan_host, const void* plan_dev, void* workspace_dev,
                       size_t workspace_bytes, void* stream) {
  const ChainHeader* hd = (const ChainHeader*)plan_host;
  Q8_REQUIRE(hd && hd->magic == kPlanMagic && plan_dev && workspace_dev, Q8_EINVAL);
  Q8_REQUIRE(workspace_bytes >= (size_t)hd->ws_words * 4, Q8_EWORKSPACE);
  Q8_REQUIRE(q8_aligned(plan_dev, 256) && q8_aligned(workspace_dev, 16), Q8_EALIGN);
  return chain_launch(hd, plan_dev, (int*)workspace_dev, (hipStream_t)stream);
}

size_t q8_conv_chain_static_workspace_limit(void) { return kStaticWsBytes; }

int q8_conv_chain_int8_static(const void* plan_host, const void* plan_dev, void* stream) {
  const ChainHeader* hd = (const ChainHeader*)plan_host;
  Q8_REQUIRE(hd && hd->magic == kPlanMagic && plan_dev, Q8_EINVAL);
  Q8_REQUIRE((size_t)hd->ws_words * 4 <= kStaticWsBytes, Q8_EWORKSPACE);
  Q8_REQUIRE(q8_aligned(plan_dev, 256), Q8_EALIGN);
  int* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != Q8_OK) return rc;
  return chain_launch(hd, plan_dev, ws, (hipStream_t)stream);
}

int q8_conv_chain_static_status(int32_t* status_host) {
  Q8_REQUIRE(status_host, Q8_EINVAL);
  int* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != Q8_OK) return rc;
  return hipMemcpy(status_host, ws + kWsStatus, 4, hipMemcpyDeviceToHost) == hipSuccess
             ? Q8_OK : Q8_EHIP;
}

int q8_conv_chain_supported(const q8_conv_desc* d) { return d && chain_capable(*d) ? 1 : 0; }

}  // extern "C"
