// C ABI of the SFC library: plans, argument checks, buffer layout, stage sequencing.
// Every numeric step runs in the kernels of sfc_kernels.hip; this file only
// validates, lays out buffers and launches.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/sfc.h"
#include "sfc_internal.hpp"
#include "sfc_mfma_input.hpp"

using sfc::FilterViews;
using sfc::Geometry;

struct sfc_plan_s {
  sfc_conv_desc d;
  Geometry g;
  int esz;  // bytes per transform-domain operand: 2 exact, 1 requantized
  // filter buffer layout (byte offsets)
  size_t off_U, off_dequant, off_inv_sw, off_inv_sx, off_wscale, off_input_tab, off_dq_single, off_U_single,
      filter_bytes;
  // workspace layout
  size_t off_V, off_M, workspace_bytes;
  std::vector<float> sx, sw;  // [P], [P][Cout]
  bool scales_set;
  std::vector<float> staging;  // host image of the float tables of the filter buffer
  void* filter_dev;
  bool filter_ready;
  int quad_filters;  // filters covered by the regrouped filter operand (0: none)
  int dq_filters;    // filters in the [filter][processing position] dequantization table (0: none)
  bool quad16;       // filter operand in groups of 16 filters (sfc_quad16.hpp, sfc_splitk.hip)
  bool splitk;       // fused path: input channels split over the waves of a workgroup
  float inv_y;  // 1 / output scale (SFC_OUT_I8_RELU), 0: not set
};

// Workspace of sfc_conv2d_nchw_static: part of the code object, one copy per GPU.  In host
// code this name is only a handle for hipGetSymbolAddress; the device address it yields is
// what kernels and copies get.
static __device__ __align__(256) unsigned char scratch[SFC_STATIC_WORKSPACE_BYTES];

namespace {

// Device address of `scratch` on the current device, looked up once per device; nullptr if
// the runtime refuses.
void* static_workspace() {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* addr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return nullptr;
    }
    addr[dev] = p;
  }
  return addr[dev];
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

FilterViews views(const sfc_plan_s* p, void* filter_dev) {
  char* b = static_cast<char*>(filter_dev);
  FilterViews f;
  f.U = b + p->off_U;
  f.dequant = reinterpret_cast<float*>(b + p->off_dequant);
  f.inv_sw = reinterpret_cast<float*>(b + p->off_inv_sw);
  f.inv_sx = reinterpret_cast<float*>(b + p->off_inv_sx);
  f.wscale = reinterpret_cast<float*>(b + p->off_wscale);
  f.input_tab = reinterpret_cast<unsigned char*>(b + p->off_input_tab);
  f.dequant_single = reinterpret_cast<float*>(b + p->off_dq_single);
  f.U_single = b + p->off_U_single;
  return f;
}

bool alg_is_7x7(int alg) { return alg == SFC_ALG_7X7_P132 || alg == SFC_ALG_7X7_P144; }

// Tile grid and padded extents of a description whose algorithm is fixed.  False when the
// tile count leaves the 32-bit range the kernels index with.
bool make_geometry(const sfc_conv_desc& d, Geometry* out) {
  Geometry g;
  g.N = d.N; g.Cin = d.Cin; g.Cout = d.Cout; g.H = d.H; g.W = d.W;
  g.alg = d.alg;
  const int mt = sfc::alg_tile(d.alg);
  g.th = (d.H + mt - 1) / mt;
  g.tw = (d.W + mt - 1) / mt;
  const int64_t strips = (int64_t)d.N * g.th;
  const int64_t T = strips * g.tw;
  if (T > (1ll << 30)) return false;
  g.strips = (int)strips;
  g.T = (int)T;
  g.Tp = (int)((T + 15) / 16 * 16);
  g.Cp = (d.Cin + 63) / 64 * 64;
  g.Kp = (d.Cout + 15) / 16 * 16;
  g.P = sfc::alg_points(d.alg);
  g.qmax = (float)((1 << ((d.transform_bits ? d.transform_bits : 8) - 1)) - 1);
  *out = g;
  return true;
}

// SFC_ALG_AUTO (3x3 filters), from per-layer timings of the ResNet shapes on one MI355X.
// Requantized mode: SFC-4's 4x4 tiles -- 46 points per tile keep two or three workgroups on a
// compute unit and the filter operand small, which outweighs even the ragged tiles of 14x14
// and 7x7 maps (256 channels at 14x14: 28.9 us against 47.5 us for 7x7 tiles at batch 64,
// 49.1 against 55.8 at batch 128; 512 channels at 7x7, batch 64: 31.2 against 38.9) -- except
// on 7x7 maps, which one 7x7 tile covers exactly, once the layer has at least 96 K (tile,
// filter) pairs: then the 31 % of surplus outputs of the ragged 4x4 tiles cost more than the
// larger point set (512 channels at 7x7, batch 256: 64.5 us with 7x7 tiles against 78.8).
// Exact mode: 6x6 tiles, the form Sec. 4 and the 3.68x figure are about.
int choose_alg(const sfc_conv_desc& d) {
  if (d.mode == SFC_MODE_EXACT) return SFC_ALG_6X6_P88;
  if (d.H == 7 && d.W == 7) {
    const int64_t pairs = (int64_t)d.N * (d.H / 7) * (d.W / 7) * d.Cout;
    // (with 512 and more channels the 7x7 tiles go through the staged path, which is ahead
    // from batch 128 on: 512 channels, 30.9 against 46.6 us with 4x4 tiles; batch 64: 28.1
    // against 26.0)
    if (pairs >= (d.Cin >= 512 ? 56 : 96) * 1024) return SFC_ALG_7X7_P132;
  }
  return SFC_ALG_4X4_P46;
}

// SFC_PATH_AUTO: one kernel where the layer allows it, else input transform + fused
// product/output kernel, else the staged path (exact mode, channel counts the fused
// kernel does not take).
int choose_path(const sfc_conv_desc& d, const Geometry& g) {
  if (d.mode != SFC_MODE_REQUANT_I8) return SFC_PATH_STAGED;
  // (with more than 128 channels the single-kernel path repeats the input transform for
  // every 64 filters and is slower than two kernels: 51 against 30 us for 256 channels on
  // 14x14 maps at batch 64; it stays available on request)
  if (g.Cp <= 128 && sfc::single_supported(g)) return SFC_PATH_SINGLE;
  // 7x7 tiles on 7x7 maps with 512 and more channels: the fused kernel would stream its
  // operands from L2 eight times over; the products as batched GEMMs through HBM are faster
  // (64.0 against 77.0 us at batch 256)
  const bool gemm = alg_is_7x7(d.alg) && d.H < 14 && d.Cin >= 512;
  if (!gemm && sfc::fused_quad_supported(g)) return SFC_PATH_FUSED;
  return SFC_PATH_STAGED;
}

}  // namespace

extern "C" {

const char* sfc_status_string(sfc_status s) {
  switch (s) {
    case SFC_OK: return "ok";
    case SFC_EINVAL: return "invalid argument";
    case SFC_EUNSUPPORTED: return "unsupported configuration";
    case SFC_ENOMEM: return "host allocation failed";
    case SFC_ENOTREADY: return "scales or filter not set";
    case SFC_EHIP: return "HIP runtime or launch failure";
    case SFC_EWORKSPACE: return "device buffer smaller than the plan needs";
  }
  return "unknown status";
}

sfc_status sfc_plan(const sfc_conv_desc* desc, sfc_plan_t** out) {
  if (!desc || !out) return SFC_EINVAL;
  *out = nullptr;
  sfc_conv_desc d = *desc;
  if (d.N <= 0 || d.Cin <= 0 || d.Cout <= 0 || d.H <= 0 || d.W <= 0) return SFC_EINVAL;
  if (d.alg < SFC_ALG_AUTO || d.alg > SFC_ALG_4X4_7X7_P196) return SFC_EINVAL;
  if (d.mode != SFC_MODE_EXACT && d.mode != SFC_MODE_REQUANT_I8) return SFC_EINVAL;
  if (d.out != SFC_OUT_F32 && d.out != SFC_OUT_I32 && d.out != SFC_OUT_I8_RELU) return SFC_EINVAL;
  if (d.path < SFC_PATH_AUTO || d.path > SFC_PATH_SINGLE) return SFC_EINVAL;
  if ((d.flags & ~SFC_FLAG_EXACT_WIDE) != 0) return SFC_EINVAL;
  if (d.per_channel_wscale != 0 && d.per_channel_wscale != 1) return SFC_EINVAL;
  if (d.transform_bits != 0 && (d.transform_bits < 2 || d.transform_bits > 8)) return SFC_EINVAL;
  if (d.transform_bits != 0 && d.mode != SFC_MODE_REQUANT_I8) return SFC_EUNSUPPORTED;
  if (d.out == SFC_OUT_I32 && d.mode != SFC_MODE_EXACT) return SFC_EUNSUPPORTED;
  if (d.out == SFC_OUT_I8_RELU && d.mode != SFC_MODE_REQUANT_I8) return SFC_EUNSUPPORTED;
  if (d.path > SFC_PATH_STAGED && d.mode != SFC_MODE_REQUANT_I8) return SFC_EUNSUPPORTED;
  // Cout: one workgroup row per filter (filter transform, abs-max) must fit a launch grid
  if (d.W > 1024 || d.H > (1 << 20) || d.Cin > (1 << 16) || d.Cout > 65520)
    return SFC_EUNSUPPORTED;
  if (d.alg == SFC_ALG_AUTO) d.alg = choose_alg(d);
  if (d.mode == SFC_MODE_EXACT && !(d.flags & SFC_FLAG_EXACT_WIDE) &&
      d.Cin > (d.alg >= SFC_ALG_4X4_7X7_P184 ? 74 : d.alg >= SFC_ALG_6X6_5X5_P184 ? 145 : 404))
    return SFC_EUNSUPPORTED;

  Geometry g;
  if (!make_geometry(d, &g)) return SFC_EUNSUPPORTED;
  if (d.path == SFC_PATH_AUTO) d.path = choose_path(d, g);
  if (d.path == SFC_PATH_FUSED && !sfc::fused_quad_supported(g)) return SFC_EUNSUPPORTED;
  if (d.path == SFC_PATH_SINGLE && !sfc::single_supported(g)) return SFC_EUNSUPPORTED;

  sfc_plan_s* p = new (std::nothrow) sfc_plan_s();
  if (!p) return SFC_ENOMEM;
  p->d = d;
  p->g = g;
  p->esz = d.mode == SFC_MODE_EXACT ? 2 : 1;
  const size_t PK = (size_t)g.P * g.Kp;
  size_t off = 0;
  p->off_U = off;        off = align_up(off + PK * g.Cp * p->esz, 256);
  p->off_dequant = off;  off = align_up(off + PK * sizeof(float), 256);
  p->off_inv_sw = off;   off = align_up(off + PK * sizeof(float), 256);
  p->off_inv_sx = off;   off = align_up(off + g.P * sizeof(float), 256);
  p->off_wscale = off;   off = align_up(off + g.Kp * sizeof(float), 256);
  p->off_input_tab = off;
  if (d.mode == SFC_MODE_REQUANT_I8 && (d.alg == SFC_ALG_4X4_P46 || d.alg == SFC_ALG_4X4_P49))
    off = align_up(off + sfc::kInputTabBytes, 256);
  if (d.mode == SFC_MODE_REQUANT_I8 && sfc::image_input_supported(g))
    off = align_up(off + sfc::image_table_bytes(g), 256);
  if (d.mode == SFC_MODE_REQUANT_I8 && sfc::rows_table_offset(g) != ~0u)
    off = align_up(off + sfc::kRowsTabBytes, 256);
  p->off_dq_single = off;
  p->off_U_single = off;
  p->quad_filters = 0;
  p->splitk = d.path == SFC_PATH_FUSED && !sfc::quad16_supported(g) && sfc::splitk_supported(g);
  p->quad16 = p->splitk || (d.path == SFC_PATH_FUSED && sfc::quad16_supported(g)) ||
              (d.path == SFC_PATH_SINGLE && (sfc::single16_supported(g) || sfc::single16k_supported(g)));
  if (d.path == SFC_PATH_SINGLE) p->quad_filters = p->quad16 ? g.Kp : (g.Cout + 63) / 64 * 64;
  if (d.path == SFC_PATH_FUSED)
    p->quad_filters = p->splitk   ? sfc::splitk_filter_count(g)
                      : p->quad16 ? sfc::quad16_filter_count(g)
                                  : sfc::quad_filter_count(g);
  // the staged output transform reads the same [filter][position] table as the fused kernels
  p->dq_filters = p->quad_filters;
  if (d.path == SFC_PATH_STAGED && d.mode == SFC_MODE_REQUANT_I8) p->dq_filters = g.Kp;
  // the kernels take the points in groups of four: positions up to a multiple of 4
  const size_t pp = (size_t)(g.P + 3) / 4 * 4;
  if (p->dq_filters > 0) {
    off = align_up(off + (size_t)p->dq_filters * pp * sizeof(float), 256);
    p->off_U_single = off;
  }
  if (p->quad_filters > 0) off = align_up(off + (size_t)p->quad_filters * pp * g.Cp, 256);
  p->filter_bytes = off;
  off = 0;
  p->off_V = off;
  // the single-kernel path keeps V on chip; its workspace only serves calibration
  if (d.path != SFC_PATH_SINGLE) off = align_up(off + (size_t)g.P * g.Tp * g.Cp * p->esz, 256);
  p->off_M = off;
  if (d.path == SFC_PATH_STAGED) off = align_up(off + (size_t)g.P * g.Tp * g.Kp * 4, 256);
  // calibration scratch (abs-max tables) must fit as well
  const size_t calib = align_up((size_t)g.P * (size_t)(g.Cout > 1 ? g.Cout : 1) * 4, 256);
  p->workspace_bytes = off > calib ? off : calib;
  p->scales_set = false;
  p->filter_dev = nullptr;
  p->filter_ready = false;
  p->inv_y = 0.0f;
  *out = p;
  return SFC_OK;
}

void sfc_plan_destroy(sfc_plan_t* plan) { delete plan; }

sfc_status sfc_plan_choice(const sfc_plan_t* plan, int32_t* alg, int32_t* path) {
  if (!plan) return SFC_EINVAL;
  if (alg) *alg = plan->d.alg;
  if (path) *path = plan->d.path;
  return SFC_OK;
}

sfc_status sfc_plan_sizes(const sfc_plan_t* plan, size_t* filter_bytes, size_t* workspace_bytes,
                          int32_t* P, int64_t* tiles) {
  if (!plan) return SFC_EINVAL;
  if (filter_bytes) *filter_bytes = plan->filter_bytes;
  if (workspace_bytes) *workspace_bytes = plan->workspace_bytes;
  if (P) *P = plan->g.P;
  if (tiles) *tiles = plan->g.T;
  return SFC_OK;
}

sfc_status sfc_set_point_scales(sfc_plan_t* plan, const float* sx_host, const float* sw_host) {
  if (!plan || !sx_host || !sw_host) return SFC_EINVAL;
  if (plan->d.mode != SFC_MODE_REQUANT_I8) return SFC_EUNSUPPORTED;
  const int P = plan->g.P, K = plan->g.Cout;
  auto ok = [](float s) {
    if (!(s > 0.0f) || !std::isfinite(s)) return false;
    const float inv = 1.0f / s;
    return std::isfinite(inv) && inv > 0.0f;
  };
  for (int p = 0; p < P; ++p)
    if (!ok(sx_host[p])) return SFC_EINVAL;
  for (size_t i = 0; i < (size_t)P * K; ++i)
    if (!ok(sw_host[i])) return SFC_EINVAL;
  try {
    plan->sx.assign(sx_host, sx_host + P);
    plan->sw.assign(sw_host, sw_host + (size_t)P * K);
  } catch (...) {
    return SFC_ENOMEM;
  }
  plan->scales_set = true;
  plan->filter_ready = false;
  return SFC_OK;
}

sfc_status sfc_group_scales(const sfc_plan_t* plan, int32_t act_granularity,
                            int32_t filter_granularity, float* sx_host, float* sw_host) {
  if (!plan || !sx_host || !sw_host) return SFC_EINVAL;
  if (act_granularity != SFC_ACT_PER_TENSOR && act_granularity != SFC_ACT_PER_POINT)
    return SFC_EINVAL;
  if (filter_granularity < SFC_FILTER_PER_CHANNEL || filter_granularity > SFC_FILTER_PER_CHANNEL_POINT)
    return SFC_EINVAL;
  const int P = plan->g.P, K = plan->g.Cout;
  if (act_granularity == SFC_ACT_PER_TENSOR) {
    float m = sx_host[0];
    for (int p = 1; p < P; ++p) m = sx_host[p] > m ? sx_host[p] : m;
    for (int p = 0; p < P; ++p) sx_host[p] = m;
  }
  if (filter_granularity == SFC_FILTER_PER_CHANNEL) {
    for (int k = 0; k < K; ++k) {
      float m = sw_host[k];
      for (int p = 1; p < P; ++p) m = sw_host[(size_t)p * K + k] > m ? sw_host[(size_t)p * K + k] : m;
      for (int p = 0; p < P; ++p) sw_host[(size_t)p * K + k] = m;
    }
  } else if (filter_granularity == SFC_FILTER_PER_POINT) {
    for (int p = 0; p < P; ++p) {
      float* row = sw_host + (size_t)p * K;
      float m = row[0];
      for (int k = 1; k < K; ++k) m = row[k] > m ? row[k] : m;
      for (int k = 0; k < K; ++k) row[k] = m;
    }
  }
  return SFC_OK;
}

sfc_status sfc_set_output_scale(sfc_plan_t* plan, float y_scale) {
  if (!plan) return SFC_EINVAL;
  if (plan->d.out != SFC_OUT_I8_RELU) return SFC_EUNSUPPORTED;
  if (!(y_scale > 0.0f) || !std::isfinite(y_scale)) return SFC_EINVAL;
  const float inv = 1.0f / y_scale;
  if (!std::isfinite(inv) || !(inv > 0.0f)) return SFC_EINVAL;
  plan->inv_y = inv;
  return SFC_OK;
}

sfc_status sfc_transform_filter(sfc_plan_t* plan, const int8_t* w_dev, const float* wscale_host,
                                void* filter_dev, size_t filter_bytes, void* stream) {
  if (!plan || !w_dev || !wscale_host || !filter_dev) return SFC_EINVAL;
  if (!aligned16(w_dev) || !aligned16(filter_dev)) return SFC_EINVAL;
  if (filter_bytes < plan->filter_bytes) return SFC_EWORKSPACE;
  const Geometry& g = plan->g;
  const bool requant = plan->d.mode == SFC_MODE_REQUANT_I8;
  if (requant && !plan->scales_set) return SFC_ENOTREADY;
  for (int k = 0; k < (plan->d.per_channel_wscale ? g.Cout : 1); ++k)
    if (!(wscale_host[k] > 0.0f) || !std::isfinite(wscale_host[k])) return SFC_EINVAL;

  // host image of the float tables: [dequant | inv_sw | inv_sx | wscale], contiguous
  // from off_dequant to filter_bytes
  const bool quad = plan->quad_filters > 0;
  const size_t table_bytes =
      (plan->dq_filters > 0 ? plan->off_U_single : plan->filter_bytes) - plan->off_dequant;
  try {
    plan->staging.assign(table_bytes / sizeof(float), 0.0f);
  } catch (...) {
    return SFC_ENOMEM;
  }
  auto table = [&](size_t off) { return plan->staging.data() + (off - plan->off_dequant) / sizeof(float); };
  float* dequant = table(plan->off_dequant);
  float* inv_sw = table(plan->off_inv_sw);
  float* inv_sx = table(plan->off_inv_sx);
  float* wscale = table(plan->off_wscale);
  for (int k = 0; k < g.Kp; ++k)
    wscale[k] = k < g.Cout ? wscale_host[plan->d.per_channel_wscale ? k : 0] : 0.0f;
  // the output transform yields den * y
  const double den = (g.alg == SFC_ALG_4X4_P46 || g.alg == SFC_ALG_4X4_P49) ? 16.0 : 36.0;
  for (int p = 0; p < g.P; ++p) {
    inv_sx[p] = requant ? 1.0f / plan->sx[p] : 1.0f;
    for (int k = 0; k < g.Kp; ++k) {
      float dq = 0.0f, inv = 1.0f;
      if (requant && k < g.Cout) {
        const float sw = plan->sw[(size_t)p * g.Cout + k];
        inv = 1.0f / sw;
        dq = (float)((double)plan->sx[p] * (double)sw * (double)wscale[k] / den);
      }
      dequant[(size_t)p * g.Kp + k] = dq;
      inv_sw[(size_t)p * g.Kp + k] = inv;
    }
  }
  if (plan->off_dq_single > plan->off_input_tab) {
    unsigned char* tab = reinterpret_cast<unsigned char*>(table(plan->off_input_tab));
    if (g.alg == SFC_ALG_4X4_P46 || g.alg == SFC_ALG_4X4_P49) sfc::build_input_table(g.alg, inv_sx, tab);
    if (sfc::image_input_supported(g))
      sfc::build_image_input_table(g, inv_sx, tab + sfc::image_table_offset(g));
    if (sfc::rows_table_offset(g) != ~0u) sfc::build_rows_table(g.alg, inv_sx, tab + sfc::rows_table_offset(g));
  }
  if (plan->dq_filters > 0) {
    const int pp = (g.P + 3) / 4 * 4;
    std::vector<int> pt(pp, -1);
    sfc::single_point_order(plan->d.alg, pt.data());
    float* dqs = table(plan->off_dq_single);
    if (plan->quad16) {
      // [group of 16 filters][processing position][lane quarter q][i]: filter 16*fg + 4*i + q
      for (int k = 0; k < g.Cout; ++k) {
        const int fg = k >> 4, i = (k & 15) >> 2, q = k & 3;
        for (int j = 0; j < pp; ++j)
          dqs[((size_t)fg * pp + j) * 16 + 4 * q + i] =
              pt[j] < 0 ? 0.0f : dequant[(size_t)pt[j] * g.Kp + k];
      }
    } else {
      // [filter][processing position]; filters beyond Cout stay zero
      for (int k = 0; k < g.Cout; ++k)
        for (int j = 0; j < pp; ++j)
          dqs[(size_t)k * pp + j] = pt[j] < 0 ? 0.0f : dequant[(size_t)pt[j] * g.Kp + k];
    }
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // the kernels of this plan's path that need more than the default 64 KB of dynamic LDS
  if (requant && sfc::prepare_kernels(plan->d.path, plan->d.out, g) != hipSuccess) return SFC_EHIP;
  if (hipMemcpyAsync(static_cast<char*>(filter_dev) + plan->off_dequant, plan->staging.data(),
                     table_bytes, hipMemcpyHostToDevice, s) != hipSuccess)
    return SFC_EHIP;
  const FilterViews f = views(plan, filter_dev);
  if (sfc::launch_filter_transform(plan->d.mode, g, w_dev, f, s) != hipSuccess)
    return SFC_EHIP;
  if (quad && (plan->quad16 ? sfc::launch_repack_filter16(g, plan->quad_filters, f.U, f.U_single, s)
                            : sfc::launch_repack_filter(g, plan->quad_filters, f.U, f.U_single, s)) !=
                  hipSuccess)
    return SFC_EHIP;
  plan->filter_dev = filter_dev;
  plan->filter_ready = true;
  return SFC_OK;
}

sfc_status sfc_conv2d_stages(const sfc_plan_t* plan, const int8_t* x_dev, float x_scale,
                             void* y_dev, void* workspace_dev, size_t workspace_bytes, void* stream,
                             int32_t stage_mask) {
  if (!plan || !x_dev || !y_dev || !workspace_dev) return SFC_EINVAL;
  if (!aligned16(x_dev) || !aligned16(y_dev) || !aligned16(workspace_dev)) return SFC_EINVAL;
  if (!(x_scale > 0.0f) || !std::isfinite(x_scale)) return SFC_EINVAL;
  if (stage_mask <= 0 || stage_mask > SFC_STAGE_ALL) return SFC_EINVAL;
  if (workspace_bytes < plan->workspace_bytes) return SFC_EWORKSPACE;
  if (!plan->filter_ready) return SFC_ENOTREADY;
  if (plan->d.out == SFC_OUT_I8_RELU && plan->inv_y == 0.0f) return SFC_ENOTREADY;
  const bool fused = plan->d.path == SFC_PATH_FUSED;
  if (plan->d.path == SFC_PATH_SINGLE) {
    if (stage_mask != SFC_STAGE_ALL) return SFC_EINVAL;  // one kernel: no stage runs alone
    const FilterViews f = views(plan, plan->filter_dev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (!plan->quad16)
      e = sfc::launch_single_conv(plan->d.out, plan->g, x_dev, f, x_scale, plan->inv_y, y_dev, s);
    else if (plan->g.Cp <= 128)
      e = sfc::launch_single16(plan->d.out, plan->g, x_dev, f, x_scale, plan->inv_y, y_dev, s);
    else
      e = sfc::launch_single16k(plan->d.out, plan->g, x_dev, f, x_scale, plan->inv_y, y_dev, s);
    if (e != hipSuccess) return SFC_EHIP;
    return SFC_OK;
  }
  const int tail = stage_mask & (SFC_STAGE_PRODUCT | SFC_STAGE_OUTPUT);
  if (fused && tail != 0 && tail != (SFC_STAGE_PRODUCT | SFC_STAGE_OUTPUT)) return SFC_EINVAL;
  const Geometry& g = plan->g;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const FilterViews f = views(plan, plan->filter_dev);
  char* ws = static_cast<char*>(workspace_dev);
  void* V = ws + plan->off_V;
  if (stage_mask & SFC_STAGE_INPUT) {
    if (sfc::launch_input_transform(plan->d.mode, g, x_dev, V, f.inv_sx, f.input_tab, s) !=
        hipSuccess)
      return SFC_EHIP;
  }
  if (fused) {
    if (tail &&
        (plan->splitk   ? sfc::launch_splitk(plan->d.out, g, V, f, x_scale, plan->inv_y, y_dev, s)
         : plan->quad16 ? sfc::launch_quad16(plan->d.out, g, V, f, x_scale, plan->inv_y, y_dev, s)
                        : sfc::launch_fused_quad(plan->d.out, g, V, f, x_scale, plan->inv_y, y_dev, s)) !=
            hipSuccess)
      return SFC_EHIP;
    return SFC_OK;
  }
  int32_t* M = reinterpret_cast<int32_t*>(ws + plan->off_M);
  if (stage_mask & SFC_STAGE_PRODUCT) {
    if (sfc::launch_product(plan->d.mode, g, V, f.U, M, s) != hipSuccess) return SFC_EHIP;
  }
  if (stage_mask & SFC_STAGE_OUTPUT) {
    if (sfc::launch_output_transform(plan->d.mode, plan->d.out, g, M, f, x_scale,
                                     plan->inv_y, y_dev, s) != hipSuccess)
      return SFC_EHIP;
  }
  return SFC_OK;
}

sfc_status sfc_conv2d_nchw(const sfc_plan_t* plan, const int8_t* x_dev, float x_scale, void* y_dev,
                           void* workspace_dev, size_t workspace_bytes, void* stream) {
  return sfc_conv2d_stages(plan, x_dev, x_scale, y_dev, workspace_dev, workspace_bytes, stream,
                           SFC_STAGE_ALL);
}

sfc_status sfc_conv2d_nchw_static(const sfc_plan_t* plan, const int8_t* x_dev, float x_scale,
                                  void* y_dev, void* stream) {
  if (!plan) return SFC_EINVAL;
  if (plan->workspace_bytes > SFC_STATIC_WORKSPACE_BYTES) return SFC_EWORKSPACE;
  void* ws = static_workspace();
  if (!ws) return SFC_EHIP;
  return sfc_conv2d_stages(plan, x_dev, x_scale, y_dev, ws, SFC_STATIC_WORKSPACE_BYTES, stream,
                           SFC_STAGE_ALL);
}

sfc_status sfc_tap_info(const sfc_plan_t* plan, const void* workspace_dev, int32_t which,
                        const void** ptr, int32_t* elem_bytes, int64_t dims[5],
                        int64_t strides[5]) {
  if (!plan || !ptr || !elem_bytes || !dims || !strides) return SFC_EINVAL;
  const Geometry& g = plan->g;
  const char* ws = static_cast<const char*>(workspace_dev);
  switch (which) {
    case 0:
      if (!workspace_dev) return SFC_EINVAL;
      if (plan->d.path == SFC_PATH_SINGLE) return SFC_EUNSUPPORTED;
      *ptr = ws + plan->off_V;
      *elem_bytes = plan->esz;
      dims[0] = g.P; dims[1] = g.Tp; dims[2] = 1; dims[3] = g.Cp; dims[4] = 1;
      strides[0] = (int64_t)g.Tp * g.Cp; strides[1] = g.Cp; strides[2] = 0; strides[3] = 1;
      strides[4] = 0;
      return SFC_OK;
    case 1:
      if (!plan->filter_ready) return SFC_ENOTREADY;
      *ptr = static_cast<const char*>(plan->filter_dev) + plan->off_U;
      *elem_bytes = plan->esz;
      dims[0] = g.P; dims[1] = g.Kp; dims[2] = 1; dims[3] = g.Cp; dims[4] = 1;
      strides[0] = (int64_t)g.Kp * g.Cp; strides[1] = g.Cp; strides[2] = 0; strides[3] = 1;
      strides[4] = 0;
      return SFC_OK;
    case 2:
      if (!workspace_dev) return SFC_EINVAL;
      if (plan->d.path != SFC_PATH_STAGED) return SFC_EUNSUPPORTED;
      *ptr = ws + plan->off_M;
      *elem_bytes = plan->d.mode == SFC_MODE_REQUANT_I8 ? sfc::m_sum_bytes(g) : 4;
      dims[0] = g.P;
      strides[0] = (int64_t)g.Tp * g.Kp;
      if (plan->d.mode == SFC_MODE_REQUANT_I8) {
        // [P][tile block][filter quad][16 tiles][4 filters]
        dims[1] = g.Tp / 16; dims[2] = 16; dims[3] = g.Kp / 4; dims[4] = 4;
        strides[1] = (int64_t)g.Kp * 16; strides[2] = 4; strides[3] = 64; strides[4] = 1;
      } else {
        dims[1] = g.Tp; dims[2] = 1; dims[3] = g.Kp; dims[4] = 1;
        strides[1] = g.Kp; strides[2] = 0; strides[3] = 1; strides[4] = 0;
      }
      return SFC_OK;
    default:
      return SFC_EINVAL;
  }
}

sfc_status sfc_stream_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream) {
  if (!dst_dev || !src_dev) return SFC_EINVAL;
  if (!aligned16(dst_dev) || !aligned16(src_dev) || (bytes & 15u) != 0) return SFC_EINVAL;
  if (sfc::launch_stream_copy(dst_dev, src_dev, bytes, static_cast<hipStream_t>(stream)) !=
      hipSuccess)
    return SFC_EHIP;
  return SFC_OK;
}

static sfc_status maxima_to_scales(const int32_t* dev, size_t count, float qmax, hipStream_t s,
                                   float* out) {
  std::vector<int32_t> host;
  try {
    host.resize(count);
  } catch (...) {
    return SFC_ENOMEM;
  }
  if (hipMemcpyAsync(host.data(), dev, count * sizeof(int32_t), hipMemcpyDeviceToHost, s) !=
      hipSuccess)
    return SFC_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return SFC_EHIP;
  for (size_t i = 0; i < count; ++i)
    out[i] = host[i] == 0 ? 1.0f : (float)host[i] / qmax;
  return SFC_OK;
}

sfc_status sfc_calibrate_act_scales(const sfc_plan_t* plan, const int8_t* x_dev, int32_t n_images,
                                    void* workspace_dev, size_t workspace_bytes, void* stream,
                                    float* sx_host_out) {
  if (!plan || !x_dev || !workspace_dev || !sx_host_out) return SFC_EINVAL;
  if (!aligned16(x_dev) || !aligned16(workspace_dev)) return SFC_EINVAL;
  if (n_images <= 0 || n_images > plan->g.N) return SFC_EINVAL;
  if (workspace_bytes < plan->workspace_bytes) return SFC_EWORKSPACE;
  Geometry g = plan->g;
  g.N = n_images;
  g.strips = n_images * g.th;
  g.T = g.strips * g.tw;
  g.Tp = (g.T + 15) / 16 * 16;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* maxima = static_cast<int32_t*>(workspace_dev);
  if (sfc::launch_act_absmax(g, x_dev, maxima, s) != hipSuccess) return SFC_EHIP;
  return maxima_to_scales(maxima, g.P, g.qmax, s, sx_host_out);
}

sfc_status sfc_calibrate_filter_scales(const sfc_plan_t* plan, const int8_t* w_dev,
                                       void* workspace_dev, size_t workspace_bytes, void* stream,
                                       float* sw_host_out) {
  if (!plan || !w_dev || !workspace_dev || !sw_host_out) return SFC_EINVAL;
  if (!aligned16(w_dev) || !aligned16(workspace_dev)) return SFC_EINVAL;
  if (workspace_bytes < plan->workspace_bytes) return SFC_EWORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  int32_t* maxima = static_cast<int32_t*>(workspace_dev);
  if (sfc::launch_filter_absmax(plan->g, w_dev, maxima, s) != hipSuccess)
    return SFC_EHIP;
  return maxima_to_scales(maxima, (size_t)plan->g.P * plan->g.Cout, plan->g.qmax, s, sw_host_out);
}

}  // extern "C"
