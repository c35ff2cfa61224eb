// Launch side of the SFC-4 products + output-transform kernel (sfc_quad16.hpp): limits, the
// regrouping of the filter operand and the dispatch over channel chunks and output type.
#include "sfc_quad16.hpp"

namespace sfc {

// waves per workgroup = groups of 16 filters per workgroup
constexpr int kQuad16Waves = 4;

bool quad16_supported(const Geometry& g) {
  if (g.alg != 4 && g.alg != 5) return false;
  const int kc = g.Cp / 64;
  // Up to four channel chunks: with eight a wave's filter operand stream (8 KiB per point) is
  // not hidden behind its own arithmetic (sfc_splitk.hip and the one-pair-per-lane kernel take
  // those layers).
  if (kc != 1 && kc != 2 && kc != 4) return false;
  // A wave takes 256 (tile, filter) pairs: with fewer than one wave per SIMD of the chip the
  // one-pair-per-lane kernel, whose waves take 64, fills it better.
  if ((long long)(g.Tp / 16) * ((g.Cout + 15) / 16) < 1024) return false;
  const long long fgroups = quad16_filter_count(g) / 16;
  const long long ybytes = 4ll * g.N * g.Cout * g.H * g.W;
  const long long vbytes = (long long)g.P * g.Tp * g.Cp;
  const long long ubytes = fgroups * 16 * ((g.P + 3) / 4 * 4) * g.Cp;
  const long long lim = 1ll << 31;
  return ybytes < lim && vbytes < lim && ubytes < lim;
}

// filters covered by the regrouped operand: Cout rounded up to whole workgroups
int quad16_filter_count(const Geometry& g) {
  const int per_wg = 16 * kQuad16Waves;
  return (g.Cout + per_wg - 1) / per_wg * per_wg;
}

// Filter operand from the canonical U[p][k][c]: block (filter group fg, position j, channel
// chunk kc) is one KiB; lane l holds the 16 channels 64*kc + 16*(l/16).. of point pt[j] for
// filter 16*fg + 4*(r%4) + r/4, r = l%16 (row r of the MFMA operand).  Filters beyond Kp and
// positions without a point are zero.
template <int ALG>
__global__ __launch_bounds__(64) void repack_filter16_kernel(const int8_t* __restrict__ U,
                                                             int8_t* __restrict__ U16, Geometry g) {
  constexpr int PP = Order<ALG>::PP;
  constexpr Order<ALG> order{};
  const int KC = g.Cp >> 6;
  const int fg = blockIdx.x / (PP * KC), rem = blockIdx.x - fg * (PP * KC);
  const int j = rem / KC, kc = rem - j * KC;
  const int l = threadIdx.x;
  const int r = l & 15, kseg = l >> 4;
  const int p = order.pt[j];
  const int k = 16 * fg + 4 * (r & 3) + (r >> 2);
  v4i val = {0, 0, 0, 0};
  if (k < g.Kp && p >= 0) val = *(const v4i*)(U + ((size_t)p * g.Kp + k) * g.Cp + 64 * kc + 16 * kseg);
  *(v4i*)(U16 + ((size_t)blockIdx.x * 64 + l) * 16) = val;
}

hipError_t launch_repack_filter16(const Geometry& g, int filters, const void* U, void* U16,
                                  hipStream_t s) {
  const dim3 grid((unsigned)((filters / 16) * ((g.P + 3) / 4 * 4) * (g.Cp / 64)));
  switch (g.alg) {
    case 2: hipLaunchKernelGGL(repack_filter16_kernel<2>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)U16, g); break;
    case 3: hipLaunchKernelGGL(repack_filter16_kernel<3>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)U16, g); break;
    case 4: hipLaunchKernelGGL(repack_filter16_kernel<4>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)U16, g); break;
    case 5: hipLaunchKernelGGL(repack_filter16_kernel<5>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)U16, g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int ALG, int KC, int OUT, int EV>
static hipError_t launch_quad16_impl(const Geometry& g, const void* V, const FilterViews& f,
                                     float x_scale, float inv_y, void* y, hipStream_t s,
                                     bool prepare) {
  constexpr int NW = kQuad16Waves;
  auto kernel = quad16_kernel<ALG, KC, OUT, EV, NW>;
  constexpr unsigned lds_bytes = quad16_lds_layout<KC, NW, OUT>(2);
  static_assert(lds_bytes <= 160u * 1024u, "V buffers and staging exceed the LDS of a compute unit");
  if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel));
  const int fgroups = quad16_filter_count(g) / 16;
  const dim3 grid((unsigned)((g.Tp / 16) * (fgroups / NW)));
  hipLaunchKernelGGL(kernel, grid, dim3(NW * 64), lds_bytes, s, (const int8_t*)V,
                     (const int8_t*)f.U_single, f.dequant_single, x_scale, inv_y, y, g, fgroups);
  return hipGetLastError();
}

template <int ALG, int KC>
static hipError_t launch_quad16_kc(int out, const Geometry& g, const void* V, const FilterViews& f,
                                   float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  // elements per store: a tile row of four outputs never crosses the end of an image row when
  // 4 divides W; else pairs (W even) or single elements
  if (g.W % 4 == 0)
    return out == 2 ? launch_quad16_impl<ALG, KC, 2, 4>(g, V, f, x_scale, inv_y, y, s, prepare)
                    : launch_quad16_impl<ALG, KC, 0, 4>(g, V, f, x_scale, inv_y, y, s, prepare);
  if (g.W % 2 == 0)
    return out == 2 ? launch_quad16_impl<ALG, KC, 2, 2>(g, V, f, x_scale, inv_y, y, s, prepare)
                    : launch_quad16_impl<ALG, KC, 0, 2>(g, V, f, x_scale, inv_y, y, s, prepare);
  return out == 2 ? launch_quad16_impl<ALG, KC, 2, 1>(g, V, f, x_scale, inv_y, y, s, prepare)
                  : launch_quad16_impl<ALG, KC, 0, 1>(g, V, f, x_scale, inv_y, y, s, prepare);
}

template <int ALG>
static hipError_t launch_quad16_alg(int out, const Geometry& g, const void* V, const FilterViews& f,
                                    float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  switch (g.Cp / 64) {
    case 1: return launch_quad16_kc<ALG, 1>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 2: return launch_quad16_kc<ALG, 2>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 4: return launch_quad16_kc<ALG, 4>(out, g, V, f, x_scale, inv_y, y, s, prepare);
  }
  return hipErrorNotSupported;
}

hipError_t launch_quad16(int out, const Geometry& g, const void* V, const FilterViews& f,
                         float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  if (!quad16_supported(g) || out == 1) return hipErrorNotSupported;
  return g.alg == 4 ? launch_quad16_alg<4>(out, g, V, f, x_scale, inv_y, y, s, prepare)
                    : launch_quad16_alg<5>(out, g, V, f, x_scale, inv_y, y, s, prepare);
}

}  // namespace sfc
