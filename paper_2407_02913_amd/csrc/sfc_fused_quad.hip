// Launch side of the fused product + output-transform kernel (sfc_fused_quad.hpp): limits,
// filter-operand size and the dispatch over algorithm, channel chunks and output type.  The
// 5x5- and 7x7-filter algorithms are instantiated in sfc_fused_quad_5tap.hip and
// sfc_fused_quad_7tap.hip.
#include "sfc_fused_quad.hpp"

namespace sfc {

hipError_t launch_fused_quad_5tap(int out, const Geometry& g, const void* V, const FilterViews& f,
                                  float x_scale, float inv_y, void* y, hipStream_t s, bool prepare);
hipError_t launch_fused_quad_7tap(int out, const Geometry& g, const void* V, const FilterViews& f,
                                  float x_scale, float inv_y, void* y, hipStream_t s, bool prepare);

bool fused_quad_supported(const Geometry& g) {
  const int kc = g.Cp / 64;
  if (kc != 1 && kc != 2 && kc != 4 && kc != 8) return false;
  const int nw = quad_waves(g.alg, kc);
  const long long kq = (long long)((g.Cout + 4 * nw - 1) / (4 * nw)) * nw;  // filter quads allocated
  const long long ybytes = 4ll * g.N * g.Cout * g.H * g.W;
  const long long vbytes = (long long)g.P * g.Tp * g.Cp, ubytes = kq * 4 * (g.P + 3) * g.Cp;
  const long long lim = 1ll << 31;
  return ybytes < lim && vbytes < lim && ubytes < lim && quad_lds_bytes(g.alg, kc) <= 160u * 1024u;
}

// filters covered by the quad-layout filter operand: Cout rounded up to whole workgroups
int quad_filter_count(const Geometry& g) { return quad_filter_count_for(g); }

hipError_t launch_fused_quad(int out, const Geometry& g, const void* V, const FilterViews& f,
                             float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  if (!fused_quad_supported(g) || out == 1) return hipErrorNotSupported;
  switch (g.alg) {
    case 0: return launch_quad_alg<0>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 1: return launch_quad_alg<1>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 2: return launch_quad_alg<2>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 3: return launch_quad_alg<3>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 4: return launch_quad_alg<4>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 5: return launch_quad_alg<5>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 6:
    case 7: return launch_fused_quad_5tap(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 8:
    case 9: return launch_fused_quad_7tap(out, g, V, f, x_scale, inv_y, y, s, prepare);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
