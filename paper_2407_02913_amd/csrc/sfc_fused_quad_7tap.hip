// The fused product + output-transform kernel for SFC-6(4x4,7x7) (184 / 196 points): its
// own translation unit so that the instantiations compile beside those of the other forms.
#include "sfc_fused_quad.hpp"

namespace sfc {

hipError_t launch_fused_quad_7tap(int out, const Geometry& g, const void* V, const FilterViews& f,
                                  float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  switch (g.alg) {
    case 8: return launch_quad_alg<8>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 9: return launch_quad_alg<9>(out, g, V, f, x_scale, inv_y, y, s, prepare);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
