// The fused product + output-transform kernel for SFC-6(6x6,5x5) (184 / 196 points): its
// own translation unit so that the instantiations compile beside those of the 3x3 forms.
#include "sfc_fused_quad.hpp"

namespace sfc {

hipError_t launch_fused_quad_5tap(int out, const Geometry& g, const void* V, const FilterViews& f,
                                  float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  switch (g.alg) {
    case 6: return launch_quad_alg<6>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 7: return launch_quad_alg<7>(out, g, V, f, x_scale, inv_y, y, s, prepare);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
