// Internal interface between the C ABI (sfc_api.hip) and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sfc {

// Everything a kernel needs to know about one convolution, by value.
struct Geometry {
  int N, Cin, Cout, H, W;
  int alg;        // sfc_alg: 0..3 SFC-6 with 6x6 / 7x7 tiles, 4..5 SFC-4, 6..7 SFC-6(6x6,5x5)
  int th, tw;     // tile grid per image: ceil(H/M), ceil(W/M), M outputs per tile edge
  int strips;     // N * th: one strip = one row of tiles of one image
  int T;          // tiles = strips * tw
  int Tp;         // T rounded up to 16 (row padding of V and M)
  int Cp;         // Cin rounded up to 64 (the K extent of one int8 MFMA)
  int Kp;         // Cout rounded up to 16
  int P;          // multiplication points per tile
  float qmax;     // largest transform-domain magnitude, 2^(bits-1) - 1 (requantized mode)
};

// Device-side views of the filter buffer (all inside the caller's filter_dev).
struct FilterViews {
  void* U;              // [P][Kp][Cp] int8 (requantized) or int16 (exact)
  float* dequant;       // requantized: [P][Kp] s_Tx[p]*s_Tf[p,k]*s_w[k]/36 (kept for inspection;
                        // the kernels read dequant_single); exact: unused
  float* inv_sw;        // [P][Kp] 1/s_Tf
  float* inv_sx;        // [P]     1/s_Tx
  float* wscale;        // [Kp]    s_w[k]
  // fused and single-kernel paths: U regrouped into MFMA operands of four points x four
  // filters
  void* U_single;
  // every requantized path: the dequantization factors as [filter][processing position],
  // positions padded to a multiple of four, rows of filters beyond Cout zero
  float* dequant_single;
  // SFC-4 forms on the fused and single paths: the table of the input transform on the
  // matrix cores (sfc_mfma_input.hpp)
  unsigned char* input_tab;
};

hipError_t launch_filter_transform(int mode, const Geometry& g, const int8_t* w,
                                   const FilterViews& f, hipStream_t s);
// input_tab: FilterViews::input_tab (read by the SFC-4 forms in requantized mode)
hipError_t launch_input_transform(int mode, const Geometry& g, const int8_t* x, void* V,
                                  const float* inv_sx, const unsigned char* input_tab,
                                  hipStream_t s);
// requantized-mode kernel; hipErrorNotSupported when the geometry is outside its limits
// Launchers with a `prepare` argument: when true nothing is launched; the call raises, on the
// current device, the dynamic-LDS limit of the kernel instantiation it would launch (the
// data pointers are not looked at) and returns what the runtime said.
hipError_t launch_input_transform_i8(const Geometry& g, const int8_t* x, void* V,
                                     const float* inv_sx, const unsigned char* input_tab,
                                     hipStream_t s, bool prepare = false);
// 3x3 filters on small feature maps (a patch within 128 bytes of a plane, at most 16 tiles per
// image; sfc_input_image.hip):
// whether the kernel applies, its table (image_table_bytes; in the filter buffer after the
// table of the SFC-4 forms, image_table_offset bytes from FilterViews::input_tab; built on the
// host for the layer's H and W), the launch
bool image_input_supported(const Geometry& g);
unsigned image_table_bytes(const Geometry& g);
unsigned image_table_offset(const Geometry& g);
// SFC-6 forms: bytes from FilterViews::input_tab to the table of the row-form input transform
// (kRowsTabBytes, after the small-image table if the geometry has one); ~0u: no such table
unsigned rows_table_offset(const Geometry& g);
void build_image_input_table(const Geometry& g, const float* inv_sx, unsigned char* tab);
hipError_t launch_input_image(const Geometry& g, const int8_t* x, void* V, const unsigned char* tab,
                              hipStream_t s, bool prepare);
hipError_t launch_product(int mode, const Geometry& g, const void* V, const void* U, int32_t* M,
                          hipStream_t s);
// requantized mode (sfc_gemm.hip): the products as P batched int8 GEMMs; the output
// transform reading their sums (out: 0 float32, 2 int8 with ReLU)
// bytes per int32 sum of M as the GEMM stores it (3: 24-bit, when no sum can exceed that; 4)
int m_sum_bytes(const Geometry& g);
hipError_t launch_product_gemm_i8(const Geometry& g, const void* V, const void* U, int32_t* M,
                                  hipStream_t s);
hipError_t launch_output_sums(int out, const Geometry& g, const int32_t* M, const FilterViews& f,
                              float x_scale, float inv_y, void* y, hipStream_t s,
                              bool prepare = false);
// out: 0 float32, 1 int32 sums (exact mode), 2 int8 with ReLU (inv_y = 1 / output scale)
hipError_t launch_output_transform(int mode, int out, const Geometry& g, const int32_t* M,
                                   const FilterViews& f, float x_scale, float inv_y, void* y,
                                   hipStream_t s);
// products + output transform in one kernel (sfc_fused_quad.hip): whether it covers this
// geometry (Cin padded to 64, 128, 256 or 512), how many filters its operand covers
bool fused_quad_supported(const Geometry& g);
int quad_filter_count(const Geometry& g);
hipError_t launch_fused_quad(int out, const Geometry& g, const void* V, const FilterViews& f,
                             float x_scale, float inv_y, void* y, hipStream_t s,
                             bool prepare = false);
// the same for the SFC-4 forms with 16 filters per wave and four pairs per lane
// (sfc_quad16.hip): U_single holds its filter operand, dequant_single its factors as
// [group of 16 filters][position][lane quarter][4]
bool quad16_supported(const Geometry& g);
int quad16_filter_count(const Geometry& g);
hipError_t launch_repack_filter16(const Geometry& g, int filters, const void* U, void* U16,
                                  hipStream_t s);
hipError_t launch_quad16(int out, const Geometry& g, const void* V, const FilterViews& f,
                         float x_scale, float inv_y, void* y, hipStream_t s, bool prepare = false);
// products + output transform with the input channels split over the waves of a workgroup
// (sfc_splitk.hip: 512 channels, 7x7 and 4x4 tiles), on the filter operand and factor table
// of launch_quad16
bool splitk_supported(const Geometry& g);
int splitk_filter_count(const Geometry& g);
hipError_t launch_splitk(int out, const Geometry& g, const void* V, const FilterViews& f,
                         float x_scale, float inv_y, void* y, hipStream_t s, bool prepare = false);
// single-kernel path of the SFC-4 forms, up to 128 input channels (sfc_single16.hip), on the
// same filter operand and factor table as launch_quad16
bool single16_supported(const Geometry& g);
hipError_t launch_single16(int out, const Geometry& g, const int8_t* x, const FilterViews& f,
                           float x_scale, float inv_y, void* y, hipStream_t s, bool prepare = false);
// the same for 129 to 512 input channels on feature maps of at most 16 tiles, the products
// accumulated in registers chunk by chunk (sfc_single16k.hip)
bool single16k_supported(const Geometry& g);
hipError_t launch_single16k(int out, const Geometry& g, const int8_t* x, const FilterViews& f,
                            float x_scale, float inv_y, void* y, hipStream_t s, bool prepare = false);
// single-kernel path: whether it covers this geometry, the bytes of its filter operand,
// the regrouping of the canonical U, the processing order (position -> canonical point)
bool single_supported(const Geometry& g);
// filters: how many the regrouped operand covers (a multiple of 4, >= Cout, zero beyond Kp)
hipError_t launch_repack_filter(const Geometry& g, int filters, const void* U, void* Uf,
                                hipStream_t s);
void single_point_order(int alg, int* pt /*[P]*/);
hipError_t launch_single_conv(int out, const Geometry& g, const int8_t* x, const FilterViews& f,
                              float x_scale, float inv_y, void* y, hipStream_t s,
                              bool prepare = false);
// Requantized mode: prepares every kernel that `path` (sfc_path) launches for this geometry
// and output type.  Once per plan, from sfc_transform_filter.
hipError_t prepare_kernels(int path, int out, const Geometry& g);
// The limit of a kernel's dynamic LDS raised to the 160 KB of a gfx950 compute unit.
inline hipError_t raise_lds_limit(const void* kernel) {
  return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}
// abs-max calibration: maxima are int32, zeroed by the launcher
hipError_t launch_act_absmax(const Geometry& g, const int8_t* x, int32_t* maxima /*[P]*/,
                             hipStream_t s);
hipError_t launch_filter_absmax(const Geometry& g, const int8_t* w,
                                int32_t* maxima /*[P][Cout]*/, hipStream_t s);

hipError_t launch_stream_copy(void* dst, const void* src, size_t bytes, hipStream_t s);

}  // namespace sfc
