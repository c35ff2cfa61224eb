// The whole hot path in one kernel, for layers with Cin <= 64 and the SFC-6 forms with 3x3
// filters (gfx950): input-tile transform, transform-domain products and output transform
// without V or M ever leaving the compute unit.  (The SFC-4 forms have their own kernel,
// sfc_single16.hip.)
//
// A workgroup of 16 waves (8 for the 7x7 forms, each wave then doing two passes) owns a
// rectangle of up to 16 tiles (S strips x tlw tile columns; a strip = one row of tiles of one
// image), all input channels and a group of 64 filters.
//
// Points are taken in groups of four (one filter-operand load per group).
//
//  1. Stage: the M+2 input rows of every (strip, channel) go to LDS with dword
//     loads, lanes running along the row, padding halo zero-filled.
//  2. Input transform: wave = tile, lane = input channel.  Each thread reads its
//     patch, applies the symbolic DFT-6 add network along rows and columns, forms
//     the multiplication points, rounds them to int8 and writes V[j][tile][c]
//     (j: processing order, 1 KiB per point = one MFMA operand) over the staging
//     area.
//  3. Products + output transform: wave w owns filters 4w..4w+3, lane l the pair
//     (tile l%16, filter 4w + l/16).  For a group of four points one 16-byte load
//     per lane fetches the filter operand: row i of the 16x64 operand holds point
//     i%4 of the group for filter i/4.  The int8 MFMA 16x16x64 of that operand
//     with V of point r leaves, in accumulator element r of every lane, exactly
//     the product of the lane's own pair; the other three elements mix points and
//     are ignored.  So the products arrive lane-local, one pair per lane, and feed
//     the streaming output transform without any exchange or barrier.  The matrix
//     pipe does 4x the necessary work; it is idle otherwise (the layer is bound by
//     HBM bytes and vector adds, the products are under a tenth of either).
//  4. Store: one output row at a time goes through a small LDS block private to
//     the wave, so that consecutive lanes store consecutive outputs of an image
//     row (dequantized float32, or the next layer's int8 activations) to NCHW.
//
// Measured on one compute unit the kernel is bound by vector-ALU instruction issue
// (about 1400 vector instructions per thread at 4 waves per SIMD), not by HBM or LDS.
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"
#include "sfc_store.hpp"
#include "sfc_tile_input.hpp"

namespace sfc {

struct SinglePlan {
  TileRect tr;
  int kgroups;         // groups of 64 filters
  unsigned stage_off;  // LDS byte offset of the per-wave output staging blocks
  unsigned lds_bytes;
};

constexpr int kWaves6 = 16;  // waves per workgroup for the 6x6 forms

template <int ALG, int OUT, bool VEC2, int NW>
__global__ __launch_bounds__(NW * 64, NW / 4) void single_conv_kernel(
    const int8_t* __restrict__ x, const int8_t* __restrict__ Uf, const float* __restrict__ dqf,
    const float* __restrict__ inv_sx, float x_scale, float inv_y, void* __restrict__ y, Geometry g,
    SinglePlan sp) {
  using Tr = AlgTraits<ALG>;
  constexpr int P = Tr::P, M = Tr::M, NC = Tr::NC;
  constexpr int PP = Order<ALG>::PP, PG = PP / 4;  // points padded to whole groups of four
  constexpr int SPW = 16 / NW;  // passes per wave over tiles / filter quads
  static_assert(NW == 8 || NW == 16, "8 or 16 waves");
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const TileRect& tr = sp.tr;
  const int bx = xcd_contiguous(blockIdx.x, gridDim.x);
  const int W = g.W, H = g.H;

  // per-tile store data for step 4, written by 16 lanes now and read after the barriers
  constexpr int STAGE_FLOATS = 64 * M;  // per wave
  int* tile_tab = (int*)(lds + sp.stage_off + NW * STAGE_FLOATS * 4);
  if (threadIdx.x < 16) {
    const int tl = threadIdx.x;
    const TileCoord tc = tile_coord(g, tr, bx, tl);
    write_tile_entry<M>(tile_tab, tl, tc.live, tc.n, tc.ti, tc.tj, g.Cout, H, W);
  }

  // ---- 1. stage, 2. input transform -----------------------------------------------
  stage_input<ALG, NW>(x, lds, g, tr, bx, 0, wave, lane);
  __syncthreads();
  transform_tiles<ALG, NW>(lds, inv_sx, g.qmax, g, tr, bx, wave, lane);
  __syncthreads();

  // ---- 3. products + output transform: lane = (tile l%16, filter 4*kq + l/16) ------
  const int kfilters = sp.kgroups * 64;
  const __amdgpu_buffer_rsrc_t ures = __builtin_amdgcn_make_buffer_rsrc(
      (void*)Uf, 0, (int)((unsigned)kfilters * (unsigned)(PP * 64)), kBufferFlags);
  const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)dqf, 0, (int)((unsigned)kfilters * (unsigned)(PP * 4)), kBufferFlags);
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      y, 0, (int)(esz * (unsigned)(g.N * g.Cout) * (unsigned)(H * W)), kBufferFlags);
  const unsigned char* vlane = lds + (lane & 15) * 64 + (lane >> 4) * 16;  // tile l%16, channels 16*(l/16)..
  // this wave's private staging block: one output row as [filter 0..3][tile 0..15][o2], or all
  // M rows in the order of y
  float* stage = (float*)(lds + sp.stage_off) + wave * STAGE_FLOATS;

#pragma unroll 1
  for (int qi = 0; qi < SPW; ++qi) {
    const int kq = blockIdx.y * 16 + wave + NW * qi;  // filter quad of this pass
    const int kcol = kq * 4 + (lane >> 4);            // this lane's filter
    const unsigned a_lane = (unsigned)lane * 16u;
    const unsigned a_wave = (unsigned)kq * (unsigned)(PG * 1024);
    const unsigned d_lane = (unsigned)kcol * (unsigned)(PP * 4);
    // Software pipeline over the points: call j of next() issues the LDS read of
    // point j+2's V operand and the MFMA of point j+1, then converts the accumulator
    // of point j.  The filter operand and the dequantization factors of group g
    // (four points) sit in ring slot g%2 and are refilled, two groups ahead, once
    // the group's last product has been taken.
    v4i aring[2];
    v4f dring[2];
    auto load_group = [&](int pg) {
      aring[pg & 1] =
          __builtin_amdgcn_raw_buffer_load_b128(ures, a_lane, a_wave + (unsigned)pg * 1024u, 0);
      dring[pg & 1] = __builtin_bit_cast(
          v4f, __builtin_amdgcn_raw_buffer_load_b128(dres, d_lane, (unsigned)pg * 16u, 0));
    };
    load_group(0);
    load_group(1);
    v4i b_nxt = *(const v4i*)(vlane + 1024);  // V operand of point 1
    v4i acc_cur;                              // accumulator of the point about to be taken
    {
      const v4i b0 = *(const v4i*)vlane;
      acc_cur = __builtin_amdgcn_mfma_i32_16x16x64_i8(aring[0], b0, v4i{0, 0, 0, 0}, 0, 0, 0);
    }
    int j = 0;  // folds to a constant after unrolling
    auto next = [&]() -> float {
      const int r = j & 3, pg = j >> 2;
      v4i b_new = b_nxt, acc_new = acc_cur;
      if (j + 2 < P) b_new = *(const v4i*)(vlane + (j + 2) * 1024);
      if (j + 1 < P)
        acc_new = __builtin_amdgcn_mfma_i32_16x16x64_i8(aring[((j + 1) >> 2) & 1], b_nxt,
                                                        v4i{0, 0, 0, 0}, 0, 0, 0);
      float v = (float)acc_cur[r] * dring[pg & 1][r];
      // The scaled product is materialized here and nothing moves across this point:
      // otherwise the compiler hoists operand reads and keeps whole accumulators alive
      // until their first use, which costs more registers than the kernel has.
      asm volatile("" : "+v"(v));
      if (r == 3 && pg + 2 < PG) load_group(pg + 2);
      b_nxt = b_new;
      acc_cur = acc_new;
      __builtin_amdgcn_sched_barrier(0);
      ++j;
      return v;
    };
    float z[NC][M];
    stream_vertical<ALG, float>(next, z);

    // ---- 4. store ----------------------------------------------------------------
    store_pairs<ALG, OUT, VEC2>(z, stage, tile_tab, lane, kq, x_scale, inv_y, yres, g.Cout, H, W);
  }
}

// Filter operand of the fused kernels from the canonical U[p][k][c]: block (filter
// quad kq, point group pg, channel chunk kc) is one KiB; lane l holds 16 channels
// 64*kc + 16*(l/16).. of point pt[4*pg + (l%16)%4], filter 4*kq + (l%16)/4.
// Filters beyond Kp are zero.
template <int ALG>
__global__ __launch_bounds__(64) void repack_filter_kernel(const int8_t* __restrict__ U,
                                                           int8_t* __restrict__ Uf, Geometry g) {
  constexpr int PG = Order<ALG>::PP / 4;
  constexpr Order<ALG> order{};
  const int KC = g.Cp >> 6;
  const int kq = blockIdx.x / (PG * KC), rem = blockIdx.x - kq * (PG * KC);
  const int pg = rem / KC, kc = rem - pg * KC;
  const int l = threadIdx.x;
  const int i = l & 15, kseg = l >> 4;
  const int p = order.pt[4 * pg + (i & 3)];
  const int k = 4 * kq + (i >> 2);
  v4i val = {0, 0, 0, 0};  // also for the positions of the last group that hold no point
  if (k < g.Kp && p >= 0) val = *(const v4i*)(U + ((size_t)p * g.Kp + k) * g.Cp + 64 * kc + 16 * kseg);
  *(v4i*)(Uf + ((size_t)blockIdx.x * 64 + l) * 16) = val;
}

// waves per workgroup: the 7x7 forms carry 10x7 partial outputs per pair and need the
// 256-register budget of 8 waves
static int single_waves(int alg) { return alg_tile(alg) == 6 ? kWaves6 : 8; }

static bool make_single_plan(const Geometry& g, SinglePlan* sp) {
  if (g.Cp != 64 || g.alg > 3) return false;  // the SFC-6 forms with 3x3 filters
  const int M = alg_tile(g.alg);
  // LDS: the staged rows of the rectangle (later overwritten by V), the per-wave output
  // staging blocks, the per-tile store table
  const unsigned vbytes = (unsigned)g.P * 1024u;
  const unsigned sbytes = (unsigned)single_waves(g.alg) * 64u * (unsigned)M * 4u + 256u;
  const unsigned lds_max = 160u * 1024u;
  if (vbytes + 16u + sbytes > lds_max) return false;
  if (!make_tile_rect(g, lds_max - 16u - sbytes, &sp->tr)) return false;
  sp->kgroups = (g.Cout + 63) / 64;
  const unsigned xbytes = tile_rect_stage_bytes(g, sp->tr);
  sp->stage_off = ((xbytes > vbytes ? xbytes : vbytes) + 15u) & ~15u;
  sp->lds_bytes = sp->stage_off + sbytes;
  const long long xb = (long long)g.N * g.Cin * g.H * g.W;
  const long long yb = 4ll * g.N * g.Cout * g.H * g.W;
  const long long ub = (long long)sp->kgroups * 64 * (g.P + 3) * 64;
  const long long lim = 1ll << 31;
  return sp->lds_bytes <= lds_max && xb < lim && yb < lim && ub < lim;
}

bool single_supported(const Geometry& g) {
  SinglePlan sp;
  return single16_supported(g) || single16k_supported(g) || make_single_plan(g, &sp);
}

hipError_t launch_repack_filter(const Geometry& g, int filters, const void* U, void* Uf,
                                hipStream_t s) {
  const dim3 grid((unsigned)((filters / 4) * ((g.P + 3) / 4) * (g.Cp / 64)));
  switch (g.alg) {
    case 0: hipLaunchKernelGGL(repack_filter_kernel<0>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 1: hipLaunchKernelGGL(repack_filter_kernel<1>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 2: hipLaunchKernelGGL(repack_filter_kernel<2>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 3: hipLaunchKernelGGL(repack_filter_kernel<3>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 4: hipLaunchKernelGGL(repack_filter_kernel<4>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 5: hipLaunchKernelGGL(repack_filter_kernel<5>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 6: hipLaunchKernelGGL(repack_filter_kernel<6>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 7: hipLaunchKernelGGL(repack_filter_kernel<7>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 8: hipLaunchKernelGGL(repack_filter_kernel<8>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 9: hipLaunchKernelGGL(repack_filter_kernel<9>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// processing position -> canonical point index (-1: no point), for the host-built tables
void single_point_order(int alg, int* pt /*[P rounded up to a multiple of 4]*/) {
  auto copy = [&](const auto& o) {
    for (int j = 0; j < (int)(sizeof(o.pt) / sizeof(o.pt[0])); ++j) pt[j] = o.pt[j];
  };
  switch (alg) {
    case 0: { constexpr Order<0> o{}; copy(o); break; }
    case 1: { constexpr Order<1> o{}; copy(o); break; }
    case 2: { constexpr Order<2> o{}; copy(o); break; }
    case 3: { constexpr Order<3> o{}; copy(o); break; }
    case 4: { constexpr Order<4> o{}; copy(o); break; }
    case 5: { constexpr Order<5> o{}; copy(o); break; }
    case 6: { constexpr Order<6> o{}; copy(o); break; }
    case 7: { constexpr Order<7> o{}; copy(o); break; }
    case 8: { constexpr Order<8> o{}; copy(o); break; }
    case 9: { constexpr Order<9> o{}; copy(o); break; }
    default: break;
  }
}

template <int ALG, int OUT, bool VEC2, int NW>
static hipError_t launch_single_impl(const Geometry& g, const SinglePlan& sp, const int8_t* x,
                                     const FilterViews& f, float x_scale, float inv_y, void* y,
                                     hipStream_t s, bool prepare) {
  auto kernel = single_conv_kernel<ALG, OUT, VEC2, NW>;
  if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel));
  const dim3 grid(tile_rect_groups(g, sp.tr), (unsigned)sp.kgroups);
  hipLaunchKernelGGL(kernel, grid, dim3(NW * 64), sp.lds_bytes, s, x, (const int8_t*)f.U_single,
                     f.dequant_single, f.inv_sx, x_scale, inv_y, y, g, sp);
  return hipGetLastError();
}

template <int ALG, int OUT>
static hipError_t launch_single_out(const Geometry& g, const SinglePlan& sp, const int8_t* x,
                                    const FilterViews& f, float x_scale, float inv_y, void* y,
                                    hipStream_t s, bool prepare) {
  constexpr int NW = AlgTraits<ALG>::M == 6 ? kWaves6 : 8;
  constexpr bool kPairs = AlgTraits<ALG>::M % 2 == 0;  // pairs of an output row stay aligned
  if constexpr (kPairs) {
    if (g.W % 2 == 0) return launch_single_impl<ALG, OUT, true, NW>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
  }
  return launch_single_impl<ALG, OUT, false, NW>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
}

template <int ALG>
static hipError_t launch_single_alg(int out, const Geometry& g, const SinglePlan& sp,
                                    const int8_t* x, const FilterViews& f, float x_scale,
                                    float inv_y, void* y, hipStream_t s, bool prepare) {
  return out == 2 ? launch_single_out<ALG, 2>(g, sp, x, f, x_scale, inv_y, y, s, prepare)
                  : launch_single_out<ALG, 0>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
}

hipError_t launch_single_conv(int out, const Geometry& g, const int8_t* x, const FilterViews& f,
                              float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  SinglePlan sp;
  if (!make_single_plan(g, &sp) || out == 1) return hipErrorNotSupported;
  switch (g.alg) {
    case 0: return launch_single_alg<0>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare);
    case 1: return launch_single_alg<1>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare);
    case 2: return launch_single_alg<2>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare);
    case 3: return launch_single_alg<3>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
