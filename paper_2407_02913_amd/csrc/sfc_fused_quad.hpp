// Transform-domain products + output transform in one kernel for any number of input
// channels (gfx950): V comes from the input-transform kernel, M never leaves the chip.
//
// A workgroup owns 16 consecutive tiles and 4*NW filters (wave w: filters 4w..4w+3,
// lane l: the pair (tile l%16, filter 4w + l/16)).  Points are taken in groups of four
// in the processing order of Order<ALG> (the SFC-4 forms pad their 46 / 49 points to
// 48 / 52 positions whose filter operand is zero and whose products are never taken).  For a group, the V rows of the 16 tiles
// (4 points x 16 tiles x Cin bytes) are copied by the whole workgroup from HBM into
// one of two LDS buffers, already laid out as MFMA operands, while the previous
// group is being multiplied; one barrier per group.  The filter operand of a group
// holds, in row i of each 16x64 block, point i%4 of the group for filter i/4, so the
// int8 MFMA 16x16x64 with V of point r leaves the product of the lane's own pair in
// accumulator element r (the other three elements mix points and are ignored): the
// products arrive lane-local, one pair per lane, and feed the streaming output
// transform directly.  The matrix pipe does four times the necessary work in exchange
// for no exchange of M between lanes.
#pragma once
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"
#include "sfc_store.hpp"

namespace sfc {

// PLANES: whole tiles cover the feature map and the 16 tiles of a wave are whole images
// (whole_image_tiles); y is then written image by image (store_planes) from staging blocks
// of M*M floats per pair, which take the place of the V buffers once the last group of
// points has been multiplied.
template <int ALG, int KC, int NW, bool PLANES>
constexpr unsigned quad_lds_layout(int what) {
  constexpr unsigned M = AlgTraits<ALG>::M;
  constexpr unsigned vbytes = 2u * 4u * 16u * 64u * KC;
  constexpr unsigned stage = NW * 64u * M * (PLANES ? M : 1u) * 4u;
  constexpr unsigned stage_off = PLANES ? 0u : vbytes;
  constexpr unsigned tab_off = PLANES ? (vbytes > stage ? vbytes : stage) : vbytes + stage;
  return what == 0 ? stage_off : what == 1 ? tab_off : tab_off + 256u;
}

template <int ALG, int KC, int OUT, bool VEC2, int NW, int WGS, bool PLANES = false>
__global__ __launch_bounds__(NW * 64, WGS) void fused_quad_kernel(
    const int8_t* __restrict__ V, const int8_t* __restrict__ Uf, const float* __restrict__ dqf,
    float x_scale, float inv_y, void* __restrict__ y, Geometry g, int kquads) {
  using Tr = AlgTraits<ALG>;
  constexpr int P = Tr::P, M = Tr::M, NC = Tr::NC;
  constexpr int PP = Order<ALG>::PP, PG = PP / 4;  // points padded to whole groups of four
  constexpr int CP = KC * 64;                 // padded input channels
  constexpr int GROUP_BYTES = 4 * 16 * CP;    // V of one group: 4 points x 16 tiles
  constexpr int CHUNKS = GROUP_BYTES / 16;    // 16-byte pieces of a group
  constexpr int NT = NW * 64;
  constexpr int NL = (CHUNKS + NT - 1) / NT;  // pieces per thread and group
  // filter operand blocks in flight (four with eight chunks, where the 8-wave forms have the
  // registers: 512 channels on 7x7 maps, 7x7 tiles, batch 256: 74.7 against 76.9 us; the 5x5-
  // and 7x7-filter forms, with 12 classes of partial outputs, do not)
  constexpr int RA = KC < 2 ? 1 : (KC >= 8 && NW <= 8 && AlgTraits<ALG>::NC <= 10) ? 4 : 2;
  constexpr Order<ALG> order{};
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* vbuf = lds;  // [2][GROUP_BYTES], block (r*KC + kc) = 16 tiles x 64 bytes

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* stage = (float*)(lds + quad_lds_layout<ALG, KC, NW, PLANES>(0)) +
                 wave * (64 * M * (PLANES ? M : 1));
  int* tile_tab = (int*)(lds + quad_lds_layout<ALG, KC, NW, PLANES>(1));

  // Workgroup -> (filter group, tile block).  Ids that share an XCD (an L2) cover a
  // contiguous range of positions; positions run over chunks of four filter groups
  // (slowest), tile blocks, and the filter groups of the chunk (fastest).  The workgroups
  // an XCD runs at a time are then a few tile blocks times four filter groups: every V
  // block they stream is used by four of them and every filter operand by all that share
  // its group, so the L2 fetches about as many bytes of V as of U.  (With the filter group
  // slowest an XCD ran one group over all tile blocks and fetched the whole of V: 148 MB
  // per launch instead of 26 MB of operands on 14x14 maps with 256 channels.)
  const int tblocks = g.Tp >> 4;
  const int pos = xcd_contiguous(blockIdx.x, gridDim.x);
  constexpr int KBG = 4;
  const int kgroups = kquads / NW;
  const int chunk = pos / (KBG * tblocks), rem = pos - chunk * (KBG * tblocks);
  const int in_chunk = min(KBG, kgroups - chunk * KBG);  // the last chunk may be smaller
  const int tb = rem / in_chunk, kb = chunk * KBG + (rem - tb * in_chunk);
  const int t0 = tb * 16;
  const int kq = kb * NW + wave;          // filter quad of this wave
  const int kcol = kq * 4 + (lane >> 4);  // this lane's filter

  if (threadIdx.x < 16) {
    const int tl = threadIdx.x, t = t0 + tl;
    const int per = g.th * g.tw;
    const int n = t / per, rem = t - n * per;
    const int ti = rem / g.tw, tj = rem - ti * g.tw;
    write_tile_entry<M>(tile_tab, tl, t < g.T, n, ti, tj, g.Cout, g.H, g.W);
  }

  const unsigned vplane = (unsigned)g.Tp * (unsigned)CP;
  const __amdgpu_buffer_rsrc_t vres =
      __builtin_amdgcn_make_buffer_rsrc((void*)V, 0, (int)(vplane * (unsigned)P), kBufferFlags);
  const __amdgpu_buffer_rsrc_t ures = __builtin_amdgcn_make_buffer_rsrc(
      (void*)Uf, 0, (int)((unsigned)kquads * (unsigned)(PP * CP * 4)), kBufferFlags);
  const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)dqf, 0, (int)((unsigned)kquads * (unsigned)(PP * 16)), kBufferFlags);
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      y, 0, (int)(esz * (unsigned)(g.N * g.Cout) * (unsigned)(g.H * g.W)), kBufferFlags);

  // ---- loader: piece q = tid + NT*i of a group is 16 bytes of (point r, tile, channels)
  // with r = q / (64*KC) uniform per wave; it lands in block r*KC + kc at
  // [tile][16*kseg..], the register image of the MFMA operand.
  unsigned gsrc[NL], ldst[NL];
  int rsel[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int q = (int)threadIdx.x + NT * i;
    const int r = (wave + NW * i) / KC;  // point of the group, uniform
    const int rem = q - r * (64 * KC);
    const int tile = rem / (4 * KC), ch = rem - tile * (4 * KC);
    rsel[i] = q < CHUNKS ? r : -1;
    gsrc[i] = (unsigned)(t0 + tile) * (unsigned)CP + (unsigned)ch * 16u;
    ldst[i] = (unsigned)(((r * KC + (ch >> 2)) * 16 + tile) * 64 + (ch & 3) * 16);
  }
  v4i lreg[NL];
  auto load_regs = [&](int pg) {
    // positions without a point (the tail of the last group of an SFC-4 form) re-read point
    // 0; their filter operand is zero and their products are never taken
    const int p0 = max(order.pt[4 * pg], 0), p1 = max(order.pt[4 * pg + 1], 0),
              p2 = max(order.pt[4 * pg + 2], 0), p3 = max(order.pt[4 * pg + 3], 0);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int r = rsel[i];
      const int p = r == 0 ? p0 : r == 1 ? p1 : r == 2 ? p2 : p3;
      if (r >= 0)
        lreg[i] = __builtin_amdgcn_raw_buffer_load_b128(vres, gsrc[i], (unsigned)p * vplane, 0);
    }
  };
  auto store_lds = [&](int pg) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
      if (rsel[i] >= 0) *(v4i*)(vbuf + (pg & 1) * GROUP_BYTES + ldst[i]) = lreg[i];
  };

  // ---- filter operand and dequantization factors -----------------------------------
  const unsigned a_lane = (unsigned)lane * 16u;
  const unsigned a_wave = (unsigned)kq * (unsigned)(PG * KC * 1024);
  const unsigned d_lane = (unsigned)kcol * (unsigned)(PP * 4);
  v4i aring[RA];
  auto load_a = [&](int s) {  // step s = pg*KC + kc
    aring[s % RA] = __builtin_amdgcn_raw_buffer_load_b128(ures, a_lane, a_wave + (unsigned)s * 1024u, 0);
  };
  v4f dnext;
  auto load_d = [&](int pg) {
    dnext = __builtin_bit_cast(
        v4f, __builtin_amdgcn_raw_buffer_load_b128(dres, d_lane, (unsigned)pg * 16u, 0));
  };

  load_regs(0);
#pragma unroll
  for (int s = 0; s < RA && s < PG * KC; ++s) load_a(s);
  load_d(0);
  store_lds(0);
  if (PG > 1) load_regs(1);
  __syncthreads();

  const unsigned char* blane = vbuf + (lane & 15) * 64 + (lane >> 4) * 16;
  int j = 0;  // folds to a constant after unrolling
  float cur[4];
  auto next = [&]() -> float {
    const int r = j & 3, pg = j >> 2;
    if (r == 0) {
      v4i acc[4] = {v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}};
      const unsigned char* bsrc = blane + (pg & 1) * GROUP_BYTES;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const int s = pg * KC + kc;
        const v4i a = aring[s % RA];
        if (s + RA < PG * KC) load_a(s + RA);
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          const v4i b = *(const v4i*)(bsrc + (rr * KC + kc) * 1024);
          acc[rr] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, acc[rr], 0, 0, 0);
        }
      }
      const v4f d = dnext;
      if (pg + 1 < PG) {
        load_d(pg + 1);
        store_lds(pg + 1);
      }
      if (pg + 2 < PG) load_regs(pg + 2);
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        float v = (float)acc[rr][rr] * d[rr];
        // the scaled products are materialized here, not the whole accumulators kept alive
        asm volatile("" : "+v"(v));
        cur[rr] = v;
      }
      __syncthreads();  // next group's V is in place, this group's buffer is free
      __builtin_amdgcn_sched_barrier(0);
    }
    ++j;
    return cur[r];
  };
  float z[NC][M];
  stream_vertical<ALG, float>(next, z);

  // (every wave has passed the barrier that ends the last group: the V buffers are free)
  if constexpr (PLANES)
    store_planes<ALG, OUT>(z, stage, tile_tab, lane, kq, x_scale, inv_y, yres, g.Cout, g.th, g.tw);
  else
    store_pairs<ALG, OUT, VEC2>(z, stage, tile_tab, lane, kq, x_scale, inv_y, yres, g.Cout, g.H, g.W);
}

// ---------------------------------------------------------------------------------

constexpr int kQuadWaves6 = 8;  // waves per workgroup for the 6x6 forms
inline int quad_waves(int alg, int kc) {
  // the 7x7 forms carry 10x7 partial outputs per pair, the 5x5-filter forms 12x6: they need
  // the 256-register budget
  (void)kc;
  return alg < 2 ? kQuadWaves6 : 8;
}

inline unsigned quad_lds_bytes(int alg, int kc) {
  const int nw = quad_waves(alg, kc), M = alg_tile(alg);
  return 2u * 4u * 16u * 64u * (unsigned)kc + (unsigned)nw * 64u * (unsigned)M * 4u + 256u;
}

// filters covered by the quad-layout filter operand: Cout rounded up to whole workgroups
inline int quad_filter_count_for(const Geometry& g) {
  const int per_wg = 4 * quad_waves(g.alg, g.Cp / 64);
  return (g.Cout + per_wg - 1) / per_wg * per_wg;
}

template <int ALG, int KC, int OUT, bool VEC2, bool PLANES = false>
inline hipError_t launch_quad_impl(const Geometry& g, const void* V, const FilterViews& f,
                                   float x_scale, float inv_y, void* y, hipStream_t s,
                                   bool prepare) {
  // The SFC-4 forms need under 100 registers: 8-wave workgroups, two of which share a compute
  // unit and run out of phase (measured 31.0 against 32.5 us per step on 128 channels at
  // 28x28).  The other forms: 8 waves with the 256-register budget (the 6x6 forms spilled with
  // 16 waves of 128 registers).
  constexpr int NW = ALG < 2 ? kQuadWaves6 : 8;
  constexpr int WGS = AlgTraits<ALG>::NC == 6 ? 2 : 1;
  auto kernel = fused_quad_kernel<ALG, KC, OUT, VEC2, NW, WGS, PLANES>;
  constexpr unsigned lds_bytes = quad_lds_layout<ALG, KC, NW, PLANES>(2);
  static_assert(lds_bytes <= 160u * 1024u, "V buffers and staging exceed the LDS of a compute unit");
  if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel));
  const int kfilters = quad_filter_count_for(g);
  const int kgroups = kfilters / (4 * NW);
  const dim3 grid((unsigned)((g.Tp / 16) * kgroups));
  hipLaunchKernelGGL(kernel, grid, dim3(NW * 64), lds_bytes, s, (const int8_t*)V,
                     (const int8_t*)f.U_single, f.dequant_single, x_scale, inv_y, y, g,
                     kfilters / 4);
  return hipGetLastError();
}

template <int ALG, int KC>
inline hipError_t launch_quad_kc(int out, const Geometry& g, const void* V, const FilterViews& f,
                                 float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  constexpr bool kPairs = AlgTraits<ALG>::M % 2 == 0;
  // 7x7 tiles on 7x7, 14x14, 28x28 ... maps, 4x4 tiles on 4x4, 8x8, 16x16 ...: a wave's
  // pairs are whole planes of y
  if constexpr (AlgTraits<ALG>::M == 7 || AlgTraits<ALG>::M == 4) {
    if (whole_image_tiles(AlgTraits<ALG>::M, g.H, g.W, g.th, g.tw, g.Cout))
      return out == 2 ? launch_quad_impl<ALG, KC, 2, false, true>(g, V, f, x_scale, inv_y, y, s, prepare)
                      : launch_quad_impl<ALG, KC, 0, false, true>(g, V, f, x_scale, inv_y, y, s, prepare);
  }
  if constexpr (kPairs) {
    if (g.W % 2 == 0)
      return out == 2 ? launch_quad_impl<ALG, KC, 2, true>(g, V, f, x_scale, inv_y, y, s, prepare)
                      : launch_quad_impl<ALG, KC, 0, true>(g, V, f, x_scale, inv_y, y, s, prepare);
  }
  return out == 2 ? launch_quad_impl<ALG, KC, 2, false>(g, V, f, x_scale, inv_y, y, s, prepare)
                  : launch_quad_impl<ALG, KC, 0, false>(g, V, f, x_scale, inv_y, y, s, prepare);
}

template <int ALG>
inline hipError_t launch_quad_alg(int out, const Geometry& g, const void* V, const FilterViews& f,
                                  float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  switch (g.Cp / 64) {
    case 1: return launch_quad_kc<ALG, 1>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 2: return launch_quad_kc<ALG, 2>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 4: return launch_quad_kc<ALG, 4>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 8: return launch_quad_kc<ALG, 8>(out, g, V, f, x_scale, inv_y, y, s, prepare);
  }
  return hipErrorNotSupported;
}

}  // namespace sfc
