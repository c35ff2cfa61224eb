// Transform-domain products + output transform in one kernel for layers with 512 input
// channels (gfx950), the input channels split over the waves of a workgroup.
//
// A workgroup of eight waves owns 16 consecutive tiles and 32 filters.  Wave (fg, ks), fg = 0, 1
// a group of 16 filters, ks = 0..3 a quarter of the input channels, multiplies for every point
// V of its channel quarter (16 tiles, from LDS) with the filter operand of its 16 filters (from
// global memory, a ring of loads ahead): int8 MFMA 16x16x64 with one point for 16 filters in the
// A operand, so that every accumulator element is a wanted partial sum (lane l: tile l%16,
// filters 16 fg + 4 i + l/16, i = 0..3) -- no surplus matrix work, and a wave reads only its
// quarter of V.  The four waves of a filter group then exchange their partial sums through
// LDS: wave ks collects element i = ks of all four, i.e. the sums over all channels of the pairs
// (tile l%16, filter 16 fg + 4 ks + l/16), one pair per lane, and feeds them to the streaming
// output transform.  Every wave ends with the pairs of one filter quad, the arrangement of the
// one-pair-per-lane kernel (sfc_fused_quad.hpp), whose stores it shares.
//
// Per group of four points: the workgroup copies V of the next group from memory into one of
// two LDS buffers, every wave writes its partial sums of the next group into one of two
// exchange buffers and takes the sums of the current group from the other; one barrier.
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"
#include "sfc_quad16.hpp"
#include "sfc_store.hpp"

namespace sfc {

constexpr int kSplitWaves = 8;    // waves per workgroup: 2 filter groups x 4 channel quarters
constexpr int kSplitFilters = 32; // filters per workgroup

template <int ALG, int KC, bool PLANES>
constexpr unsigned splitk_lds_layout(int what) {
  constexpr unsigned M = AlgTraits<ALG>::M;
  constexpr unsigned vbytes = 2u * 4u * 16u * 64u * KC;       // two groups of V
  constexpr unsigned xbytes = 2u * 4u * kSplitWaves * 1024u;  // two groups of partial sums
  constexpr unsigned stage = kSplitWaves * 64u * M * (PLANES ? M : 1u) * 4u;
  // the store staging takes the place of the buffers once the last sums have been taken
  constexpr unsigned body = vbytes + xbytes > stage ? vbytes + xbytes : stage;
  return what == 0 ? vbytes : what == 1 ? body : body + 256u;
}

template <int ALG, int KC, int OUT, bool VEC2, bool PLANES>
__global__ __launch_bounds__(kSplitWaves * 64, 1) void splitk_kernel(
    const int8_t* __restrict__ V, const int8_t* __restrict__ U16, const float* __restrict__ dq16,
    float x_scale, float inv_y, void* __restrict__ y, Geometry g, int fgroups) {
  using Tr = AlgTraits<ALG>;
  constexpr int P = Tr::P, M = Tr::M, NC = Tr::NC;
  constexpr int PP = Order<ALG>::PP, PG = PP / 4;
  constexpr int NW = kSplitWaves, KS = 4, CPW = KC / KS;  // chunks per wave
  static_assert(KC % KS == 0, "whole chunks per wave");
  constexpr int CP = KC * 64;
  constexpr int GROUP_BYTES = 4 * 16 * CP;   // V of one group: 4 points x 16 tiles
  constexpr int CHUNKS = GROUP_BYTES / 16;   // 16-byte pieces of a group
  constexpr int NT = NW * 64;
  constexpr int NL = CHUNKS / NT;            // pieces per thread and group
  static_assert(NL * NT == CHUNKS, "every thread loads the same number of pieces of a group");
  constexpr int XGROUP = 4 * NW * 1024;      // partial sums of one group: [point][fg][i][ks][lane]
  constexpr int RA = 8;                      // filter operand blocks in flight
  constexpr int STEPS = PP * CPW;            // filter operand blocks of the wave
  constexpr int NDB = (PP + 15) / 16;        // blocks of 16 positions' factors
  constexpr Order<ALG> order{};
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* vbuf = lds;
  unsigned char* xbuf = lds + splitk_lds_layout<ALG, KC, PLANES>(0);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int fgl = wave >> 2, ks = wave & 3;
  float* stage = (float*)lds + wave * (64 * M * (PLANES ? M : 1));
  int* tile_tab = (int*)(lds + splitk_lds_layout<ALG, KC, PLANES>(1));

  // workgroup -> (tile block, pair of filter groups).  Ids that share an XCD (an L2) cover a
  // contiguous range of positions; positions run over chunks of four filter pairs (slowest),
  // tile blocks, and the pairs of the chunk (fastest): the workgroups an XCD runs at a time are
  // then a few tile blocks times four filter pairs, and its L2 fetches about as many bytes of
  // V as of the filter operand (with the pairs fastest over all of them it would stream the
  // whole operand, 35 MB with 512 channels and 132 points, for two tile blocks).
  const int wpairs = fgroups / 2, tblocks = g.Tp >> 4;
  const int pos = xcd_contiguous(blockIdx.x, gridDim.x);
  constexpr int KBG = 4;
  const int chunk = pos / (KBG * tblocks), crem = pos - chunk * (KBG * tblocks);
  const int in_chunk = min(KBG, wpairs - chunk * KBG);  // the last chunk may be smaller
  const int tb = crem / in_chunk, kb = chunk * KBG + (crem - tb * in_chunk);
  const int t0 = tb * 16;
  const int fg = kb * 2 + fgl;    // this wave's group of 16 filters
  const int kq = 4 * fg + ks;     // the filter quad whose pairs it finishes

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
      (void*)U16, 0, (int)((unsigned)fgroups * (unsigned)(PP * CP * 16)), kBufferFlags);
  const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)dq16, 0, (int)((unsigned)fgroups * (unsigned)(PP * 64)), kBufferFlags);
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      y, 0, (int)(esz * (unsigned)(g.N * g.Cout) * (unsigned)(g.H * g.W)), kBufferFlags);

  // ---- V loader: piece q = tid + NT*i of a group is 16 bytes of (point r, tile, channels) with
  // r = q / (64*KC) uniform per wave; it lands in block r*KC + kc at [tile][16*kseg..], the
  // register image of the MFMA operand
  unsigned gsrc[NL], ldst[NL];
  int rsel[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int q = (int)threadIdx.x + NT * i;
    const int r = (wave * 64 + NT * i) / (64 * KC);  // uniform over the wave
    const int rem = q - r * (64 * KC);
    const int tile = rem / (4 * KC), ch = rem - tile * (4 * KC);
    rsel[i] = r;
    gsrc[i] = (unsigned)(t0 + tile) * (unsigned)CP + (unsigned)ch * 16u;
    ldst[i] = (unsigned)(((r * KC + (ch >> 2)) * 16 + tile) * 64 + (ch & 3) * 16);
  }
  v4i lreg[NL];
  auto load_regs = [&](int pg) {
    // positions without a point (the tail of the last group of an SFC-4 form) re-read point 0;
    // their filter operand is zero and their sums are never taken
    const int p0 = max(order.pt[4 * pg], 0), p1 = max(order.pt[4 * pg + 1], 0),
              p2 = max(order.pt[4 * pg + 2], 0), p3 = max(order.pt[4 * pg + 3], 0);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int r = rsel[i];
      const int p = r == 0 ? p0 : r == 1 ? p1 : r == 2 ? p2 : p3;
      lreg[i] = __builtin_amdgcn_raw_buffer_load_b128(vres, gsrc[i], (unsigned)p * vplane, 0);
    }
  };
  auto store_lds = [&](int pg) {
#pragma unroll
    for (int i = 0; i < NL; ++i) *(v4i*)(vbuf + (pg & 1) * GROUP_BYTES + ldst[i]) = lreg[i];
  };

  // ---- filter operand of (fg, channel quarter ks): block (position j, chunk) 1 KiB, 16 bytes
  // per lane; dequantization factors of the wave's final pairs (filter 16 fg + 4 ks + l/16):
  // 16 positions per load, taken by a row broadcast (sfc_quad16.hpp)
  const unsigned a_lane = (unsigned)lane * 16u;
  const unsigned a_wave = (unsigned)fg * (unsigned)(PP * KC * 1024) + (unsigned)(CPW * ks) * 1024u;
  v4i aring[RA];
  auto load_a = [&](int s) {  // step s = position * CPW + chunk of the wave
    const int j = s / CPW, c = s - j * CPW;
    aring[s % RA] = __builtin_amdgcn_raw_buffer_load_b128(ures, a_lane, a_wave + (unsigned)((j * KC + c) * 1024), 0);
  };
  const unsigned d_lane = (unsigned)(lane & 15) * 64u + (unsigned)(lane >> 4) * 16u + 4u * (unsigned)ks;
  const unsigned d_wave = (unsigned)fg * (unsigned)(PP * 64);
  float dblk[NDB];
#pragma unroll
  for (int m = 0; m < NDB; ++m)  // (a last block may reach past the wave's table: never used)
    dblk[m] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(dres, d_lane, d_wave + (unsigned)m * 1024u, 0));

  // ---- partial sums of group pg: CPW chained matrix instructions per point, the four
  // accumulator elements to xbuf[pg % 2][point][fg][i][ks][lane]
  const unsigned char* blane = vbuf + (CPW * ks) * 1024 + (lane & 15) * 64 + (lane >> 4) * 16;
  unsigned char* xw = xbuf + (fgl * 16 + ks) * 256 + lane * 4;        // + point*8 KiB + i*1 KiB
  const unsigned char* xr = xbuf + (fgl * 16 + ks * 4) * 256 + lane * 4;  // + point*8 KiB + ks'*256
  // (every LDS read of a step is issued before the first result is waited for: the operand
  // reads of four points, and the partial sums of the group that is being finished)
  auto read_b = [&](int pg, v4i (&b)[4][CPW]) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int c = 0; c < CPW; ++c)
        b[r][c] = *(const v4i*)(blane + (pg & 1) * GROUP_BYTES + (r * KC + c) * 1024);
  };
  auto partials = [&](int pg, const v4i (&b)[4][CPW]) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      v4i acc = {0, 0, 0, 0};
#pragma unroll
      for (int c = 0; c < CPW; ++c) {
        const int s = (4 * pg + r) * CPW + c;
        acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(aring[s % RA], b[r][c], acc, 0, 0, 0);
        if (s + RA < STEPS) load_a(s + RA);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) *(int*)(xw + (pg & 1) * XGROUP + r * (NW * 1024) + i * 1024) = acc[i];
    }
  };

  load_regs(0);
#pragma unroll
  for (int s = 0; s < RA && s < STEPS; ++s) load_a(s);
  store_lds(0);
  if (PG > 1) load_regs(1);
  __syncthreads();
  {
    v4i b[4][CPW];
    read_b(0, b);
    partials(0, b);
  }
  if (PG > 1) store_lds(1);
  if (PG > 2) load_regs(2);
  __syncthreads();

  float cur[4];
  auto next = [&](auto position) __attribute__((always_inline)) -> float {
    constexpr int j = decltype(position)::value;
    constexpr int r = j & 3, pg = j >> 2;
    if constexpr (r == 0) {
      // the partial sums of group pg (all four waves of the filter group wrote them before the
      // last barrier) and the operands of group pg + 1: every read goes out first
      int part[4][4];
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        const unsigned char* src = xr + (pg & 1) * XGROUP + rr * (NW * 1024);
#pragma unroll
        for (int k = 0; k < 4; ++k) part[rr][k] = *(const int*)(src + 256 * k);
      }
      v4i b[4][CPW];
      if (pg + 1 < PG) read_b(pg + 1, b);
      // V of group pg + 2 into the buffer group pg has left; group pg + 3 requested
      if (pg + 2 < PG) store_lds(pg + 2);
      if (pg + 3 < PG) load_regs(pg + 3);
      __builtin_amdgcn_sched_barrier(0);
      // group pg + 1: its partial sums go to the other exchange buffer
      if (pg + 1 < PG) partials(pg + 1, b);
      // the sums of group pg over all channels, scaled
      constexpr int jj = 4 * pg;  // the lane index of a row broadcast is a compile-time constant
      const float d0 = row_lane<(jj + 0) & 15>(dblk[(jj + 0) >> 4]), d1 = row_lane<(jj + 1) & 15>(dblk[(jj + 1) >> 4]),
                  d2 = row_lane<(jj + 2) & 15>(dblk[(jj + 2) >> 4]), d3 = row_lane<(jj + 3) & 15>(dblk[(jj + 3) >> 4]);
      const float dd[4] = {d0, d1, d2, d3};
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        float v = (float)((part[rr][0] + part[rr][1]) + (part[rr][2] + part[rr][3])) * dd[rr];
        asm volatile("" : "+v"(v));
        cur[rr] = v;
      }
      __syncthreads();  // partial sums of group pg + 1 and V of group pg + 2 are in place
      __builtin_amdgcn_sched_barrier(0);
    }
    return cur[r];
  };
  float z[NC][M];
  stream_vertical<ALG, float>(next, z);

  __syncthreads();  // every wave has taken its last sums: the buffers become store staging
  if constexpr (PLANES)
    store_planes<ALG, OUT>(z, stage, tile_tab, lane, kq, x_scale, inv_y, yres, g.Cout, g.th, g.tw);
  else
    store_pairs<ALG, OUT, VEC2>(z, stage, tile_tab, lane, kq, x_scale, inv_y, yres, g.Cout, g.H, g.W);
}

// filters covered by the regrouped operand: Cout rounded up to whole workgroups
int splitk_filter_count(const Geometry& g) {
  return (g.Cout + kSplitFilters - 1) / kSplitFilters * kSplitFilters;
}

bool splitk_supported(const Geometry& g) {
  if (g.alg < 2 || g.alg > 5) return false;  // SFC-6(7x7,3x3) and SFC-4(4x4,3x3)
  if (g.Cp != 512) return false;
  const long long fgroups = splitk_filter_count(g) / 16;
  // Small layers only (at most two workgroups per compute unit): there it is ahead of the
  // one-pair-per-lane kernel (512 channels on 7x7 maps, batch 64, 4x4 tiles: 27.3 against
  // 30.7 us per layer; 7x7 tiles at batch 256: 67.3 against 74.7), on larger ones level or
  // behind (4x4 tiles at batch 256: 85 to 91 against 85.9).
  if ((long long)(g.Tp / 16) * (fgroups / 2) > 512) return false;
  const long long ybytes = 4ll * g.N * g.Cout * g.H * g.W;
  const long long vbytes = (long long)g.P * g.Tp * g.Cp;
  const long long ubytes = fgroups * 16 * ((g.P + 3) / 4 * 4) * g.Cp;
  const long long lim = 1ll << 31;
  return ybytes < lim && vbytes < lim && ubytes < lim;
}

template <int ALG, int OUT, bool VEC2, bool PLANES>
static hipError_t launch_splitk_impl(const Geometry& g, const void* V, const FilterViews& f,
                                     float x_scale, float inv_y, void* y, hipStream_t s,
                                     bool prepare) {
  constexpr int KC = 8;
  auto kernel = splitk_kernel<ALG, KC, OUT, VEC2, PLANES>;
  constexpr unsigned lds_bytes = splitk_lds_layout<ALG, KC, PLANES>(2);
  static_assert(lds_bytes <= 160u * 1024u, "buffers and staging exceed the LDS of a compute unit");
  if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel));
  const int fgroups = splitk_filter_count(g) / 16;
  const dim3 grid((unsigned)((g.Tp / 16) * (fgroups / 2)));
  hipLaunchKernelGGL(kernel, grid, dim3(kSplitWaves * 64), lds_bytes, s, (const int8_t*)V,
                     (const int8_t*)f.U_single, f.dequant_single, x_scale, inv_y, y, g, fgroups);
  return hipGetLastError();
}

template <int ALG>
static hipError_t launch_splitk_alg(int out, const Geometry& g, const void* V, const FilterViews& f,
                                    float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  constexpr int M = AlgTraits<ALG>::M;
  if (whole_image_tiles(M, g.H, g.W, g.th, g.tw, g.Cout))
    return out == 2 ? launch_splitk_impl<ALG, 2, false, true>(g, V, f, x_scale, inv_y, y, s, prepare)
                    : launch_splitk_impl<ALG, 0, false, true>(g, V, f, x_scale, inv_y, y, s, prepare);
  if constexpr (M % 2 == 0) {
    if (g.W % 2 == 0)
      return out == 2 ? launch_splitk_impl<ALG, 2, true, false>(g, V, f, x_scale, inv_y, y, s, prepare)
                      : launch_splitk_impl<ALG, 0, true, false>(g, V, f, x_scale, inv_y, y, s, prepare);
  }
  return out == 2 ? launch_splitk_impl<ALG, 2, false, false>(g, V, f, x_scale, inv_y, y, s, prepare)
                  : launch_splitk_impl<ALG, 0, false, false>(g, V, f, x_scale, inv_y, y, s, prepare);
}

hipError_t launch_splitk(int out, const Geometry& g, const void* V, const FilterViews& f,
                         float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  if (!splitk_supported(g) || out == 1) return hipErrorNotSupported;
  switch (g.alg) {
    case 2: return launch_splitk_alg<2>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 3: return launch_splitk_alg<3>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 4: return launch_splitk_alg<4>(out, g, V, f, x_scale, inv_y, y, s, prepare);
    case 5: return launch_splitk_alg<5>(out, g, V, f, x_scale, inv_y, y, s, prepare);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
