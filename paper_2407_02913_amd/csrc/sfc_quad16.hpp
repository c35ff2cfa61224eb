// Transform-domain products + output transform for the SFC-4(4x4,3x3) forms with no surplus
// matrix work (gfx950): a wave owns 16 tiles x 16 filters, four (tile, filter) pairs per lane.
//
// The int8 MFMA 16x16x64 gives lane l the four results D[4(l/16) + i][l%16], i = 0..3.  With
// the A operand holding ONE point for 16 filters (row r = filter f0 + 4(r%4) + r/4) and the B
// operand V of the same point for 16 tiles, every accumulator element is a wanted product:
// lane l gets, for tile l%16, the filters f0 + 4i + l/16 -- filter l/16 of the four filter
// quads f0/4 + i.  The 46 / 49 points of SFC-4 leave 6 x 4 partial outputs per pair, so four
// pairs fit a lane's registers and the streaming output transform runs on four-element
// vectors.  Per product that is a quarter of the matrix instructions, LDS reads of V and
// filter-operand bytes of the one-pair-per-lane form (sfc_fused_quad.hpp), which spends three
// of four accumulator elements on mixed points.
#pragma once
#include <type_traits>

#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"
#include "sfc_store.hpp"

namespace sfc {

// four floats that the add networks of sfc_points.hpp treat as one value
struct f4 {
  float v[4];
  f4() = default;
  __device__ __forceinline__ explicit f4(float s) : v{s, s, s, s} {}
};
__device__ __forceinline__ f4 operator+(const f4& a, const f4& b) {
  f4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r.v[i] = a.v[i] + b.v[i];
  return r;
}
__device__ __forceinline__ f4 operator-(const f4& a, const f4& b) {
  f4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r.v[i] = a.v[i] - b.v[i];
  return r;
}
__device__ __forceinline__ f4 operator*(const f4& a, const f4& b) {
  f4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r.v[i] = a.v[i] * b.v[i];
  return r;
}
__device__ __forceinline__ f4 operator-(const f4& a) {
  f4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r.v[i] = -a.v[i];
  return r;
}
template <>
struct Half<f4> {
  static __device__ __forceinline__ f4 apply(const f4& a) { return a * f4(0.5f); }
};

// Lane n of the reader's row of 16 lanes (its quarter of the wave), as a DPP row broadcast:
// folds into the instruction that takes the value.
template <int N>
__device__ __forceinline__ float row_lane(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x150 + N, 0xf, 0xf, false));
}

// V buffers of the fused kernel (groups of four points in LDS) and groups in flight in
// registers behind them, by channel chunks: the load of a group is issued kVRegs groups
// before its products
constexpr int quad16_vbufs(int kc) { return kc >= 8 ? 2 : 3; }
// (four chunks: three groups ahead, 256 channels on 14x14 maps at batch 128 38.2 us per layer
// against 39.8 with one; eight chunks leave no registers for more than one)
constexpr int quad16_vregs(int kc) { return kc >= 8 ? 1 : kc == 4 ? 3 : 2; }

// LDS of the products + output kernel: the V buffers, which the per-wave store staging
// blocks (16 filters x 16 tiles x 16 outputs, float32 or int8) take over once the last
// products are done, then the tile table.
template <int KC, int NW, int OUT>
constexpr unsigned quad16_lds_layout(int what) {
  constexpr unsigned vbytes = (unsigned)quad16_vbufs(KC) * 4u * 16u * 64u * KC;
  constexpr unsigned stage = NW * 4096u * (OUT == 2 ? 1u : 4u);
  constexpr unsigned tab_off = vbytes > stage ? vbytes : stage;
  return what == 0 ? 0u : what == 1 ? tab_off : tab_off + 256u;
}

// The products and the output transform of one wave: 16 tiles (V in LDS, groups of four
// points in a ring of buffers kept filled by `sync`) x 16 filters (operand and dequantization
// factors from global memory, a ring of loads ahead).
//   vbuf, VB      ring of VB buffers of 4 x KC blocks of 1 KiB ([point][chunk][tile][64 channels]);
//                 group pg lives in buffer pg % VB
//   ures, a_wave  filter operand: block (position j, chunk kc) at a_wave + (j*KC + kc) KiB,
//                 16 bytes per lane
//   dres, d_wave  dequantization factors: 16 floats per position at d_wave + 64 j, lane
//                 quarter l/16 takes four.  They are loaded once, 16 positions per
//                 instruction (lane (quarter, n) fetches those of position 16 m + n), and a
//                 product takes its factors from lane n of its quarter by a row broadcast: a
//                 load per position and wave instead kept the compute unit's vector-memory
//                 path busy with 64-byte pieces.
//   sync(pg)      called when the wave has read the last V of group pg (or issued its last
//                 products): returns once group pg + 1 is in place; it may overwrite the
//                 buffers of the groups before pg
// Software pipeline: call j issues the matrix instructions of position j + 1 and then converts
// the sums of position j, so the matrix pipe works under the vector arithmetic of the output
// transform.  Leaves z[b][o1] of the lane's four pairs (f4 element i: filter quad i).
template <int ALG, int KC, int VB, int PS = KC * 1024, typename Sync>
__device__ __forceinline__ void quad16_products(const unsigned char* vbuf, int lane,
                                                __amdgpu_buffer_rsrc_t ures, unsigned a_wave,
                                                __amdgpu_buffer_rsrc_t dres, unsigned d_wave,
                                                Sync&& sync,
                                                f4 (&z)[AlgTraits<ALG>::NC][AlgTraits<ALG>::M]) {
  constexpr int PP = Order<ALG>::PP;
  constexpr int GROUP_BYTES = 4 * PS;      // PS: bytes from one position's V to the next
  constexpr int STEPS = PP * KC;           // filter-operand blocks of the wave
  constexpr int RA = 8;                    // ... in flight
  constexpr int NDB = (PP + 15) / 16;      // blocks of 16 positions' factors
  const unsigned a_lane = (unsigned)lane * 16u;
  const unsigned d_lane = (unsigned)(lane & 15) * 64u + (unsigned)(lane >> 4) * 16u;
  v4i aring[RA];
  v4f dblk[NDB];
  auto load_a = [&](int s) {
    aring[s % RA] = __builtin_amdgcn_raw_buffer_load_b128(ures, a_lane, a_wave + (unsigned)s * 1024u, 0);
  };
#pragma unroll
  for (int m = 0; m < NDB; ++m)  // (a last block may reach past the wave's table: never used)
    dblk[m] = __builtin_bit_cast(
        v4f, __builtin_amdgcn_raw_buffer_load_b128(dres, d_lane, d_wave + (unsigned)m * 1024u, 0));
#pragma unroll
  for (int s = 0; s < RA && s < STEPS; ++s) load_a(s);
  const unsigned char* blane = vbuf + (lane & 15) * 64 + (lane >> 4) * 16;
  // V of position jj for the lane's tile: KC reads of 16 bytes.  Up to two chunks they are
  // issued a call ahead of the matrix instructions that take them (PREB); with more the
  // chain of matrix instructions is long enough to read them as it goes.
  constexpr bool PREB = KC <= 2;
  constexpr int NB = PREB ? KC : 1;
  v4i breg[NB];
  auto read_b = [&](int jj) {
    const unsigned char* bsrc = blane + ((jj >> 2) % VB) * GROUP_BYTES + (jj & 3) * PS;
#pragma unroll
    for (int kc = 0; kc < NB; ++kc) breg[kc] = *(const v4i*)(bsrc + kc * 1024);
  };
  // the sums of position jj: KC chained matrix instructions
  auto products = [&](int jj) -> v4i {
    v4i acc = {0, 0, 0, 0};
    const unsigned char* bsrc = blane + ((jj >> 2) % VB) * GROUP_BYTES + (jj & 3) * PS;
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int s = jj * KC + kc;
      v4i b;
      if constexpr (PREB) b = breg[kc];
      else b = *(const v4i*)(bsrc + kc * 1024);
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(aring[s % RA], b, acc, 0, 0, 0);
      if (s + RA < STEPS) load_a(s + RA);
    }
    return acc;
  };
  if constexpr (PREB) read_b(0);
  v4i acc_cur = products(0);
  if constexpr (PREB) read_b(1);
  // (the streaming output transform asks for the products in order and names the position)
  auto next = [&](auto position) __attribute__((always_inline)) -> f4 {
    constexpr int j = decltype(position)::value;
    v4i acc_new = acc_cur;
    if constexpr (PREB) {
      if (j + 1 < PP) acc_new = products(j + 1);
      if (j + 2 < PP) {
        if (((j + 2) & 3) == 0) sync((j + 2) / 4 - 1);
        read_b(j + 2);
      }
    } else if (j + 1 < PP) {
      if (((j + 1) & 3) == 0) sync((j + 1) / 4 - 1);
      acc_new = products(j + 1);
    }
    __builtin_amdgcn_sched_barrier(0);  // the matrix instructions go first
    f4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float t = (float)acc_cur[i] * row_lane<j & 15>(dblk[j >> 4][i]);
      // the scaled products are materialized here, the accumulator is not kept alive
      asm volatile("" : "+v"(t));
      v.v[i] = t;
    }
    acc_cur = acc_new;
    __builtin_amdgcn_sched_barrier(0);
    return v;
  };
  // positions P .. PP-1 hold no point: their filter operand is zero, their products unused
  stream_vertical<ALG, f4>(next, z);
}

// y of the wave's 16 tiles x 16 filters from z (pair i of lane l: tile l%16, filter
// 4*(kq0 + i) + l/16).  Every lane finishes its 4 x 4 x 4 outputs (inverse along the horizontal
// axis, activation scale; OUT = 2: ReLU and rounding to the next layer's int8) and stages them
// in the wave's block as [filter 16][tile 16][row 4][4 outputs]; then lane l takes row l/16 of
// tile l%16 for one filter after the other, so that a store instruction writes, for one
// filter, four image rows of 16 neighbouring tiles: consecutive lanes hold consecutive
// pieces of an image row.  No branches: a piece outside the image, or of a filter beyond
// Cout, gets an offset outside the buffer and is dropped by the bounds check.
// EV: elements per store instruction, 4 when W is a multiple of 4 (a tile row never crosses
// the end of an image row), else 2 (W even) or 1.
template <int ALG, int OUT, int EV>
__device__ __forceinline__ void quad16_store(const f4 (&z)[AlgTraits<ALG>::NC][AlgTraits<ALG>::M],
                                             unsigned char* stage, const int* tile_tab, int lane,
                                             int kq0, float x_scale, float inv_y,
                                             __amdgpu_buffer_rsrc_t yres, const Geometry& g) {
  constexpr int NC = AlgTraits<ALG>::NC, M = AlgTraits<ALG>::M;
  static_assert(M == 4, "tiles of 4 x 4 outputs");
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  constexpr unsigned kOutOfRange = 0x80000000u;
  constexpr float kMagic = 12582912.0f;
  const int tl = lane & 15, q = lane >> 4;
  const float act = x_scale * inv_y;  // int8 output: activation scale over output scale
  // float32 staging: 16-byte slots, slot (tile, row) of a filter moved round by tile/4 so
  // that the 16 lanes of a quarter wave fall into different banks, writing and reading
  auto slot = [](int tile, int row) { return tile * 4 + ((row + (tile >> 2)) & 3); };
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float zi[NC][M];
#pragma unroll
    for (int b = 0; b < NC; ++b)
#pragma unroll
      for (int o = 0; o < M; ++o) zi[b][o] = z[b][o].v[i];
    const int f = 4 * i + q;
#pragma unroll
    for (int o1 = 0; o1 < M; ++o1) {
      float out[M];
      stream_row<ALG, float>(zi, o1, out);
      if constexpr (OUT == 2) {
        unsigned b[M];
#pragma unroll
        for (int o2 = 0; o2 < M; ++o2) {
          // next layer's activation: ReLU, round half to even, clamp to [0, 127]
          float t = __fmaf_rn(out[o2], act, kMagic);
          t = __builtin_amdgcn_fmed3f(t, kMagic, kMagic + 127.0f);
          b[o2] = __float_as_uint(t);
        }
        // the low bytes of the four outputs -> one dword
        const unsigned word = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u) | __builtin_amdgcn_perm(b[3], b[2], 0x04000c0cu);
        // (rows moved round by the quarter: the four quarters of the wave write different banks)
        *(unsigned*)(stage + ((f * 16 + tl) * 4 + ((o1 + q) & 3)) * 4) = word;
      } else {
        *(v4f*)(stage + (f * 64 + slot(tl, o1)) * 16) =
            v4f{out[0] * x_scale, out[1] * x_scale, out[2] * x_scale, out[3] * x_scale};
      }
    }
  }
  __builtin_amdgcn_wave_barrier();  // LDS accesses of one wave complete in order
  // this lane's piece: row q of tile tl
  const int HW = g.H * g.W;
  const bool row_ok = q < tile_tab[16 + tl];
  const int cols = row_ok ? tile_tab[32 + tl] : 0;
  const unsigned base = (unsigned)(tile_tab[tl] + q * g.W);  // elements, filter 0
  const bool stream = g.W >= 48;  // whole long rows per workgroup: past the L2
  auto run = [&](auto policy) {
  constexpr bool kStream = decltype(policy)::value;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int kc = 4 * kq0 + k;
    const unsigned off = esz * (base + (unsigned)kc * (unsigned)HW);
    const int ncol = kc < g.Cout ? cols : 0;
    if constexpr (OUT == 2) {
      const unsigned word = *(const unsigned*)(stage + ((k * 16 + tl) * 4 + ((q + k) & 3)) * 4);
      if constexpr (EV == 4) {
        const unsigned o = ncol > 0 ? off : kOutOfRange;
        if constexpr (kStream) __builtin_amdgcn_raw_buffer_store_b32(word, yres, o, 0, kStreamStore);
        else __builtin_amdgcn_raw_buffer_store_b32(word, yres, o, 0, 0);
      } else if constexpr (EV == 2) {
        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)word, yres, ncol > 0 ? off : kOutOfRange, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(word >> 16), yres,
                                              ncol > 2 ? off + 2u : kOutOfRange, 0, 0);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          __builtin_amdgcn_raw_buffer_store_b8((unsigned char)(word >> (8 * e)), yres,
                                               ncol > e ? off + (unsigned)e : kOutOfRange, 0, 0);
      }
    } else {
      const v4f v = *(const v4f*)(stage + (k * 64 + slot(tl, q)) * 16);
      if constexpr (EV == 4) {
        const unsigned o = ncol > 0 ? off : kOutOfRange;
        if constexpr (kStream) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, v), yres, o, 0, kStreamStore);
        else __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, v), yres, o, 0, 0);
      } else if constexpr (EV == 2) {
        __builtin_amdgcn_raw_buffer_store_b64(v2f{v[0], v[1]}, yres, ncol > 0 ? off : kOutOfRange, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b64(v2f{v[2], v[3]}, yres, ncol > 2 ? off + 8u : kOutOfRange, 0, 0);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v[e]), yres,
                                                ncol > e ? off + 4u * (unsigned)e : kOutOfRange, 0, 0);
      }
    }
  }
  };
  if (stream) run(std::true_type{});
  else run(std::false_type{});
}

// Products + output transform with V from the input-transform kernel (fused path).  A
// workgroup of NW waves owns 16 consecutive tiles and 16*NW filters; per group of four points
// it copies 4 x 16 x Cin bytes of V from memory into one of two LDS buffers (already in
// operand order) while the previous group is multiplied, one barrier per group.
template <int ALG, int KC, int OUT, int EV, int NW>
__global__ __launch_bounds__(NW * 64, 2) void quad16_kernel(
    const int8_t* __restrict__ V, const int8_t* __restrict__ U16, const float* __restrict__ dq16,
    float x_scale, float inv_y, void* __restrict__ y, Geometry g, int fgroups) {
  using Tr = AlgTraits<ALG>;
  constexpr int P = Tr::P, M = Tr::M, NC = Tr::NC;
  constexpr int PP = Order<ALG>::PP, PG = PP / 4;
  constexpr int CP = KC * 64;
  constexpr int GROUP_BYTES = 4 * 16 * CP;
  constexpr int CHUNKS = GROUP_BYTES / 16;
  constexpr int NT = NW * 64;
  constexpr int NL = CHUNKS / NT;
  static_assert(NL * NT == CHUNKS, "every thread loads the same number of pieces of a group");
  constexpr Order<ALG> order{};
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* vbuf = lds;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  unsigned char* stage = lds + wave * (4096 * (OUT == 2 ? 1 : 4));
  int* tile_tab = (int*)(lds + quad16_lds_layout<KC, NW, OUT>(1));

  // workgroup -> (tile block, group of NW*16 filters): the workgroups an XCD runs side by
  // side share tile blocks (filter group fastest), so V is fetched into its L2 once
  const int wgroups = fgroups / NW;  // filter groups of a workgroup's size
  const int pos = xcd_contiguous(blockIdx.x, gridDim.x);
  const int tb = pos / wgroups, kb = pos - tb * wgroups;
  const int t0 = tb * 16;
  const int fg = kb * NW + wave;  // this wave's group of 16 filters

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

  // loader: piece q = tid + NT*i of a group is 16 bytes of (point r, tile, channels) with
  // r = q / (64*KC) uniform per wave; it lands in block r*KC + kc at [tile][16*kseg..]
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
  // Group pg is loaded into register set pg % VR when group pg - VR has been handed to LDS,
  // and handed to LDS buffer pg % VB when the products of group pg - 1 have been issued; the
  // barrier after that also tells that every wave is done with group pg - 2, whose buffer
  // group pg + 1 will take (VB >= 2; with VB = 3 the store may run a group earlier).
  constexpr int VB = quad16_vbufs(KC), VR = quad16_vregs(KC);
  v4i lreg[VR][NL];
  auto load_regs = [&](int pg) {
    const int p0 = max(order.pt[4 * pg], 0), p1 = max(order.pt[4 * pg + 1], 0),
              p2 = max(order.pt[4 * pg + 2], 0), p3 = max(order.pt[4 * pg + 3], 0);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int r = rsel[i];
      const int p = r == 0 ? p0 : r == 1 ? p1 : r == 2 ? p2 : p3;
      lreg[pg % VR][i] = __builtin_amdgcn_raw_buffer_load_b128(vres, gsrc[i], (unsigned)p * vplane, 0);
    }
  };
  auto store_lds = [&](int pg) {
#pragma unroll
    for (int i = 0; i < NL; ++i) *(v4i*)(vbuf + (pg % VB) * GROUP_BYTES + ldst[i]) = lreg[pg % VR][i];
  };
#pragma unroll
  for (int pg = 0; pg < VR && pg < PG; ++pg) load_regs(pg);
  store_lds(0);
  if (VR < PG) load_regs(VR);
  __syncthreads();

  auto sync = [&](int pg) {  // the products of group pg are issued: bring in group pg + 1
    if (pg + 1 < PG) store_lds(pg + 1);
    if (pg + 1 + VR < PG) load_regs(pg + 1 + VR);
    __syncthreads();
  };
  f4 z[NC][M];
  quad16_products<ALG, KC, VB>(vbuf, lane, ures, (unsigned)fg * (unsigned)(PP * KC * 1024), dres,
                           (unsigned)fg * (unsigned)(PP * 64), sync, z);
  __syncthreads();  // the staging blocks take the place of the V buffers
  quad16_store<ALG, OUT, EV>(z, stage, tile_tab, lane, fg * 4, x_scale, inv_y, yres, g);
}

}  // namespace sfc
