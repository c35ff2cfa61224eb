// The whole hot path of the SFC-4(4x4,3x3) forms in one kernel for layers with 129 to 512
// input channels on small feature maps (gfx950): neither V nor M leaves the compute unit.
//
// With more than two 64-channel chunks V of a workgroup's 16 tiles no longer fits the LDS at
// once.  Instead the sums of the multiplication points stay in accumulator registers while the
// workgroup walks over the channel chunks:
//  1. Stage: the channel planes of the workgroup's images (whole images of at most 16 tiles),
//     all chunks, are copied to LDS once.
//  2. Per chunk: input transform on the matrix cores (sfc_mfma_input.hpp), V of this chunk
//     to LDS (1 KiB per point), then one matrix instruction per point adds the chunk's
//     products to the point's accumulator: a wave owns 16 tiles x 16 filters, four (tile,
//     filter) pairs per lane, filter operand from global memory (sfc_quad16.hpp's layout).
//  3. Output transform of the four pairs from the accumulators, block store.
// The 46 / 49 points of a filter group are split between two waves (real columns, complex
// column group), so that a wave holds at most 28 accumulators and two waves share a SIMD.
// A workgroup covers 64 filters; with more filters the workgroups of a tile block repeat its
// input transform, which the matrix cores make cheap enough (256 channels and filters: four
// times).
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_mfma_input.hpp"
#include "sfc_points.hpp"
#include "sfc_quad16.hpp"
#include "sfc_tile_input.hpp"

namespace sfc {

struct Single16kPlan {
  TileRect tr;
  int fgroups;        // groups of 16 filters in all; a workgroup takes four
  unsigned chunk_in;  // LDS bytes of one staged 64-channel chunk
  unsigned v_off;     // LDS byte offset of the chunk's V
  unsigned tab_off;   // ... of the tile table
  unsigned lds_bytes;
};

// The products of positions J0 .. J1-1 for one chunk: one matrix instruction per position
// into its accumulator, V from LDS a position ahead, the filter operand from a ring of RA
// loads ahead that runs on into the next chunk.
template <int J0, int J1, int NA, int RA, int VS, typename LoadA>
__device__ __forceinline__ void chunk_products(const unsigned char* blane, v4i (&acc)[NA],
                                               v4i (&aring)[RA], int kc, LoadA&& load_a) {
  constexpr int NJ = J1 - J0;
  static_assert(NJ % RA == 0, "the ring index of a position does not depend on the chunk");
  v4i b_nxt = *(const v4i*)(blane + J0 * VS);
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const v4i b = b_nxt;
    if (j + 1 < NJ) b_nxt = *(const v4i*)(blane + (J0 + j + 1) * VS);
    acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(aring[j % RA], b, acc[j], 0, 0, 0);
    // the slot is free: the block RA positions on, which may lie in the next chunk
    if (j + RA < NJ) load_a(J0 + j + RA, kc, j % RA);
    else load_a(J0 + j + RA - NJ, kc + 1, j % RA);
  }
}

// A workgroup of eight waves owns 16 tiles and 64 filters.  Waves 0..3 ("real") take, for one
// group of 16 filters each, the 28 points of the four real columns; waves 4..7 ("complex") the
// points of the complex column group of the same filters.  The two halves of the output
// transform touch different partial outputs (z[0,1,4,5] and z[2,3]), so each wave finishes its
// own; the complex waves then hand z[2], z[3] over through LDS and the real waves store.
template <int ALG, int OUT, int EV>
__global__ __launch_bounds__(512, 2) void single16k_kernel(
    const int8_t* __restrict__ x, const int8_t* __restrict__ U16, const float* __restrict__ dq16,
    const unsigned char* __restrict__ intab, float x_scale, float inv_y, void* __restrict__ y,
    Geometry g, Single16kPlan sp) {
  using Tr = AlgTraits<ALG>;
  constexpr int M = Tr::M, NC = Tr::NC, PAD = Tr::PAD;
  constexpr int PP = Order<ALG>::PP;
  constexpr int NW = 8, SPW = 16 / NW;
  constexpr int JR = 28;             // positions of the real columns (4 x 7)
  constexpr int JC = PP - JR;        // ... of the complex column group, padded (20 / 24)
  constexpr int VS = 1024 + 16;      // bytes of V per position (16 positions written at once: banks)
  constexpr int NPB = MfmaInput<ALG>::NPB;
  constexpr int RA = 4, RD = 4;
  const int KC = g.Cp >> 6;  // 64-channel chunks
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int role = wave >> 2;  // 0: real columns, 1: complex column group
  const TileRect& tr = sp.tr;
  const int bx = xcd_contiguous(blockIdx.x, gridDim.x);
  unsigned char* vbuf = lds + sp.v_off;
  int* tile_tab = (int*)(lds + sp.tab_off);
  if (threadIdx.x < 16) {
    const int tl = threadIdx.x;
    const TileCoord tc = tile_coord(g, tr, bx, tl);
    write_tile_entry<M>(tile_tab, tl, tc.live, tc.n, tc.ti, tc.tj, g.Cout, g.H, g.W);
  }

  // ---- 1. stage every chunk ------------------------------------------------------------
#pragma unroll 1
  for (int kc = 0; kc < KC; ++kc)
    stage_images<NW, 16>(x, lds + 16 + kc * sp.chunk_in, g, tr, bx, 64 * kc, wave, lane);

  // ---- filter operand and accumulators ---------------------------------------------------
  const int fg = blockIdx.y * 4 + (wave & 3);  // groups beyond the last read zeros, store nothing
  const __amdgpu_buffer_rsrc_t ures = __builtin_amdgcn_make_buffer_rsrc(
      (void*)U16, 0, (int)((unsigned)sp.fgroups * (unsigned)(PP * KC * 1024)), kBufferFlags);
  const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)dq16, 0, (int)((unsigned)sp.fgroups * (unsigned)(PP * 64)), kBufferFlags);
  const unsigned a_lane = (unsigned)lane * 16u;
  const unsigned a_wave = (unsigned)fg * (unsigned)(PP * KC * 1024);
  v4i aring[RA];
  // block (position j, chunk kc) of the wave's operand into ring slot `slot`; beyond the last
  // chunk the offset leaves the buffer and the load returns zeros
  auto load_a = [&](int j, int kc, int slot) {
    const unsigned off = kc < KC ? a_wave + (unsigned)(j * KC + kc) * 1024u : 0x80000000u;
    aring[slot] = __builtin_amdgcn_raw_buffer_load_b128(ures, a_lane, off, 0);
  };
  static_assert(JC <= JR, "one accumulator array serves both roles");
  v4i acc[JR];  // the complex waves use the first JC
#pragma unroll
  for (int j = 0; j < RA; ++j) load_a((role == 0 ? 0 : JR) + j, 0, j);
#pragma unroll
  for (int j = 0; j < JR; ++j) acc[j] = v4i{0, 0, 0, 0};
  MfmaInput<ALG> mi;
  mi.load(intab, lane);
  __syncthreads();

  // ---- 2. chunk by chunk: input transform, V, products --------------------------------------
  const unsigned char* blane = vbuf + (lane & 15) * 64 + (lane >> 4) * 16;
  // the wave's tiles: plane offsets and patch geometry do not depend on the chunk
  typename MfmaInput<ALG>::PlaneTile pt[SPW];
  int pbase[SPW];
#pragma unroll
  for (int it = 0; it < SPW; ++it) {
    const int tile = wave + NW * it;
    const int tpi = g.th * g.tw;
    const int slot = tile / tpi, rem = tile - slot * tpi;
    const int ti = rem / g.tw, tj = rem - ti * g.tw;
    pbase[it] = 16 + slot * 64 * tr.cs;  // (16: the patch reads start up to 4 bytes early)
    pt[it] = MfmaInput<ALG>::plane_tile(M * ti - PAD, M * tj - PAD, g.H, g.W, lane);
  }
#pragma unroll 1
  for (int kc = 0; kc < KC; ++kc) {
    const unsigned char* in = lds + kc * sp.chunk_in;
    unsigned packed[SPW * 4][NPB];
#pragma unroll
    for (int it = 0; it < SPW; ++it) {
      const int tile = wave + NW * it;
      if (tile < tr.ntiles) {
#pragma unroll
        for (int cg = 0; cg < 4; ++cg)
          mi.transform(MfmaInput<ALG>::operand_plane(in + pbase[it], tr.cs, 16 * cg, pt[it], lane), g.qmax,
                       packed[4 * it + cg]);
      }
    }
    if (kc > 0) __syncthreads();  // every wave is done with the previous chunk's V
#pragma unroll
    for (int it = 0; it < SPW; ++it) {
      const int tile = wave + NW * it;
      if (tile < tr.ntiles) {
#pragma unroll
        for (int cg = 0; cg < 4; ++cg)
#pragma unroll
          for (int m = 0; m < NPB; ++m) {
            const int pos = 16 * m + (lane & 15);
            if (pos < PP)
              *(unsigned*)(vbuf + pos * VS + tile * 64 + 16 * cg + 4 * (lane >> 4)) = packed[4 * it + cg][m];
          }
      }
    }
    __syncthreads();
    if (role == 0) chunk_products<0, JR, JR, RA, VS>(blane, acc, aring, kc, load_a);
    else chunk_products<JR, PP, JR, RA, VS>(blane, acc, aring, kc, load_a);
  }

  // ---- 3. output transform from the accumulators, hand-over, store ------------------------------
  const unsigned d_lane = (unsigned)(lane >> 4) * 16u;
  const unsigned d_wave = (unsigned)fg * (unsigned)(PP * 64);
  v4f dring[RD];
  auto load_d = [&](int j, int slot) {
    dring[slot] = __builtin_bit_cast(
        v4f, __builtin_amdgcn_raw_buffer_load_b128(dres, d_lane, d_wave + (unsigned)j * 64u, 0));
  };
  f4 z[NC][M];
  // the hand-over block of filter group fg%4: z[2], z[3] as [component][row][lane] of four floats
  f4* xchg = (f4*)lds + (wave & 3) * (2 * M * 64);
  if (role == 0) {
#pragma unroll
    for (int j = 0; j < RD; ++j) load_d(j, j);
    int j = 0;  // folds to a constant after unrolling
    auto next = [&]() -> f4 {
      f4 v;
      const v4f d = dring[j % RD];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float t = (float)acc[j][i] * d[i];
        asm volatile("" : "+v"(t));  // the accumulator's registers are free from here on
        v.v[i] = t;
      }
      if (j + RD < JR) load_d(j + RD, j % RD);
      ++j;
      return v;
    };
    stream_vertical4_real<ALG, f4>(next, z);
  } else {
#pragma unroll
    for (int j = 0; j < RD; ++j) load_d(JR + j, j);
    int j = 0;
    auto next = [&]() -> f4 {
      f4 v;
      const v4f d = dring[j % RD];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float t = (float)acc[j][i] * d[i];
        asm volatile("" : "+v"(t));
        v.v[i] = t;
      }
      if (j + RD < JC) load_d(JR + j + RD, j % RD);
      ++j;
      return v;
    };
    stream_vertical4_complex<ALG, f4>(next, z);
  }
  __syncthreads();  // every wave is done with V and the staged planes: hand-over and staging blocks
  if (role == 1) {
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int o = 0; o < M; ++o) xchg[(b * M + o) * 64 + lane] = z[2 + b][o];
  }
  __syncthreads();
  if (role == 0) {
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int o = 0; o < M; ++o) z[2 + b][o] = xchg[(b * M + o) * 64 + lane];
  }
  __syncthreads();  // the staging blocks lie over the hand-over blocks
  if (role == 0) {
    constexpr unsigned esz = OUT == 2 ? 1u : 4u;
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
        y, 0, (int)(esz * (unsigned)(g.N * g.Cout) * (unsigned)(g.H * g.W)), kBufferFlags);
    quad16_store<ALG, OUT, EV>(z, lds + (wave & 3) * (4096 * (OUT == 2 ? 1 : 4)), tile_tab, lane, fg * 4,
                               x_scale, inv_y, yres, g);
  }
}

static bool make_single16k_plan(const Geometry& g, int out, Single16kPlan* sp) {
  if ((g.alg != 4 && g.alg != 5) || g.Cp <= 128 || g.Cp > 512) return false;
  const int kc = g.Cp / 64;
  const unsigned pp = (unsigned)((g.P + 3) / 4 * 4);
  const unsigned vbytes = pp * (1024u + 16u);
  const unsigned sbytes = 4u * (out == 2 ? 4096u : 16384u);
  const unsigned lds_max = 160u * 1024u - 256u;
  if (vbytes + sbytes > lds_max) return false;
  // whole images only (at most 16 tiles each), every chunk staged at once next to one chunk's V
  const int tpi = g.th * g.tw;
  if (tpi > 16 || g.H * g.W > 1024) return false;
  TileRect& tr = sp->tr;
  tr.whole = 1;
  tr.cs = plane_stride_bytes(g.H * g.W);
  tr.ipw = 16 / tpi < g.N ? 16 / tpi : g.N;
  while (tr.ipw > 1 && (unsigned)(tr.ipw * 64 * tr.cs) > (lds_max - vbytes - 16u) / (unsigned)kc) --tr.ipw;
  if ((unsigned)(tr.ipw * 64 * tr.cs) > (lds_max - vbytes - 16u) / (unsigned)kc) return false;
  tr.S = tr.chunks = tr.tlw = 1;
  tr.ntiles = tr.ipw * tpi;
  tr.th_magic = 0;
  sp->chunk_in = tile_rect_stage_bytes(g, sp->tr);
  unsigned in_bytes = 16u + sp->chunk_in * (unsigned)kc;
  if (in_bytes < sbytes) in_bytes = sbytes;  // the store staging blocks lie over the planes
  sp->v_off = (in_bytes + 15u) & ~15u;
  sp->tab_off = sp->v_off + ((vbytes + 15u) & ~15u);
  sp->lds_bytes = sp->tab_off + 256u;
  sp->fgroups = (g.Cout + 15) / 16;
  const long long xb = (long long)g.N * g.Cin * g.H * g.W;
  const long long yb = 4ll * g.N * g.Cout * g.H * g.W;
  const long long ub = (long long)sp->fgroups * 16 * pp * g.Cp;
  const long long lim = 1ll << 31;
  return sp->lds_bytes <= 160u * 1024u && xb < lim && yb < lim && ub < lim;
}

bool single16k_supported(const Geometry& g) {
  Single16kPlan sp;
  return make_single16k_plan(g, 0, &sp);
}

template <int ALG, int OUT, int EV>
static hipError_t launch_single16k_impl(const Geometry& g, const Single16kPlan& sp, const int8_t* x,
                                        const FilterViews& f, float x_scale, float inv_y, void* y,
                                        hipStream_t s, bool prepare) {
  auto kernel = single16k_kernel<ALG, OUT, EV>;
  if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel));
  const dim3 grid(tile_rect_groups(g, sp.tr), (unsigned)((sp.fgroups + 3) / 4));
  hipLaunchKernelGGL(kernel, grid, dim3(512), sp.lds_bytes, s, x, (const int8_t*)f.U_single,
                     f.dequant_single, f.input_tab, x_scale, inv_y, y, g, sp);
  return hipGetLastError();
}

template <int ALG>
static hipError_t launch_single16k_alg(int out, const Geometry& g, const Single16kPlan& sp,
                                       const int8_t* x, const FilterViews& f, float x_scale,
                                       float inv_y, void* y, hipStream_t s, bool prepare) {
  if (g.W % 4 == 0)
    return out == 2 ? launch_single16k_impl<ALG, 2, 4>(g, sp, x, f, x_scale, inv_y, y, s, prepare)
                    : launch_single16k_impl<ALG, 0, 4>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
  if (g.W % 2 == 0)
    return out == 2 ? launch_single16k_impl<ALG, 2, 2>(g, sp, x, f, x_scale, inv_y, y, s, prepare)
                    : launch_single16k_impl<ALG, 0, 2>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
  return out == 2 ? launch_single16k_impl<ALG, 2, 1>(g, sp, x, f, x_scale, inv_y, y, s, prepare)
                  : launch_single16k_impl<ALG, 0, 1>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
}

hipError_t launch_single16k(int out, const Geometry& g, const int8_t* x, const FilterViews& f,
                            float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  Single16kPlan sp;
  if (out == 1 || !make_single16k_plan(g, out, &sp)) return hipErrorNotSupported;
  return g.alg == 4 ? launch_single16k_alg<4>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare)
                    : launch_single16k_alg<5>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare);
}

}  // namespace sfc
