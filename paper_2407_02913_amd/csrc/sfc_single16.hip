// The whole hot path of the SFC-4(4x4,3x3) forms in one kernel for layers with up to 128 input
// channels (gfx950): input-tile transform, transform-domain products and output transform
// without V or M ever leaving the compute unit.
//
// A workgroup owns a rectangle of up to 16 tiles (S strips x tlw tile columns, or whole small
// images; sfc_tile_input.hpp), all input channels (one or two chunks of 64) and up to 128
// filters:
//  1. Stage: the six input rows of every (strip, channel) go to LDS with dword loads, lanes
//     running along the row, padding halo zero-filled.
//  2. Input transform: wave = tile, lane = input channel, one (tile, chunk) item after the
//     other.  Each thread reads its 6 x 6 patch, applies the four-point symbolic DFT add
//     network along rows and columns, forms the 46 / 49 multiplication points, rounds them to
//     int8 and writes V[position][chunk][tile][channel] (1 KiB per (position, chunk) = one MFMA
//     operand) over the staging area.
//  3. Products + output transform: a wave takes 16 filters at a time, four (tile, filter) pairs
//     per lane (sfc_quad16.hpp): V from LDS, filter operand and dequantization factors from
//     global memory, streaming output transform on four-element vectors.
//  4. Store: the wave's 16 x 16 x 16 outputs go through its LDS block (over V, once every
//     wave is done with it) and out as whole tile rows, four image rows of 16 tiles per filter
//     and instruction.
#include <cstring>

#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_mfma_input.hpp"
#include "sfc_points.hpp"
#include "sfc_quad16.hpp"
#include "sfc_tile_input.hpp"

namespace sfc {

struct Single16Plan {
  TileRect tr;
  int fgroups;         // groups of 16 filters in all; a workgroup takes one per wave
  unsigned chunk_in;   // LDS bytes of one staged 64-channel chunk
  unsigned tab_off;    // LDS byte offset of the tile table
  unsigned lds_bytes;
};

template <int ALG, int KC, int OUT, int EV, int NW>
__global__ __launch_bounds__(NW * 64, 2) void single16_kernel(
    const int8_t* __restrict__ x, const int8_t* __restrict__ U16, const float* __restrict__ dq16,
    const unsigned char* __restrict__ intab, float x_scale, float inv_y, void* __restrict__ y,
    Geometry g, Single16Plan sp) {
  using Tr = AlgTraits<ALG>;
  constexpr int M = Tr::M, NI = Tr::NI, NC = Tr::NC, PAD = Tr::PAD;
  constexpr int PP = Order<ALG>::PP, PG = PP / 4;
  static_assert(NW == 4 * KC, "one wave per (channel chunk, group of 16 channels)");
  constexpr int CS = stage_channel_bytes(NI);
  // bytes of V per position: KC operand blocks of 1 KiB and 16 bytes that put the 16 positions
  // a wave writes at once into different LDS banks
  constexpr int VS = KC * 1024 + 16;
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const TileRect& tr = sp.tr;
  const int bx = xcd_contiguous(blockIdx.x, gridDim.x);
  int* tile_tab = (int*)(lds + sp.tab_off);
  if (threadIdx.x < 16) {
    const int tl = threadIdx.x;
    const TileCoord tc = tile_coord(g, tr, bx, tl);
    write_tile_entry<M>(tile_tab, tl, tc.live, tc.n, tc.ti, tc.tj, g.Cout, g.H, g.W);
    if (!tr.whole) {
      // rectangle: where the patch of tile slot tl starts in the staged rows of a chunk
      // (slots beyond the rectangle repeat its last tile)
      const int t = min(tl, tr.ntiles - 1), s = t / tr.tlw, tj0 = (bx % tr.chunks) * tr.tlw;
      const int halo = M * tj0 - PAD - ((M * tj0) & ~3) + 4;  // LDS byte of the rectangle's first patch column
      tile_tab[48 + tl] = s * 64 * CS + halo + M * (t - s * tr.tlw);
    }
  }

  // ---- 1. stage ----------------------------------------------------------------------
#pragma unroll
  for (int kc = 0; kc < KC; ++kc)
    stage_input<ALG, NW>(x, lds + 16 + kc * sp.chunk_in, g, tr, bx, 64 * kc, wave, lane);
  __syncthreads();

  // ---- 2. input transform (sfc_mfma_input.hpp) --------------------------------------------
  // A patch is (tile, 64-channel chunk, group of 16 channels).  Wave w takes the patches of
  // chunk w / 4, channel group w % 4 of every tile, so all waves have the same number of them.
  // All patches are transformed, rounded and packed in registers before the first byte of V
  // is written, because V lies over the staged rows.
  {
    MfmaInput<ALG> mi;
    mi.load(intab, lane);
    constexpr int NPB = MfmaInput<ALG>::NPB;
    constexpr int NQ = 16;  // tile slots
    const int kc = wave >> 2, cg = wave & 3;
    const unsigned char* in = lds + 16 + kc * sp.chunk_in;  // (16: plane patches are read from up to 4 bytes early)
    unsigned packed[NQ][NPB];
    // Software pipeline: the LDS reads of patch q + 2 and the matrix instructions of patch
    // q + 1 are issued before patch q is rounded, so neither latency is waited for.  (An empty
    // tile slot repeats the last tile: its bytes are not written.)
    auto run = [&](auto whole_images) __attribute__((always_inline)) {
      constexpr bool kWhole = decltype(whole_images)::value;
      auto fetch = [&](int q) __attribute__((always_inline)) -> v4i {  // q folds to a constant
        if constexpr (kWhole) {
          const int tile = min(q, tr.ntiles - 1);
          const int tpi = g.th * g.tw;
          const int slot = tile / tpi, rem = tile - slot * tpi;
          const int ti = rem / g.tw, tj = rem - ti * g.tw;
          return MfmaInput<ALG>::operand_plane(in + slot * 64 * tr.cs, tr.cs, 16 * cg, M * ti - PAD,
                                               M * tj - PAD, g.H, g.W, lane);
        } else {
          const int off = __builtin_amdgcn_readfirstlane(tile_tab[48 + q]);
          return MfmaInput<ALG>::template operand_rect<CS>(in, 16 * cg, off, lane);
        }
      };
      v4i d_cur[NPB], d_nxt[NPB];
      v4i a_nxt = fetch(0);
      mi.sums(a_nxt, d_cur);
      a_nxt = fetch(1);
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        if (q < tr.ntiles) {  // (the same for every wave)
          if (q + 1 < NQ) mi.sums(a_nxt, d_nxt);
          if (q + 2 < NQ) a_nxt = fetch(q + 2);
          __builtin_amdgcn_sched_barrier(0);  // reads and matrix instructions go first
          mi.round(d_cur, g.qmax, packed[q]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int m = 0; m < NPB; ++m) d_cur[m] = d_nxt[m];
        }
      }
    };
    if (tr.whole) run(std::true_type{});
    else run(std::false_type{});
    __syncthreads();  // every patch has been read: the staging area becomes V
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
      // (an empty tile slot keeps stale bytes: they only reach products of that slot, which
      // are never stored)
      if (q < tr.ntiles) {
#pragma unroll
        for (int m = 0; m < NPB; ++m) {
          const int pos = 16 * m + (lane & 15);
          if (pos < PP)
            *(unsigned*)(lds + pos * VS + kc * 1024 + q * 64 + 16 * cg + 4 * (lane >> 4)) = packed[q][m];
        }
      }
    }
  }
  __syncthreads();

  // ---- 3. products + output transform, 4. store ------------------------------------------
  const __amdgpu_buffer_rsrc_t ures = __builtin_amdgcn_make_buffer_rsrc(
      (void*)U16, 0, (int)((unsigned)sp.fgroups * (unsigned)(PP * KC * 1024)), kBufferFlags);
  const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)dq16, 0, (int)((unsigned)sp.fgroups * (unsigned)(PP * 64)), kBufferFlags);
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      y, 0, (int)(esz * (unsigned)(g.N * g.Cout) * (unsigned)(g.H * g.W)), kBufferFlags);
  unsigned char* stage = lds + wave * (4096 * (OUT == 2 ? 1 : 4));
  // groups beyond the last one read zeros (offsets outside the operand) and store nothing
  const int fg = blockIdx.y * NW + wave;
  f4 z[NC][M];
  quad16_products<ALG, KC, PG, VS>(lds, lane, ures, (unsigned)fg * (unsigned)(PP * KC * 1024), dres,
                               (unsigned)fg * (unsigned)(PP * 64), [](int) {}, z);
  __syncthreads();  // the staging blocks take the place of V
  quad16_store<ALG, OUT, EV>(z, stage, tile_tab, lane, fg * 4, x_scale, inv_y, yres, g);
}

// Coefficients of the input transform by processing position, from the add networks: the
// image of every unit patch under fwd_input (rows, then columns) and for_each_point.
template <int ALG>
static void fill_input_table(const float* inv_sx, unsigned char* tab) {
  using Tr = AlgTraits<ALG>;
  constexpr int NI = Tr::NI, NC = Tr::NC;
  constexpr Order<ALG> order{};
  float* inv_pos = reinterpret_cast<float*>(tab);
  signed char* coeff = reinterpret_cast<signed char*>(tab) + kInputTabRows * 4;
  std::memset(tab, 0, kInputTabBytes);
  for (int p = 0; p < Tr::P; ++p) inv_pos[order.pos[p]] = inv_sx[p];
  int* point = reinterpret_cast<int*>(tab + kInputTabPoints);
  for (int j = 0; j < kInputTabRows; ++j) point[j] = j < Order<ALG>::PP ? order.pt[j] : -1;
  for (int i = 0; i < NI; ++i)
    for (int j = 0; j < NI; ++j) {
      int half[NI][NC], comp[NC][NC];
      for (int r = 0; r < NI; ++r) {
        int row[NI] = {};
        if (r == i) row[j] = 1;
        fwd_input<NI, NC>(row, half[r]);
      }
      for (int b = 0; b < NC; ++b) {
        int colv[NI], cc[NC];
        for (int r = 0; r < NI; ++r) colv[r] = half[r][b];
        fwd_input<NI, NC>(colv, cc);
        for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
      }
      for_each_point<ALG>(comp, [&](int p, int v) { coeff[order.pos[p] * 64 + 8 * i + j] = (signed char)v; });
    }
}

// The same for the 8x8 to 10x10 patches of the SFC-6 forms: k = 16 i + j.
template <int ALG>
static void fill_rows_table(const float* inv_sx, unsigned char* tab) {
  using Tr = AlgTraits<ALG>;
  constexpr int NI = Tr::NI, NC = Tr::NC;
  constexpr Order<ALG> order{};
  static_assert(NI <= 12 && Order<ALG>::PP <= kRowsTabRows, "three steps of four rows, table rows");
  std::memset(tab, 0, kRowsTabBytes);
  float* inv_pos = reinterpret_cast<float*>(tab);
  int* point = reinterpret_cast<int*>(tab + kRowsTabPoint);
  signed char* coeff = reinterpret_cast<signed char*>(tab) + kRowsTabCoeff;
  for (int p = 0; p < Tr::P; ++p) inv_pos[order.pos[p]] = inv_sx[p];
  for (int j = 0; j < kRowsTabRows; ++j) point[j] = j < Order<ALG>::PP ? order.pt[j] : -1;
  for (int i = 0; i < NI; ++i)
    for (int j = 0; j < NI; ++j) {
      int half[NI][NC], comp[NC][NC];
      for (int r = 0; r < NI; ++r) {
        int row[NI] = {};
        if (r == i) row[j] = 1;
        fwd_input<NI, NC>(row, half[r]);
      }
      for (int b = 0; b < NC; ++b) {
        int colv[NI], cc[NC];
        for (int r = 0; r < NI; ++r) colv[r] = half[r][b];
        fwd_input<NI, NC>(colv, cc);
        for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
      }
      for_each_point<ALG>(comp, [&](int p, int v) { coeff[order.pos[p] * 192 + 16 * i + j] = (signed char)v; });
    }
}

void build_rows_table(int alg, const float* inv_sx, unsigned char* tab) {
  switch (alg) {
    case 0: fill_rows_table<0>(inv_sx, tab); break;
    case 1: fill_rows_table<1>(inv_sx, tab); break;
    case 2: fill_rows_table<2>(inv_sx, tab); break;
    case 3: fill_rows_table<3>(inv_sx, tab); break;
    case 6: fill_rows_table<6>(inv_sx, tab); break;
    case 7: fill_rows_table<7>(inv_sx, tab); break;
    case 8: fill_rows_table<8>(inv_sx, tab); break;
    case 9: fill_rows_table<9>(inv_sx, tab); break;
    default: std::memset(tab, 0, kRowsTabBytes);
  }
}

void build_input_table(int alg, const float* inv_sx, unsigned char* tab) {
  if (alg == 4) fill_input_table<4>(inv_sx, tab);
  else if (alg == 5) fill_input_table<5>(inv_sx, tab);
  else std::memset(tab, 0, kInputTabBytes);
}

// waves per workgroup: one group of 16 filters each; with two channel chunks eight waves share
// the 16 tiles' V (128 filters), with one chunk four (64 filters), two such workgroups to a
// compute unit
static int single16_waves(const Geometry& g) { return g.Cp > 64 ? 8 : 4; }

static bool make_single16_plan(const Geometry& g, int out, Single16Plan* sp) {
  if ((g.alg != 4 && g.alg != 5) || (g.Cp != 64 && g.Cp != 128)) return false;
  const int kc = g.Cp / 64, nw = single16_waves(g);
  const unsigned pp = (unsigned)((g.P + 3) / 4 * 4);
  const unsigned vbytes = pp * ((unsigned)kc * 1024u + 16u);
  const unsigned sbytes = (unsigned)nw * (out == 2 ? 4096u : 16384u);
  const unsigned lds_max = 160u * 1024u - 256u;
  if (vbytes > lds_max || sbytes > lds_max) return false;
  if (!make_tile_rect(g, (lds_max - 16u) / (unsigned)kc, &sp->tr)) return false;
  sp->chunk_in = tile_rect_stage_bytes(g, sp->tr);
  unsigned top = 16u + sp->chunk_in * (unsigned)kc;
  if (vbytes > top) top = vbytes;
  if (sbytes > top) top = sbytes;
  sp->tab_off = (top + 15u) & ~15u;
  sp->lds_bytes = sp->tab_off + 256u;
  sp->fgroups = (g.Cout + 15) / 16;
  const long long xb = (long long)g.N * g.Cin * g.H * g.W;
  const long long yb = 4ll * g.N * g.Cout * g.H * g.W;
  const long long ub = (long long)sp->fgroups * 16 * pp * g.Cp;
  const long long lim = 1ll << 31;
  return sp->lds_bytes <= 160u * 1024u && xb < lim && yb < lim && ub < lim;
}

bool single16_supported(const Geometry& g) {
  Single16Plan sp;
  return make_single16_plan(g, 0, &sp);
}

template <int ALG, int KC, int OUT, int EV>
static hipError_t launch_single16_impl(const Geometry& g, const Single16Plan& sp, const int8_t* x,
                                       const FilterViews& f, float x_scale, float inv_y, void* y,
                                       hipStream_t s, bool prepare) {
  constexpr int NW = KC == 2 ? 8 : 4;
  auto kernel = single16_kernel<ALG, KC, OUT, EV, NW>;
  if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel));
  const dim3 grid(tile_rect_groups(g, sp.tr), (unsigned)((sp.fgroups + NW - 1) / NW));
  hipLaunchKernelGGL(kernel, grid, dim3(NW * 64), sp.lds_bytes, s, x, (const int8_t*)f.U_single,
                     f.dequant_single, f.input_tab, x_scale, inv_y, y, g, sp);
  return hipGetLastError();
}

template <int ALG, int KC>
static hipError_t launch_single16_kc(int out, const Geometry& g, const Single16Plan& sp,
                                     const int8_t* x, const FilterViews& f, float x_scale,
                                     float inv_y, void* y, hipStream_t s, bool prepare) {
  if (g.W % 4 == 0)
    return out == 2 ? launch_single16_impl<ALG, KC, 2, 4>(g, sp, x, f, x_scale, inv_y, y, s, prepare)
                    : launch_single16_impl<ALG, KC, 0, 4>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
  if (g.W % 2 == 0)
    return out == 2 ? launch_single16_impl<ALG, KC, 2, 2>(g, sp, x, f, x_scale, inv_y, y, s, prepare)
                    : launch_single16_impl<ALG, KC, 0, 2>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
  return out == 2 ? launch_single16_impl<ALG, KC, 2, 1>(g, sp, x, f, x_scale, inv_y, y, s, prepare)
                  : launch_single16_impl<ALG, KC, 0, 1>(g, sp, x, f, x_scale, inv_y, y, s, prepare);
}

hipError_t launch_single16(int out, const Geometry& g, const int8_t* x, const FilterViews& f,
                           float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  Single16Plan sp;
  if (out == 1 || !make_single16_plan(g, out, &sp)) return hipErrorNotSupported;
  if (g.alg == 4)
    return g.Cp == 64 ? launch_single16_kc<4, 1>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare)
                      : launch_single16_kc<4, 2>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare);
  return g.Cp == 64 ? launch_single16_kc<5, 1>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare)
                    : launch_single16_kc<5, 2>(out, g, sp, x, f, x_scale, inv_y, y, s, prepare);
}

}  // namespace sfc
