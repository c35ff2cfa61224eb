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
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
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
    const float* __restrict__ inv_sx, float x_scale, float inv_y, void* __restrict__ y, Geometry g,
    Single16Plan sp) {
  using Tr = AlgTraits<ALG>;
  constexpr int M = Tr::M, NI = Tr::NI, NC = Tr::NC, PAD = Tr::PAD;
  constexpr int PP = Order<ALG>::PP, PG = PP / 4;
  constexpr int SPW = 16 / NW, NITEM = SPW * KC;
  constexpr int WP = kStageRow, CS = stage_channel_bytes(NI);
  constexpr int ND = (NI + 6) / 4;
  constexpr int VS = KC * 1024;  // bytes of V per position
  constexpr Order<ALG> order{};
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
  }

  // ---- 1. stage ----------------------------------------------------------------------
#pragma unroll
  for (int kc = 0; kc < KC; ++kc)
    stage_input<ALG, NW>(x, lds + kc * sp.chunk_in, g, tr, bx, 64 * kc, wave, lane);
  __syncthreads();

  // ---- 2. input transform --------------------------------------------------------------
  {
    const int tj0 = tr.whole ? 0 : (bx % tr.chunks) * tr.tlw;
    const int colbase = (M * tj0) & ~3;
    const int halo = M * tj0 - PAD - colbase + 4;  // LDS byte of the rectangle's first patch column
    int half[NITEM][NI][NC];  // rows transformed: half[.][i][b]
#pragma unroll
    for (int it = 0; it < NITEM; ++it) {
      const int tile = wave + NW * (it / KC), kc = it % KC, c = lane;
      const unsigned char* in = lds + kc * sp.chunk_in;
      if (tile < tr.ntiles) {
        if (tr.whole) {
          // whole images: sign-extending byte reads of the plane, zeros outside the image
          const int tpi = g.th * g.tw;
          const int slot = tile / tpi, rem = tile - slot * tpi;
          const int ti = rem / g.tw, tj = rem - ti * g.tw;
          const signed char* plane = (const signed char*)in + (slot * 64 + c) * tr.cs;
          const int r0 = M * ti - PAD, q0 = M * tj - PAD;
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            int row[NI];
            const bool rok = (unsigned)(r0 + i) < (unsigned)g.H;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
              row[j] = 0;
              if (rok && (unsigned)(q0 + j) < (unsigned)g.W) row[j] = plane[(r0 + i) * g.W + q0 + j];
            }
            fwd_input<NI, NC>(row, half[it][i]);
          }
        } else {
          const int s = tile / tr.tlw, tjl = tile - s * tr.tlw;
          const int o = halo + M * tjl;
          const unsigned* src = (const unsigned*)(in + (unsigned)(s * 64 + c) * CS + (o & ~3));
          const unsigned sh = (unsigned)(o & 3);
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            unsigned d[ND], w[ND];
#pragma unroll
            for (int k = 0; k < ND; ++k) d[k] = src[i * (WP / 4) + k];
#pragma unroll
            for (int k = 0; k + 1 < ND; ++k) w[k] = __builtin_amdgcn_alignbyte(d[k + 1], d[k], sh);
            w[ND - 1] = d[ND - 1] >> (8 * sh);
            int row[NI];
#pragma unroll
            for (int j = 0; j < NI; ++j) row[j] = (int)(signed char)(w[j / 4] >> (8 * (j % 4)));
            fwd_input<NI, NC>(row, half[it][i]);
          }
        }
      }
    }
    __syncthreads();  // every patch is in registers: the staging area becomes V
#pragma unroll
    for (int it = 0; it < NITEM; ++it) {
      const int tile = wave + NW * (it / KC), kc = it % KC, c = lane;
      unsigned char* outp = lds + kc * 1024 + tile * 64 + c;
      if (tile < tr.ntiles) {
        int comp[NC][NC];
#pragma unroll
        for (int b = 0; b < NC; ++b) {
          int colv[NI], cc[NC];
#pragma unroll
          for (int i = 0; i < NI; ++i) colv[i] = half[it][i][b];
          fwd_input<NI, NC>(colv, cc);
#pragma unroll
          for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
        }
        for_each_point<ALG>(comp, [&](int p, int v) {
          outp[order.pos[p] * VS] = (unsigned char)quantize_byte(v, inv_sx[p], g.qmax);
        });
      }
      // (an empty tile slot keeps stale bytes: they only reach products of that slot, which
      // are never stored)
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
  quad16_products<ALG, KC, PG>(lds, lane, ures, (unsigned)fg * (unsigned)(PP * KC * 1024), dres,
                               (unsigned)fg * (unsigned)(PP * 64), [](int) {}, z);
  __syncthreads();  // the staging blocks take the place of V
  quad16_store<ALG, OUT, EV>(z, stage, tile_tab, lane, fg * 4, x_scale, inv_y, yres, g);
}

// waves per workgroup: one group of 16 filters each; with two channel chunks eight waves share
// the 16 tiles' V (128 filters), with one chunk four (64 filters), two such workgroups to a
// compute unit
static int single16_waves(const Geometry& g) { return g.Cp > 64 ? 8 : 4; }

static bool make_single16_plan(const Geometry& g, int out, Single16Plan* sp) {
  if ((g.alg != 4 && g.alg != 5) || (g.Cp != 64 && g.Cp != 128)) return false;
  const int kc = g.Cp / 64, nw = single16_waves(g);
  const unsigned pp = (unsigned)((g.P + 3) / 4 * 4);
  const unsigned vbytes = pp * (unsigned)kc * 1024u;
  const unsigned sbytes = (unsigned)nw * (out == 2 ? 4096u : 16384u);
  const unsigned lds_max = 160u * 1024u - 256u;
  if (vbytes > lds_max || sbytes > lds_max) return false;
  if (!make_tile_rect(g, lds_max / (unsigned)kc, &sp->tr)) return false;
  sp->chunk_in = tile_rect_stage_bytes(g, sp->tr);
  unsigned top = sp->chunk_in * (unsigned)kc;
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
                     f.dequant_single, f.inv_sx, x_scale, inv_y, y, g, sp);
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
