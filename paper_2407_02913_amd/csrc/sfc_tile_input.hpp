// Input side shared by the kernels that transform input tiles (gfx950): the rectangle
// of tiles a workgroup owns, the staging of its image rows in LDS and the input-tile
// transform V = B^T x B with rounding to int8.
#pragma once
#include <type_traits>

#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"

namespace sfc {

// A workgroup owns S strips x tlw tile columns (a strip = one row of tiles of one
// image), at most 16 tiles, for 64 input channels.
struct TileRect {
  int S;       // strips per workgroup
  int chunks;  // tile-column chunks per strip
  int tlw;     // tile columns per chunk
  int ntiles;  // S * tlw <= 16
  unsigned long long th_magic;  // ceil(2^32 / th): strip / th = (strip * th_magic) >> 32
};

// Staging layout: 64 bytes per image row (byte 4 holds image column colbase, a
// multiple of 4 at or left of the rectangle's first column), M+2 rows per (strip,
// channel), plus one dword so that the channel stride is an odd number of dwords
// and lanes running along channels hit distinct banks.
constexpr int kStageRow = 64;
__host__ __device__ constexpr int stage_channel_bytes(int tile) { return (tile + 2) * kStageRow + 4; }

// Chooses the rectangle that fills most of the 16 tile slots, given the LDS bytes
// available for the staged rows.  False if no rectangle fits.
inline bool make_tile_rect(const Geometry& g, unsigned stage_budget, TileRect* tr) {
  const int M = alg_tile(g.alg);
  const int tlw_max = (kStageRow - 7) / M < 16 ? (kStageRow - 7) / M : 16;  // 5 + M*tlw + 2 <= 64
  const int min_chunks = (g.tw + tlw_max - 1) / tlw_max;
  const int s_fit = (int)(stage_budget / (64u * (unsigned)stage_channel_bytes(M)));
  if (s_fit < 1) return false;
  double best = -1.0;
  for (int chunks = min_chunks; chunks <= min_chunks + 4 && chunks <= g.tw; ++chunks) {
    const int tlw = (g.tw + chunks - 1) / chunks;
    int S = 16 / tlw;
    if (S > g.strips) S = g.strips;
    if (S > s_fit) S = s_fit;
    const int groups = (g.strips + S - 1) / S;
    // fraction of the 16 tile slots of all workgroups that hold a real tile
    const double use = (double)g.T / ((double)groups * chunks * 16.0);
    if (use > best + 1e-9) {
      best = use;
      tr->chunks = chunks;
      tr->tlw = tlw;
      tr->S = S;
    }
  }
  tr->ntiles = tr->S * tr->tlw;
  // the reciprocal is exact while strip * th < 2^32
  if ((long long)g.strips * g.th >= (1ll << 32) || g.th < 1) return false;
  tr->th_magic = ((1ull << 32) + (unsigned long long)g.th - 1) / (unsigned long long)g.th;
  return tr->ntiles >= 1 && tr->ntiles <= 16 && 5 + M * tr->tlw + 2 <= kStageRow;
}

inline unsigned tile_rect_stage_bytes(const Geometry& g, const TileRect& tr) {
  return (unsigned)tr.S * 64u * (unsigned)stage_channel_bytes(alg_tile(g.alg));
}
inline unsigned tile_rect_groups(const Geometry& g, const TileRect& tr) {
  return (unsigned)(((g.strips + tr.S - 1) / tr.S) * tr.chunks);
}

#ifdef __HIPCC__

__device__ __forceinline__ int strip_image(const TileRect& tr, int strip) {
  return (int)(((unsigned long long)(unsigned)strip * tr.th_magic) >> 32);
}

// Stage the M+2 input rows of every (strip, channel) of the rectangle, channels
// c0 .. c0+63, zero outside the image.  One instruction covers four rows x 16 dwords
// of one (strip, channel): lane = (row within the group, dword).  A wave walks over
// (strip, row group) combinations; within one, only the channel plane changes from
// load to load (wave w takes channels w, w+NW, ...), so the lane address and its
// validity are computed once per combination.  Lanes without data (padding halo, dead
// strips) get an offset beyond the buffer, for which a buffer load returns zero
// without touching memory; a dword that straddles the end of an image row keeps its
// valid bytes only.  Global dwords need not be aligned.  All loads of a batch are in
// flight before the first LDS write.  Channels beyond Cin re-read the last one (their
// filter operand is zero).
template <int ALG, int NW>
__device__ __forceinline__ void stage_tiles(const int8_t* __restrict__ x, unsigned char* lds,
                                            const Geometry& g, const TileRect& tr, int strip0,
                                            int tj0, int c0, int wave, int lane) {
  constexpr int M = AlgTraits<ALG>::M, NI = AlgTraits<ALG>::NI;
  constexpr int ROWG = (NI + 3) / 4;  // groups of four staged rows
  constexpr int WP = kStageRow, CS = stage_channel_bytes(M);
  constexpr unsigned kOutOfRange = 0x80000000u;
  const int W = g.W, H = g.H;
  const unsigned xbytes = (unsigned)(g.N * g.Cin) * (unsigned)(H * W);
  const __amdgpu_buffer_rsrc_t xres =
      __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)xbytes, kBufferFlags);
  const int colbase = (M * tj0) & ~3;
  const int rsub = lane >> 4, dcol = lane & 15;
  const int col = colbase + 4 * dcol - 4;  // image column of the first byte of this lane's dword
  const int nvalid = col < 0 ? 0 : min(4, max(0, W - col));  // bytes of it inside the row
  const unsigned bmask = nvalid >= 4 ? 0xffffffffu : ((1u << (8 * nvalid)) - 1u);
  const int lane_off = rsub * W + col;  // lane part of the byte offset
  const unsigned plane_stride = (unsigned)(H * W);
  constexpr int CPW = 64 / NW;  // channels per wave
  constexpr int CB = 6;         // combinations per batch
  const int ncombo = tr.S * ROWG;
  // A dword can reach past the end of the tensor only if rows are not whole dwords; the
  // buffer load then returns zero for all of it, so those bytes are fetched one by one.
  // Rows of whole dwords take the loop without that check.
  auto run = [&](auto tail_check) {
    constexpr bool kTail = decltype(tail_check)::value;
    for (int k0 = 0; k0 < ncombo; k0 += CB) {
      unsigned vals[CB][CPW];
#pragma unroll
      for (int kk = 0; kk < CB; ++kk) {
        const int k = k0 + kk;
        const int s = k / ROWG, rg = k - s * ROWG;
        const int strip = strip0 + s;
        const bool live = k < ncombo && strip < g.strips;
        const int n = strip_image(tr, strip);
        const int ti = strip - n * g.th;
        const int hlo = M * ti - 1 + 4 * rg;        // image row of rsub = 0
        const int base = (n * g.Cin * H + hlo) * W;  // its offset in channel 0 of image n
        const bool ok = live && nvalid > 0 && 4 * rg + rsub < NI &&
                        (unsigned)(hlo + rsub) < (unsigned)H;
        const unsigned voff = ok ? (unsigned)(base + lane_off) : kOutOfRange;
#pragma unroll
        for (int ci = 0; ci < CPW; ++ci) {
          const int c = min(c0 + wave + NW * ci, g.Cin - 1);
          const unsigned plane = (unsigned)c * plane_stride;
          unsigned v = __builtin_amdgcn_raw_buffer_load_b32(xres, voff, plane, 0);
          if constexpr (kTail) {
            v &= bmask;
            if (n == g.N - 1 && c == g.Cin - 1) {
              if (ok && voff + plane + 4u > xbytes) {
                v = 0;
                for (int bb = 0; bb < nvalid; ++bb)
                  v |= (unsigned)__builtin_amdgcn_raw_buffer_load_b8(xres, voff + bb, plane, 0)
                       << (8 * bb);
              }
            }
          }
          vals[kk][ci] = v;
        }
      }
#pragma unroll
      for (int kk = 0; kk < CB; ++kk) {
        const int k = k0 + kk;
        const int s = k / ROWG, rg = k - s * ROWG;
        const int row = rg * 4 + rsub;
        if (k < ncombo && row < NI) {
          unsigned char* dst = lds + (unsigned)(s * 64 + wave) * CS + row * WP + 4 * dcol;
#pragma unroll
          for (int ci = 0; ci < CPW; ++ci) *(unsigned*)(dst + NW * ci * CS) = vals[kk][ci];
        }
      }
    }
  };
  if ((W & 3) == 0)
    run(std::false_type{});  // every dword lies wholly inside or outside its row
  else
    run(std::true_type{});
}

// Input-tile transform of the staged rectangle: wave = tile (16/NW of them per wave),
// lane = channel.  Lanes running along channels are an odd number of dwords apart in
// the staging area, so the aligned dword reads of a patch row hit 64 different banks.
// Each thread applies the symbolic DFT-6 add network along rows and columns, forms
// the multiplication points and rounds them to int8; the bytes go to
// lds[order.pos[p]*1024 + tile*64 + channel], over the staging area (every patch is in
// registers by then).  Call between two workgroup barriers; contains one itself.
template <int ALG, int NW>
__device__ __forceinline__ void transform_tiles(unsigned char* lds, const float* __restrict__ inv_sx,
                                                float qmax, const TileRect& tr, int tj0, int wave,
                                                int lane) {
  using Tr = AlgTraits<ALG>;
  constexpr int M = Tr::M, NI = Tr::NI, NC = Tr::NC;
  constexpr int SPW = 16 / NW;
  constexpr int WP = kStageRow, CS = stage_channel_bytes(M);
  constexpr Order<ALG> order{};
  const int colbase = (M * tj0) & ~3;
  const int halo = M * tj0 - 1 - colbase + 4;  // LDS byte of the rectangle's first patch column
  int half[SPW][NI][NC];  // rows transformed: half[.][i][b]
#pragma unroll
  for (int it = 0; it < SPW; ++it) {
    const int tile = wave + NW * it, c = lane;
    if (tile < tr.ntiles) {
      const int s = tile / tr.tlw, tjl = tile - s * tr.tlw;
      // the patch row starts at an odd byte: three aligned dwords, shifted into place
      const int o = halo + M * tjl;
      const unsigned* src = (const unsigned*)(lds + (unsigned)(s * 64 + c) * CS + (o & ~3));
      const unsigned sh = (unsigned)(o & 3);
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const unsigned d0 = src[i * (WP / 4)], d1 = src[i * (WP / 4) + 1], d2 = src[i * (WP / 4) + 2];
        const unsigned w[3] = {__builtin_amdgcn_alignbyte(d1, d0, sh),
                               __builtin_amdgcn_alignbyte(d2, d1, sh), d2 >> (8 * sh)};
        int row[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) row[j] = (int)(signed char)(w[j / 4] >> (8 * (j % 4)));
        fwd_input<NI, NC>(row, half[it][i]);
      }
    }
  }
  __syncthreads();  // every patch is in registers: the staging area becomes V
#pragma unroll
  for (int it = 0; it < SPW; ++it) {
    const int tile = wave + NW * it, c = lane;
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
      unsigned char* outp = lds + tile * 64 + c;
      for_each_point<ALG>(comp, [&](int p, int v) {
        outp[order.pos[p] * 1024] = (unsigned char)quantize_byte(v, inv_sx[p], qmax);
      });
    }
  }
}

// Copies the rounded points of the rectangle from LDS ([position][tile][channel]) to
// V: wave w takes positions w, w+NW, ...; lane = (tile, 16-byte quarter of its 64
// channels); lane_off is the lane's byte offset inside a point's plane of V.
template <int ALG, int NW>
__device__ __forceinline__ void copy_out_points(const unsigned char* lds,
                                                __amdgpu_buffer_rsrc_t vres, unsigned lane_off,
                                                unsigned vplane, int wave, int lane) {
  constexpr int P = AlgTraits<ALG>::P;
  constexpr Order<ALG> order{};
#pragma unroll
  for (int jj = 0; jj < (P + NW - 1) / NW; ++jj) {
    // the position is one of NW compile-time values chosen by the uniform wave index,
    // so the canonical point index, and with it the plane offset, stays scalar
    int p = -1;
#pragma unroll
    for (int w = 0; w < NW; ++w)
      if (w == wave && jj * NW + w < P) p = order.pt[jj * NW + w];
    if (p >= 0) {
      const v4i d = *(const v4i*)(lds + (jj * NW + wave) * 1024 + lane * 16);
      __builtin_amdgcn_raw_buffer_store_b128(d, vres, lane_off, (unsigned)p * vplane, 0);
    }
  }
}

#endif  // __HIPCC__

}  // namespace sfc
