// Input side shared by the kernels that transform input tiles (gfx950): the rectangle
// of tiles a workgroup owns, the staging of its image rows in LDS and the input-tile
// transform V = B^T x B with rounding to int8.
#pragma once
#include <type_traits>

#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"

namespace sfc {

// A workgroup owns at most 16 tiles for 64 input channels, in one of two shapes:
//  - a rectangle of S strips x tlw tile columns (a strip = one row of tiles of one image);
//  - whole images (small feature maps: at most 16 tiles per image): ipw images, staged as
//    plain copies of their 64 channel planes.
struct TileRect {
  int S;       // strips per workgroup
  int chunks;  // tile-column chunks per strip
  int tlw;     // tile columns per chunk
  int ntiles;  // S * tlw, or ipw * tiles per image; <= 16
  unsigned long long th_magic;  // ceil(2^32 / th): strip / th = (strip * th_magic) >> 32
  int whole;   // 1: whole images
  int ipw;     // images per workgroup
  int cs;      // whole images: LDS bytes per channel plane (an odd number of dwords)
};

// Staging layout: 64 bytes per image row (byte 4 holds image column colbase, a
// multiple of 4 at or left of the rectangle's first column), NI = M+R-1 rows per (strip,
// channel), plus one dword so that the channel stride is an odd number of dwords
// and lanes running along channels hit distinct banks.
constexpr int kStageRow = 64;
__host__ __device__ constexpr int stage_channel_bytes(int rows) { return rows * kStageRow + 4; }
// input rows per tile and zero padding of an algorithm
__host__ __device__ constexpr int alg_rows(int alg) { return alg_tile(alg) + alg_taps(alg) - 1; }
__host__ __device__ constexpr int alg_pad(int alg) { return (alg_taps(alg) - 1) / 2; }

// Chooses the rectangle that fills most of the 16 tile slots, given the LDS bytes
// available for the staged rows.  False if no rectangle fits.
// LDS bytes per channel plane of a whole image: H*W rounded up to dwords, plus one dword
// if that makes the stride between channels (= lanes of the transform) an odd number of
// dwords, so that the byte reads of 64 channels hit different banks.
__host__ __device__ constexpr int plane_stride_bytes(int hw) {
  const int d = (hw + 3) / 4;
  return 4 * (d % 2 == 0 ? d + 1 : d);
}

// max_tiles: tile slots of a workgroup (16, or 8 for workgroups of eight one-tile waves).
// partial_images: take whole images even if they leave tile slots empty, when the
// alternative is a rectangle whose rows are not whole dwords (byte-wise staging).
// whole_images: false keeps to rectangles whatever the size of the feature map.
inline bool make_tile_rect(const Geometry& g, unsigned stage_budget, TileRect* tr,
                           int max_tiles = 16, bool partial_images = false, bool whole_images = true) {
  const int M = alg_tile(g.alg), PAD = alg_pad(g.alg);
  tr->whole = 0;
  tr->ipw = 0;
  tr->cs = 0;
  // Small feature maps: whole images, if the tile slots are used at least as well as a
  // rectangle would (always the case when the tiles of an image divide 16).
  const int tpi = g.th * g.tw;
  if (whole_images && tpi <= max_tiles && g.H * g.W <= 1024) {
    const int cs = plane_stride_bytes(g.H * g.W);
    int ipw = max_tiles / tpi;
    if (ipw > g.N) ipw = g.N;
    while (ipw > 1 && (unsigned)(ipw * 64 * cs) > stage_budget) --ipw;
    if ((unsigned)(ipw * 64 * cs) <= stage_budget &&
        (max_tiles % tpi == 0 || (partial_images && g.W % 4 != 0))) {
      tr->whole = 1;
      tr->ipw = ipw;
      tr->cs = cs;
      tr->S = tr->chunks = tr->tlw = 1;
      tr->ntiles = ipw * tpi;
      tr->th_magic = 0;
      return true;
    }
  }
  // the first patch column lies at LDS byte 7-PAD at most, the last one M*tlw + 2*PAD - 1 further
  const int tlw_max = (kStageRow - 7 - PAD) / M < max_tiles ? (kStageRow - 7 - PAD) / M : max_tiles;
  const int min_chunks = (g.tw + tlw_max - 1) / tlw_max;
  const int s_fit = (int)(stage_budget / (64u * (unsigned)stage_channel_bytes(alg_rows(g.alg))));
  if (s_fit < 1) return false;
  double best = -1.0;
  for (int chunks = min_chunks; chunks <= min_chunks + 4 && chunks <= g.tw; ++chunks) {
    const int tlw = (g.tw + chunks - 1) / chunks;
    int S = max_tiles / tlw;
    if (S > g.strips) S = g.strips;
    if (S > s_fit) S = s_fit;
    const int groups = (g.strips + S - 1) / S;
    // fraction of the tile slots of all workgroups that hold a real tile
    const double use = (double)g.T / ((double)groups * chunks * (double)max_tiles);
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
  return tr->ntiles >= 1 && tr->ntiles <= max_tiles && M * tr->tlw <= kStageRow - 7 - PAD;
}

inline unsigned tile_rect_stage_bytes(const Geometry& g, const TileRect& tr) {
  if (tr.whole) return (unsigned)(tr.ipw * 64 * tr.cs);
  return (unsigned)tr.S * 64u * (unsigned)stage_channel_bytes(alg_rows(g.alg));
}
inline unsigned tile_rect_groups(const Geometry& g, const TileRect& tr) {
  if (tr.whole) return (unsigned)((g.N + tr.ipw - 1) / tr.ipw);
  return (unsigned)(((g.strips + tr.S - 1) / tr.S) * tr.chunks);
}

#ifdef __HIPCC__

__device__ __forceinline__ int strip_image(const TileRect& tr, int strip) {
  return (int)(((unsigned long long)(unsigned)strip * tr.th_magic) >> 32);
}

// Tile slot tl of workgroup bx: image, tile row, tile column, and whether the slot holds
// a tile at all.
struct TileCoord {
  int n, ti, tj;
  bool live;
};
__device__ __forceinline__ TileCoord tile_coord(const Geometry& g, const TileRect& tr, int bx,
                                                int tl) {
  TileCoord tc;
  if (tr.whole) {
    const int tpi = g.th * g.tw;
    const int img = tl / tpi, rem = tl - img * tpi;
    tc.n = bx * tr.ipw + img;
    tc.ti = rem / g.tw;
    tc.tj = rem - tc.ti * g.tw;
    tc.live = tl < tr.ntiles && tc.n < g.N;
  } else {
    const int chunk = bx % tr.chunks;
    const int s = tl / tr.tlw, tjl = tl - s * tr.tlw;
    const int strip = (bx / tr.chunks) * tr.S + s;
    tc.tj = chunk * tr.tlw + tjl;
    tc.n = strip_image(tr, strip);
    tc.ti = strip - tc.n * g.th;
    tc.live = tl < tr.ntiles && strip < g.strips && tc.tj < g.tw;
  }
  return tc;
}

// Whole-image staging: the 64 channel planes c0 .. c0+63 of the workgroup's ipw images,
// each copied as it lies in memory (H*W contiguous bytes) to lds[(slot*64 + c)*cs ..].
// One load instruction covers CPI planes with LPC lanes each (LPC = dwords of a plane
// rounded up to a power of two), or a 64-dword piece of one plane when a plane has more
// than 64 dwords; wave w takes instructions w, w+NW, ...  Planes need not be dword
// aligned in memory.  A plane's last dword may carry bytes of the next plane (they land
// in the padding of its LDS slot and are never read); only at the very end of the tensor
// would it reach past the buffer, so there the bytes are fetched one by one.  Images
// beyond N read nothing (zeros).  Channels beyond Cin re-read the last one (their filter
// operand is zero).
template <int NW, int BATCH = 8>
__device__ __forceinline__ void stage_images(const int8_t* __restrict__ x, unsigned char* lds,
                                             const Geometry& g, const TileRect& tr, int bx, int c0,
                                             int wave, int lane) {
  const int HW = g.H * g.W;
  const unsigned xbytes = (unsigned)(g.N * g.Cin) * (unsigned)HW;
  const __amdgpu_buffer_rsrc_t xres =
      __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)xbytes, kBufferFlags);
  const int dpc = (HW + 3) >> 2;  // dwords per plane
  int lpc = 1;
  while (lpc < dpc && lpc < 64) lpc <<= 1;
  const int cpi = 64 / lpc;               // planes per instruction
  const int ipp = (dpc + 63) >> 6;        // instructions per plane (1 unless dpc > 64)
  const int per_image = (64 / cpi) * ipp; // instructions per image
  const int total = tr.ipw * per_image;
  const int sub = lane / lpc, dw_lane = lane - sub * lpc;
  // BATCH: loads in flight per wave before the first LDS write
  for (int k0 = wave; k0 < total; k0 += NW * BATCH) {
    unsigned vals[BATCH];
    int dst[BATCH];
#pragma unroll
    for (int kk = 0; kk < BATCH; ++kk) {
      const int k = k0 + NW * kk;
      const int slot = k / per_image, rem = k - slot * per_image;
      const int cg = rem / ipp, piece = rem - cg * ipp;
      const int c = cg * cpi + sub;  // channel of this lane within the 64
      const int dw = piece * 64 + dw_lane;
      const int n = bx * tr.ipw + slot;
      const bool ok = k < total && n < g.N && dw < dpc;
      const int cc = min(c0 + c, g.Cin - 1);
      const unsigned off = (unsigned)((n * g.Cin + cc) * HW + 4 * dw);
      unsigned v = 0;
      if (ok) {
        if (off + 4u <= xbytes) {
          v = __builtin_amdgcn_raw_buffer_load_b32(xres, off, 0, 0);
        } else {
          for (unsigned bb = 0; off + bb < xbytes; ++bb)
            v |= (unsigned)__builtin_amdgcn_raw_buffer_load_b8(xres, off + bb, 0, 0) << (8 * bb);
        }
      }
      vals[kk] = v;
      dst[kk] = ok ? (slot * 64 + c) * tr.cs + 4 * dw : -1;
    }
#pragma unroll
    for (int kk = 0; kk < BATCH; ++kk)
      if (dst[kk] >= 0) *(unsigned*)(lds + dst[kk]) = vals[kk];
  }
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
  constexpr int M = AlgTraits<ALG>::M, NI = AlgTraits<ALG>::NI, PAD = AlgTraits<ALG>::PAD;
  constexpr int ROWG = (NI + 3) / 4;  // groups of four staged rows
  constexpr int WP = kStageRow, CS = stage_channel_bytes(NI);
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
  const int ncombo = tr.S * ROWG;
  // A dword can reach past the end of the tensor only if rows are not whole dwords; the
  // buffer load then returns zero for all of it, so those bytes are fetched one by one.
  // Rows of whole dwords take the loop without that check.
  // CB: combinations per batch (every load of a batch is issued, live or not)
  auto run = [&](auto tail_check, auto batch) {
    constexpr bool kTail = decltype(tail_check)::value;
    constexpr int CB = decltype(batch)::value;
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
        const int hlo = M * ti - PAD + 4 * rg;      // image row of rsub = 0
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
  if ((W & 3) == 0) {  // every dword lies wholly inside or outside its row
    if (ncombo <= ROWG) run(std::false_type{}, std::integral_constant<int, ROWG>{});
    else if (ncombo <= 2 * ROWG) run(std::false_type{}, std::integral_constant<int, 2 * ROWG>{});
    else run(std::false_type{}, std::integral_constant<int, 6>{});
  } else {
    run(std::true_type{}, std::integral_constant<int, 6>{});
  }
}

// Stage the input of workgroup bx in the shape its TileRect says.
template <int ALG, int NW>
__device__ __forceinline__ void stage_input(const int8_t* __restrict__ x, unsigned char* lds,
                                            const Geometry& g, const TileRect& tr, int bx, int c0,
                                            int wave, int lane) {
  if (tr.whole) {
    stage_images<NW>(x, lds, g, tr, bx, c0, wave, lane);
  } else {
    const int chunk = bx % tr.chunks;
    stage_tiles<ALG, NW>(x, lds, g, tr, (bx / tr.chunks) * tr.S, chunk * tr.tlw, c0, wave, lane);
  }
}

// Input-tile transform of the staged tiles: wave = tile (16/NW of them per wave),
// lane = channel.  Lanes running along channels are an odd number of dwords apart in
// the staging area, so the reads of a patch row (aligned dwords of a rectangle, bytes
// of a whole image) hit 64 different banks.
// Each thread applies the symbolic DFT-6 add network along rows and columns, forms
// the multiplication points and rounds them to int8; the bytes go to
// lds[order.pos[p]*VS + tile*64 + channel], over the staging area (every patch is in
// registers by then); VS = 1024 (16 tile slots per point), or 512 for workgroups of
// eight tiles.  Call between two workgroup barriers; contains one itself.
template <int ALG, int NW, int SPW = 16 / NW, int VS = 1024>
__device__ __forceinline__ void transform_tiles(unsigned char* lds, const float* __restrict__ inv_sx,
                                                float qmax, const Geometry& g, const TileRect& tr,
                                                int bx, int wave, int lane) {
  using Tr = AlgTraits<ALG>;
  constexpr int M = Tr::M, NI = Tr::NI, NC = Tr::NC, PAD = Tr::PAD;
  constexpr int WP = kStageRow, CS = stage_channel_bytes(NI);
  constexpr int ND = (NI + 6) / 4;  // aligned dwords that hold a patch row at any byte offset
  constexpr Order<ALG> order{};
  const int tj0 = tr.whole ? 0 : (bx % tr.chunks) * tr.tlw;
  const int colbase = (M * tj0) & ~3;
  const int halo = M * tj0 - PAD - colbase + 4;  // LDS byte of the rectangle's first patch column
  int half[SPW][NI][NC];  // rows transformed: half[.][i][b]
#pragma unroll
  for (int it = 0; it < SPW; ++it) {
    const int tile = wave + NW * it, c = lane;
    if (tile < tr.ntiles) {
      if (tr.whole) {
        // whole images: sign-extending byte reads of the plane, zeros outside the image
        // (tile position and with it every bound is uniform over the wave)
        const int tpi = g.th * g.tw;
        const int slot = tile / tpi, rem = tile - slot * tpi;
        const int ti = rem / g.tw, tj = rem - ti * g.tw;
        const signed char* plane = (const signed char*)lds + (slot * 64 + c) * tr.cs;
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
        // the patch row starts at any byte: ND aligned dwords, shifted into place (the last
        // one may lie beyond the row's 64 bytes when the row does not need it: still inside
        // the channel's staging block, never used)
        const int o = halo + M * tjl;
        const unsigned* src = (const unsigned*)(lds + (unsigned)(s * 64 + c) * CS + (o & ~3));
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
        outp[order.pos[p] * VS] = (unsigned char)quantize_byte(v, inv_sx[p], qmax);
      });
    }
  }
}

// Copies the rounded points of the rectangle from LDS ([position][tile][channel]) to
// V: wave w takes positions w, w+NW, ...; lane = (tile, 16-byte quarter of its 64
// channels); lane_off is the lane's byte offset inside a point's plane of V.
// VS = 512 (eight tiles per workgroup): a wave takes two positions at a time, lanes 0..31
// the first, lanes 32..63 the second.
// VSP: LDS bytes from one position to the next (VS, or more when the points are padded).
template <int ALG, int NW, int VS = 1024, int VSP = VS>
__device__ __forceinline__ void copy_out_points(const unsigned char* lds,
                                                __amdgpu_buffer_rsrc_t vres, unsigned lane_off,
                                                unsigned vplane, int wave, int lane) {
  constexpr int P = AlgTraits<ALG>::P;
  constexpr Order<ALG> order{};
  if constexpr (VS == 512) {
    const int hi = lane >> 5;  // which of the wave's two positions
#pragma unroll
    for (int jj = 0; jj < (P + 2 * NW - 1) / (2 * NW); ++jj) {
      // positions 2*(jj*NW + wave) and the next one: compile-time candidates selected by
      // the uniform wave index and the half of the wave
      int p = -1;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const int j0 = 2 * (jj * NW + w);
        if (w == wave) {
          const int pa = j0 < P ? order.pt[j0 < P ? j0 : 0] : -1;
          const int pb = j0 + 1 < P ? order.pt[j0 + 1 < P ? j0 + 1 : 0] : -1;
          p = hi ? pb : pa;
        }
      }
      if (p >= 0) {
        const v4i d = *(const v4i*)(lds + (2 * (jj * NW + wave) + hi) * VSP + (lane & 31) * 16);
        __builtin_amdgcn_raw_buffer_store_b128(d, vres, lane_off + (unsigned)p * vplane, 0, 0);
      }
    }
    return;
  }
#pragma unroll
  for (int jj = 0; jj < (P + NW - 1) / NW; ++jj) {
    // the position is one of NW compile-time values chosen by the uniform wave index,
    // so the canonical point index, and with it the plane offset, stays scalar
    int p = -1;
#pragma unroll
    for (int w = 0; w < NW; ++w)
      if (w == wave && jj * NW + w < P) p = order.pt[jj * NW + w];
    if (p >= 0) {
      const v4i d = *(const v4i*)(lds + (jj * NW + wave) * VSP + lane * 16);
      __builtin_amdgcn_raw_buffer_store_b128(d, vres, lane_off, (unsigned)p * vplane, 0);
    }
  }
}

#endif  // __HIPCC__

}  // namespace sfc
