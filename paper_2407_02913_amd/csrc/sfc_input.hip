// Input-tile transform V = B^T x B with transform-domain requantization to int8,
// the HBM-facing first stage of the two-kernel paths (gfx950), every algorithm, on the
// matrix cores (sfc_mfma_input.hpp; small feature maps: sfc_input_image.hip).
//
// A workgroup owns up to NW tiles (a rectangle of S strips x tlw tile columns, or whole
// images of a small feature map), one per wave, and 64 input channels:
//  1. stage the input rows of every (strip, channel) in LDS (coalesced dword loads),
//  2. transform: wave = tile, four groups of 16 channels, lane = (position, four channels);
//  3. SFC-4 forms: the rounded points land in LDS as [processing position][tile][channel],
//     over the staging area, and are copied out with 16-byte lanes, 64 contiguous bytes per
//     (point, tile) and NW tiles in a row; SFC-6 forms: every wave turns blocks of 16
//     positions round in LDS of its own and stores them directly.
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_mfma_input.hpp"
#include "sfc_points.hpp"
#include "sfc_tile_input.hpp"

namespace sfc {

constexpr int kWaveRowBytes = 80;  // LDS bytes per position in a wave's block (conflict-free dword writes)

struct InputPlan {
  TileRect tr;
  unsigned tab_off;  // LDS byte offset of the tile -> V row table
  unsigned lds_bytes;
};

// VS: bytes of V per point in LDS, 64 per tile slot (512 for the 8-tile workgroups: half the
// LDS, so that more workgroups share a compute unit and overlap their phases).
// TPW: tiles per wave (SFC-4 forms: 2 when the workgroup takes whole images of 9 to 16 tiles,
// whose planes it copies as they lie in memory instead of staging sparse 64-byte row windows).
template <int ALG, int NW, int VS, int TPW = 1>
__global__ __launch_bounds__(NW * 64) void input_transform_i8_kernel(
    const int8_t* __restrict__ x, int8_t* __restrict__ V, const float* __restrict__ inv_sx,
    const unsigned char* __restrict__ intab, Geometry g, InputPlan ip) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int P = AlgTraits<ALG>::P;
  // LDS bytes from one position's V to the next: the SFC-4 forms write 16 positions per
  // instruction (sfc_mfma_input.hpp) and need them in different banks
  constexpr bool kRows16 = AlgTraits<ALG>::kFamily == 6;  // 8x8 to 10x10 patches on the matrix cores, below
  constexpr int VSP = AlgTraits<ALG>::kFamily == 4 ? VS + 16 : VS;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const TileRect& tr = ip.tr;
  // Workgroups are dealt to the 8 XCDs round-robin by id; remap so that each XCD (each
  // L2) gets a contiguous range of rectangles: neighbours share halo rows and columns.
  // Position = (tile group, 64-channel group), the channel group varying fastest: the
  // workgroups that write the two 64-byte halves of a line of V (Cp = 128) run next to
  // each other on one XCD.
  const int cgn = g.Cp >> 6;
  const int pos = xcd_contiguous(blockIdx.x, gridDim.x);
  const int bx = pos / cgn;
  const int c0 = (pos - bx * cgn) * 64;

  // tile slot -> row of V (-1: no such tile)
  int* row_tab = (int*)(lds + ip.tab_off);
  if (threadIdx.x < 16) {
    const int tl = threadIdx.x;
    const TileCoord tc = tile_coord(g, tr, bx, tl);
    row_tab[tl] = tc.live ? (tc.n * g.th + tc.ti) * g.tw + tc.tj : -1;
  }

  // (the SFC-4 forms stage 16 bytes into the LDS: plane patches are read from up to 4 bytes early)
  unsigned char* in = lds + (AlgTraits<ALG>::kFamily == 4 ? 16 : 0);
  stage_input<ALG, NW>(x, in, g, tr, bx, c0, wave, lane);
  __syncthreads();
  if constexpr (AlgTraits<ALG>::kFamily == 4) {
    // on the matrix cores: wave = tile, four groups of 16 channels; rounded and packed in
    // registers before V is written over the staged rows
    using Tr = AlgTraits<ALG>;
    constexpr int NPB = MfmaInput<ALG>::NPB, PP = Order<ALG>::PP;
    MfmaInput<ALG> mi;
    mi.load(intab, lane);
    unsigned packed[TPW][4][NPB];
#pragma unroll
    for (int it = 0; it < TPW; ++it) {
      const int tile = wave + NW * it;
      if (tile < tr.ntiles) {
        if (tr.whole) {
          const int tpi = g.th * g.tw;
          const int slot = tile / tpi, rem = tile - slot * tpi;
          const int ti = rem / g.tw, tj = rem - ti * g.tw;
#pragma unroll
          for (int cg = 0; cg < 4; ++cg)
            mi.transform(MfmaInput<ALG>::operand_plane(in + slot * 64 * tr.cs, tr.cs, 16 * cg,
                                                       Tr::M * ti - Tr::PAD, Tr::M * tj - Tr::PAD, g.H,
                                                       g.W, lane),
                         g.qmax, packed[it][cg]);
        } else {
          const int tj0 = (bx % tr.chunks) * tr.tlw;
          const int halo = Tr::M * tj0 - Tr::PAD - ((Tr::M * tj0) & ~3) + 4;
          const int s = tile / tr.tlw, tjl = tile - s * tr.tlw;
#pragma unroll
          for (int cg = 0; cg < 4; ++cg)
            mi.transform(MfmaInput<ALG>::template operand_rect<stage_channel_bytes(Tr::NI)>(
                             in, s, 16 * cg, halo + Tr::M * tjl, lane),
                         g.qmax, packed[it][cg]);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < TPW; ++it) {
      const int tile = wave + NW * it;
      if (tile < tr.ntiles) {
#pragma unroll
        for (int cg = 0; cg < 4; ++cg)
#pragma unroll
          for (int m = 0; m < NPB; ++m) {
            const int pos = 16 * m + (lane & 15);
            if (pos < PP)
              *(unsigned*)(lds + pos * VSP + tile * 64 + 16 * cg + 4 * (lane >> 4)) = packed[it][cg][m];
          }
      }
    }
  } else if constexpr (kRows16) {
    // SFC-6 forms: the sums of an 8x8, 9x9 or 10x10 patch as int8 matrix instructions, wave =
    // tile, four groups of 16 channels; per block of 16 positions two or three steps of 64
    // k-bytes (sfc_mfma_input.hpp).  The coefficients of a block (16-byte loads per lane
    // from the table, the next block's under way) serve the four channel groups.  The rounded
    // bytes of a block are turned round in a piece of LDS that only this wave uses and written
    // to V with 16-byte lanes, 64 contiguous bytes per (position, tile): V never lies in LDS
    // as a whole, so three workgroups share a compute unit and overlap their phases (5x5
    // filters, 128 channels on 28x28 maps, batch 64: 29.1 us with V collected in LDS).
    using Tr = AlgTraits<ALG>;
    static_assert(TPW == 1, "one tile per wave");
    constexpr int PP = Order<ALG>::PP, NPB = (PP + 15) / 16, CS = stage_channel_bytes(Tr::NI);
    static_assert(16 * NPB <= kRowsTabRows && Tr::NI <= 12, "table rows, three steps of four patch rows");
    constexpr int KST = (Tr::NI + 3) / 4;  // steps that carry patch rows
    const float* inv_pos = (const float*)intab;
    const int* point = (const int*)(intab + kRowsTabPoint);
    const unsigned char* ctab = intab + kRowsTabCoeff;
    const int t = wave < tr.ntiles ? row_tab[wave] : -1;  // the same for the whole wave
    if (t >= 0) {
      const int tj0 = (bx % tr.chunks) * tr.tlw;
      const int halo = Tr::M * tj0 - Tr::PAD - ((Tr::M * tj0) & ~3) + 4;
      const int s = wave / tr.tlw, tjl = wave - s * tr.tlw;
      const int o = s * 64 * CS + halo + Tr::M * tjl;
      v4i a[4][KST];
#pragma unroll
      for (int cg = 0; cg < 4; ++cg)
#pragma unroll
        for (int st = 0; st < KST; ++st) a[cg][st] = operand_rows16<CS, Tr::NI>(in, 16 * cg, o, lane, st);
      // this lane's part of a store: position 16 m + lane / 4, channels c0 + 16 (lane % 4) ..
      const unsigned vplane = (unsigned)g.Tp * (unsigned)g.Cp;
      const __amdgpu_buffer_rsrc_t vres =
          __builtin_amdgcn_make_buffer_rsrc((void*)V, 0, (int)(vplane * (unsigned)P), kBufferFlags);
      const unsigned trow = (unsigned)t * (unsigned)g.Cp;
      unsigned char* blk = lds + ip.tab_off - (NW - wave) * (16 * kWaveRowBytes);
      constexpr float kMagic = 12582912.0f;
      const float lo = kMagic - g.qmax, hi = kMagic + g.qmax;
      v4i c_cur[KST], c_nxt[KST];
      float inv_cur, inv_nxt = 0.0f;
      int pt_cur, pt_nxt = -1;
      auto load_block = [&](int m, v4i (&c)[KST], float& inv, int& pt) __attribute__((always_inline)) {
        const int pos = 16 * m + (lane & 15);
        inv = inv_pos[pos];
        pt = point[16 * m + (lane >> 2)];
#pragma unroll
        for (int st = 0; st < KST; ++st) c[st] = *(const v4i*)(ctab + pos * 192 + 64 * st + 16 * (lane >> 4));
      };
      load_block(0, c_cur, inv_cur, pt_cur);
#pragma unroll
      for (int m = 0; m < NPB; ++m) {
        if (m + 1 < NPB) load_block(m + 1, c_nxt, inv_nxt, pt_nxt);
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) {
          v4i d = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[cg][0], c_cur[0], v4i{0, 0, 0, 0}, 0, 0, 0);
#pragma unroll
          for (int st = 1; st < KST; ++st) d = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[cg][st], c_cur[st], d, 0, 0, 0);
          unsigned b[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float v = __fmaf_rn((float)d[i], inv_cur, kMagic);
            v = __builtin_amdgcn_fmed3f(v, lo, hi);
            b[i] = __float_as_uint(v);
          }
          const unsigned w = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u) | __builtin_amdgcn_perm(b[3], b[2], 0x04000c0cu);
          *(unsigned*)(blk + (lane & 15) * kWaveRowBytes + 16 * cg + 4 * (lane >> 4)) = w;
        }
        __builtin_amdgcn_wave_barrier();  // LDS accesses of one wave complete in order
        const v4i d = *(const v4i*)(blk + (lane >> 2) * kWaveRowBytes + 16 * (lane & 3));
        const unsigned pofs =
            pt_cur >= 0 ? (unsigned)pt_cur * vplane + (unsigned)(c0 + 16 * (lane & 3)) : 0x80000000u;
        __builtin_amdgcn_raw_buffer_store_b128(d, vres, pofs, trow, 0);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int st = 0; st < KST; ++st) c_cur[st] = c_nxt[st];
        inv_cur = inv_nxt;
        pt_cur = pt_nxt;
      }
    }
    return;  // (no workgroup barrier after this point on this path)
  } else {
    static_assert(AlgTraits<ALG>::kFamily == 4 || kRows16, "every form has its matrix-core transform");
  }
  __syncthreads();

  // ---- copy out: wave w takes positions w, w+NW, ...; lane = (tile, 16-byte quarter) ---
  const unsigned vplane = (unsigned)g.Tp * (unsigned)g.Cp;
  const __amdgpu_buffer_rsrc_t vres =
      __builtin_amdgcn_make_buffer_rsrc((void*)V, 0, (int)(vplane * (unsigned)P), kBufferFlags);
  const int t = row_tab[VS == 512 ? (lane >> 2) & 7 : lane >> 2];
  const unsigned lane_off = (unsigned)t * (unsigned)g.Cp + (unsigned)(c0 + 16 * (lane & 3));
  if (t >= 0) {
    copy_out_points<ALG, NW, VS, VSP>(lds, vres, lane_off, vplane, wave, lane);
  }
}

// SFC-4 forms on small feature maps (whole images staged as they lie in memory): after the
// one barrier that follows the staging every wave works on its own.  It transforms its tiles on
// the matrix cores (sfc_mfma_input.hpp: lane = (position, four channels)), turns the rounded
// bytes of a tile round in a block of LDS that only it uses -- [position][64 channels], 80 bytes
// from row to row -- and writes them to V with 16-byte lanes, 64 contiguous bytes per
// (position, tile).  No further barrier and no separate copy-out phase: a wave's stores are
// under way while it, and the other waves, transform the next tile.

struct WaveInputPlan {
  TileRect tr;
  unsigned blk_off;  // LDS byte offset of the waves' blocks
  unsigned tab_off;  // ... of the tile -> V row table
  unsigned lds_bytes;
};

template <int ALG, int NW, int TPW>
__global__ __launch_bounds__(NW * 64) void input_transform_waves_kernel(
    const int8_t* __restrict__ x, int8_t* __restrict__ V, const unsigned char* __restrict__ intab,
    Geometry g, WaveInputPlan ip) {
  using Tr = AlgTraits<ALG>;
  static_assert(Tr::kFamily == 4, "the SFC-4 forms");
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int P = Tr::P, PP = Order<ALG>::PP, NPB = MfmaInput<ALG>::NPB;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const TileRect& tr = ip.tr;
  const int cgn = g.Cp >> 6;
  const int pos = xcd_contiguous(blockIdx.x, gridDim.x);
  const int bx = pos / cgn;
  const int c0 = (pos - bx * cgn) * 64;
  int* row_tab = (int*)(lds + ip.tab_off);
  if (threadIdx.x < 16) {
    const int tl = threadIdx.x;
    const TileCoord tc = tile_coord(g, tr, bx, tl);
    row_tab[tl] = tc.live ? (tc.n * g.th + tc.ti) * g.tw + tc.tj : -1;
  }
  unsigned char* in = lds + 16;  // (plane patches are read from up to 4 bytes early)
  stage_images<NW>(x, in, g, tr, bx, c0, wave, lane);

  MfmaInput<ALG> mi;
  mi.load(intab, lane);
  // this lane's part of a store: position 16 m + lane / 4, channels 16 (lane % 4) ..
  const unsigned vplane = (unsigned)g.Tp * (unsigned)g.Cp;
  const __amdgpu_buffer_rsrc_t vres =
      __builtin_amdgcn_make_buffer_rsrc((void*)V, 0, (int)(vplane * (unsigned)P), kBufferFlags);
  const int* point = (const int*)(intab + kInputTabPoints);
  unsigned pofs[NPB];
#pragma unroll
  for (int m = 0; m < NPB; ++m) {
    const int p = point[16 * m + (lane >> 2)];
    pofs[m] = p >= 0 ? (unsigned)p * vplane + (unsigned)(c0 + 16 * (lane & 3)) : 0x80000000u;
  }
  unsigned char* blk = lds + ip.blk_off + wave * (PP * kWaveRowBytes);
  __syncthreads();

  // patch q = 4 * (tile of the wave) + channel group, software-pipelined as in the
  // single-kernel path: reads of patch q + 2 and matrix instructions of patch q + 1 go before
  // the rounding of patch q
  constexpr int NQ = 4 * TPW;
  const int tpi = g.th * g.tw;
  typename MfmaInput<ALG>::PlaneTile ptile = {};
  const unsigned char* planes = in;
  auto fetch = [&](int q) __attribute__((always_inline)) -> v4i {  // q folds to a constant
    if ((q & 3) == 0) {
      const int tile = min(wave + NW * (q >> 2), tr.ntiles - 1);
      const int slot = tile / tpi, rem = tile - slot * tpi;
      const int ti = rem / g.tw, tj = rem - ti * g.tw;
      ptile = MfmaInput<ALG>::plane_tile(Tr::M * ti - Tr::PAD, Tr::M * tj - Tr::PAD, g.H, g.W, lane);
      planes = in + slot * 64 * tr.cs;
    }
    return MfmaInput<ALG>::operand_plane(planes, tr.cs, 16 * (q & 3), ptile, lane);
  };
  unsigned packed[NQ][NPB];
  v4i d_cur[NPB], d_nxt[NPB];
  v4i a_nxt = fetch(0);
  mi.sums(a_nxt, d_cur);
  a_nxt = fetch(1);
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    if (q + 1 < NQ) mi.sums(a_nxt, d_nxt);
    if (q + 2 < NQ) a_nxt = fetch(q + 2);
    __builtin_amdgcn_sched_barrier(0);
    mi.round(d_cur, g.qmax, packed[q]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int m = 0; m < NPB; ++m) d_cur[m] = d_nxt[m];
  }
#pragma unroll
  for (int it = 0; it < TPW; ++it) {
    const int tile = wave + NW * it;
    const int t = tile < tr.ntiles ? row_tab[tile] : -1;  // the same for the whole wave
    if (t >= 0) {
#pragma unroll
      for (int cg = 0; cg < 4; ++cg)
#pragma unroll
        for (int m = 0; m < NPB; ++m) {
          const int j = 16 * m + (lane & 15);
          if (j < PP) *(unsigned*)(blk + j * kWaveRowBytes + 16 * cg + 4 * (lane >> 4)) = packed[4 * it + cg][m];
        }
      __builtin_amdgcn_wave_barrier();  // LDS accesses of one wave complete in order
#pragma unroll
      for (int m = 0; m < NPB; ++m) {
        const int j = 16 * m + (lane >> 2);
        if (j < PP) {
          const v4i d = *(const v4i*)(blk + j * kWaveRowBytes + 16 * (lane & 3));
          __builtin_amdgcn_raw_buffer_store_b128(d, vres, pofs[m], (unsigned)t * (unsigned)g.Cp, 0);
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

static bool make_wave_input_plan(const Geometry& g, WaveInputPlan* ip) {
  if (g.alg != 4 && g.alg != 5) return false;
  const int tpi = g.th * g.tw;
  if (tpi > 16) return false;
  const int slots = tpi > 8 ? 16 : 8;
  const unsigned lds_max = 160u * 1024u;
  if (!make_tile_rect(g, lds_max / 2, &ip->tr, slots, true) || !ip->tr.whole) return false;
  const unsigned pp = (unsigned)((g.P + 3) / 4 * 4);
  ip->blk_off = (16u + tile_rect_stage_bytes(g, ip->tr) + 16u + 15u) & ~15u;
  ip->tab_off = ip->blk_off + 8u * pp * (unsigned)kWaveRowBytes;
  ip->lds_bytes = ip->tab_off + 64u;
  const long long xb = (long long)g.N * g.Cin * g.H * g.W;
  const long long vb = (long long)g.P * g.Tp * g.Cp;
  return ip->lds_bytes <= lds_max && xb < (1ll << 31) && vb < (1ll << 31);
}

template <int ALG>
static hipError_t launch_input_waves_alg(const Geometry& g, const WaveInputPlan& ip, const int8_t* x,
                                         void* V, const unsigned char* intab, hipStream_t s,
                                         bool prepare) {
  const dim3 grid(tile_rect_groups(g, ip.tr) * (unsigned)(g.Cp / 64));
  auto launch = [&](auto kernel) {
    if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel));
    hipLaunchKernelGGL(kernel, grid, dim3(8 * 64), ip.lds_bytes, s, x, (int8_t*)V, intab, g, ip);
    return hipGetLastError();
  };
  return g.th * g.tw > 8 ? launch(input_transform_waves_kernel<ALG, 8, 2>)
                         : launch(input_transform_waves_kernel<ALG, 8, 1>);
}

// waves per workgroup = tiles per workgroup: 16 for the 6x6 forms (rectangles of 16 tiles
// fit their feature maps best); 8 for the 7x7 forms (a 9x10 half-transformed patch per tile
// needs the registers, the 10x12 one of the 5x5-filter forms all the more) and the 4x4
// forms, with half the LDS per workgroup
static int input_waves(int alg) { return alg < 2 ? 16 : 8; }
// tile slots of a workgroup: one per wave, or two per wave for the SFC-4 forms on feature
// maps of 9 to 16 tiles when these then go through whole-image staging: the 64 channel planes
// of an image are one contiguous run, against sparse 64-byte row windows for the 8-tile
// rectangles of two strips (256 channels on 14x14 maps, 128 images: 23.0 -> 14.1 us)
static int input_tile_slots(const Geometry& g) {
  const int tpi = g.th * g.tw;
  if ((g.alg == 4 || g.alg == 5) && tpi > 8 && tpi <= 16) {
    TileRect tr;
    if (make_tile_rect(g, 160u * 1024u - 32u - 64u, &tr, 16, true) && tr.whole) return 16;
  }
  return input_waves(g.alg);
}

static bool make_input_plan(const Geometry& g, InputPlan* ip) {
  const unsigned lds_max = 160u * 1024u;
  const long long xb = (long long)g.N * g.Cin * g.H * g.W;
  const long long vb = (long long)g.P * g.Tp * g.Cp;
  if (xb >= (1ll << 31) || vb >= (1ll << 31)) return false;
  if (g.alg < 4 || g.alg >= 6) {
    // SFC-6 forms: staged rows of one strip (rectangles only), then a block of 16
    // positions per wave; a third of the LDS, so that three workgroups share a compute unit
    const int waves = input_waves(g.alg);  // one tile slot each
    if (!make_tile_rect(g, 48u * 1024u, &ip->tr, waves, true, false)) return false;
    const unsigned xbytes = tile_rect_stage_bytes(g, ip->tr) + 32u;  // (patch reads reach 8 bytes past a row)
    ip->tab_off = ((xbytes + 15u) & ~15u) + (unsigned)waves * 16u * (unsigned)kWaveRowBytes;
    ip->lds_bytes = ip->tab_off + 64u;
    return ip->lds_bytes <= lds_max;
  }
  // (16 more bytes per position for the SFC-4 forms, whose points are padded to 48 / 52)
  const int slots = input_tile_slots(g);
  const unsigned vbytes = (unsigned)((g.P + 3) / 4 * 4) * ((slots == 8 ? 512u : 1024u) + 16u);
  if (vbytes + 16u + 64u > lds_max) return false;
  if (!make_tile_rect(g, lds_max - 32u - 64u, &ip->tr, slots, true)) return false;
  const unsigned xbytes = tile_rect_stage_bytes(g, ip->tr) + 16u;
  ip->tab_off = ((xbytes > vbytes ? xbytes : vbytes) + 15u) & ~15u;
  ip->lds_bytes = ip->tab_off + 64u;
  return ip->lds_bytes <= lds_max;
}

unsigned rows_table_offset(const Geometry& g) {
  if (g.alg == 4 || g.alg == 5) return ~0u;
  return (image_table_bytes(g) + 255u) & ~255u;
}

template <int ALG>
static hipError_t launch_input_i8_alg(const Geometry& g, const InputPlan& ip, const int8_t* x,
                                      void* V, const float* inv_sx, const unsigned char* intab,
                                      hipStream_t s, bool prepare) {
  constexpr int NW = ALG < 2 ? 16 : 8;
  const dim3 grid(tile_rect_groups(g, ip.tr) * (unsigned)(g.Cp / 64));
  if constexpr (AlgTraits<ALG>::kFamily == 4) {
    if (input_tile_slots(g) == 16) {  // two tiles per wave
      auto kernel2 = input_transform_i8_kernel<ALG, NW, 1024, 2>;
      if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel2));
      hipLaunchKernelGGL(kernel2, grid, dim3(NW * 64), ip.lds_bytes, s, x, (int8_t*)V, inv_sx, intab, g, ip);
      return hipGetLastError();
    }
  }
  auto kernel = input_transform_i8_kernel<ALG, NW, NW == 8 ? 512 : 1024>;
  if (prepare) return raise_lds_limit(reinterpret_cast<const void*>(kernel));
  // (the SFC-6 forms read the table of the row-form transform)
  const unsigned toff = rows_table_offset(g);
  const unsigned char* tab = intab && toff != ~0u ? intab + toff : intab;
  hipLaunchKernelGGL(kernel, grid, dim3(NW * 64), ip.lds_bytes, s, x, (int8_t*)V, inv_sx, tab, g, ip);
  return hipGetLastError();
}

// Returns hipErrorNotSupported when the geometry is outside this kernel's limits;
// the caller then uses the generic kernel.
hipError_t launch_input_transform_i8(const Geometry& g, const int8_t* x, void* V,
                                     const float* inv_sx, const unsigned char* intab,
                                     hipStream_t s, bool prepare) {
  if (image_input_supported(g))
    return launch_input_image(g, x, V, intab ? intab + image_table_offset(g) : nullptr, s, prepare);
  WaveInputPlan wp;
  if (make_wave_input_plan(g, &wp))
    return g.alg == 4 ? launch_input_waves_alg<4>(g, wp, x, V, intab, s, prepare)
                      : launch_input_waves_alg<5>(g, wp, x, V, intab, s, prepare);
  InputPlan ip;
  if (!make_input_plan(g, &ip)) return hipErrorNotSupported;
  switch (g.alg) {
    case 0: return launch_input_i8_alg<0>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 1: return launch_input_i8_alg<1>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 2: return launch_input_i8_alg<2>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 3: return launch_input_i8_alg<3>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 4: return launch_input_i8_alg<4>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 5: return launch_input_i8_alg<5>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 6: return launch_input_i8_alg<6>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 7: return launch_input_i8_alg<7>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 8: return launch_input_i8_alg<8>(g, ip, x, V, inv_sx, intab, s, prepare);
    case 9: return launch_input_i8_alg<9>(g, ip, x, V, inv_sx, intab, s, prepare);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
