// The whole hot path in one kernel, for layers with Cin <= 64 (gfx950): input-tile
// transform, transform-domain products and output transform without V or M ever
// leaving the compute unit.
//
// A workgroup of 16 waves (8 for the 7x7 forms, each wave then doing two passes)
// owns a rectangle of up to 16 tiles (S strips x tlw tile columns; a strip = one
// row of tiles of one image), all input channels and a group of 64 filters.
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

namespace sfc {

struct SinglePlan {
  int S;       // strips per workgroup
  int chunks;  // tile-column chunks per strip
  int tlw;     // tile columns per chunk
  int ntiles;  // S * tlw <= 16
  int kgroups; // groups of 64 filters
  unsigned long long th_magic;  // ceil(2^32 / th): strip / th = (strip * th_magic) >> 32
  unsigned stage_off;  // LDS byte offset of the per-wave output staging blocks
  unsigned lds_bytes;
};

constexpr int kWaves6 = 16;  // waves per workgroup for the 6x6 forms

template <int ALG, int OUT, bool VEC2, bool ALIGNED, int NW>
__global__ __launch_bounds__(NW * 64) void single_conv_kernel(
    const int8_t* __restrict__ x, const int8_t* __restrict__ Uf, const float* __restrict__ dqf,
    const float* __restrict__ inv_sx, float x_scale, float inv_y, void* __restrict__ y, Geometry g,
    SinglePlan sp) {
  using Tr = AlgTraits<ALG>;
  constexpr int P = Tr::P, M = Tr::M, NI = Tr::NI, NC = Tr::NC, PG = P / 4;
  constexpr int ROWG = (NI + 3) / 4;  // groups of four staged rows
  constexpr int SPW = 16 / NW;        // passes per wave over tile groups / filter quads
  // staging layout: 64 bytes per image row (byte 4 = image column colbase), M+2 rows per
  // (strip, channel), one extra dword so that the channel stride is an odd number of
  // dwords and lanes running along channels hit distinct banks
  constexpr int WP = 64, CS = NI * WP + 4;
  static_assert(NW == 8 || NW == 16, "8 or 16 waves");
  constexpr Order<ALG> order{};
  static_assert(P % 4 == 0, "points are processed in groups of four");
  extern __shared__ __align__(16) unsigned char lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int bx = xcd_contiguous(blockIdx.x, gridDim.x);
  const int chunk = bx % sp.chunks;
  const int strip0 = (bx / sp.chunks) * sp.S;
  const int tj0 = chunk * sp.tlw;
  const int colbase = (M * tj0) & ~3;            // image column held at LDS byte 4 of a row
  const int halo = M * tj0 - 1 - colbase + 4;    // LDS byte of the chunk's first patch column
  const int W = g.W, H = g.H;

  // per-tile store data for step 4, written by 16 lanes now and read after the barriers:
  // output offset of the tile's first element for filter 0, valid rows (0: no tile), valid columns
  int* tile_tab = (int*)(lds + sp.stage_off + NW * 64 * M * 4);
  if (threadIdx.x < 16) {
    const int tl = threadIdx.x;
    const int s = tl / sp.tlw, tjl = tl - s * sp.tlw;
    const int strip = strip0 + s, tj = tj0 + tjl;
    const int n = (int)(((unsigned long long)(unsigned)strip * sp.th_magic) >> 32);
    const int ti = strip - n * g.th;
    const bool live = tl < sp.ntiles && strip < g.strips && tj < g.tw;
    tile_tab[tl] = ((n * g.Cout) * H + M * ti) * W + M * tj;
    tile_tab[16 + tl] = live ? min(M, H - M * ti) : 0;
    tile_tab[32 + tl] = min(M, W - M * tj);
  }

  // ---- 1. stage ------------------------------------------------------------------
  // One instruction covers four rows x 16 dwords of one (strip, channel): lane =
  // (row within the group, dword).  Wave w takes the (strip, channel) pairs w,
  // w+NW, ...; a batch of pairs is in flight before the first LDS write.
  {
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)x, 0, (int)((unsigned)(g.N * g.Cin) * (unsigned)(H * W)), kBufferFlags);
    const int rsub = lane >> 4, dcol = lane & 15;
    const int col = colbase + 4 * dcol - 4;  // image column of this lane's dword
    const unsigned plane_stride = (unsigned)(H * W);
    const int npairs = sp.S * 64;
    constexpr int BATCH = 24 / ROWG;
    if constexpr (ALIGNED) {
      // W % 4 == 0: every dword lies wholly inside or outside its image row, and every
      // address is dword aligned.  A wave walks over (strip, row group) combinations;
      // within one, only the channel plane changes from load to load (wave w takes
      // channels w, w+NW, ...), so the lane address and its validity are computed once
      // per combination.  Lanes without data (padding halo, dead strips) get an offset
      // beyond the buffer, for which a buffer load returns zero without touching memory.
      // All loads of a batch are in flight before the first LDS write.
      const bool lane_ok = col >= 0 && col < W;
      const int lane_off = rsub * W + col;     // lane part of the byte offset
      constexpr unsigned kOutOfRange = 0x80000000u;  // beyond any x: the buffer load returns 0
      constexpr int CPW = 64 / NW;  // channels per wave
      constexpr int CB = 6;         // combinations per batch
      const int ncombo = sp.S * ROWG;
      for (int k0 = 0; k0 < ncombo; k0 += CB) {
        unsigned vals[CB][CPW];
#pragma unroll
        for (int kk = 0; kk < CB; ++kk) {
          const int k = k0 + kk;
          const int s = k / ROWG, rg = k - s * ROWG;
          const int strip = strip0 + s;
          const bool live = k < ncombo && strip < g.strips;
          const int n = (int)(((unsigned long long)(unsigned)strip * sp.th_magic) >> 32);
          const int ti = strip - n * g.th;
          const int hlo = M * ti - 1 + 4 * rg;             // image row of rsub = 0
          const int base = (n * g.Cin * H + hlo) * W;       // its offset in channel 0 of image n
          const bool ok = live && lane_ok && 4 * rg + rsub < NI &&
                          (unsigned)(hlo + rsub) < (unsigned)H;
          const unsigned voff = ok ? (unsigned)(base + lane_off) : kOutOfRange;
#pragma unroll
          for (int ci = 0; ci < CPW; ++ci) {
            // channels beyond Cin re-read the last one: their filter operand is zero
            const int c = min(wave + NW * ci, g.Cin - 1);
            vals[kk][ci] =
                __builtin_amdgcn_raw_buffer_load_b32(xres, voff, (unsigned)c * plane_stride, 0);
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
    } else {
      // Any W: global dwords need not be aligned; a dword that straddles the end of an
      // image row is assembled from its valid bytes.
      const int nvalid = col < 0 ? 0 : min(4, max(0, W - col));
      for (int q0 = wave; q0 < npairs; q0 += NW * BATCH) {
        unsigned vals[BATCH][ROWG];
#pragma unroll
        for (int bi = 0; bi < BATCH; ++bi) {
          const int q = q0 + NW * bi;
          const int s = q >> 6, c = q & 63;
          const int strip = strip0 + s;
          const bool live = q < npairs && strip < g.strips && c < g.Cin && nvalid > 0;
          const int n = (int)(((unsigned long long)(unsigned)strip * sp.th_magic) >> 32);
          const int ti = strip - n * g.th;
          const unsigned plane = (unsigned)(n * g.Cin + c) * plane_stride;
#pragma unroll
          for (int rg = 0; rg < ROWG; ++rg) {
            const int row = rg * 4 + rsub;
            const int h = M * ti - 1 + row;
            unsigned val = 0;
            if (live && row < NI && h >= 0 && h < H) {
              const unsigned voff = (unsigned)(h * W + col);
              if (nvalid == 4) {
                val = __builtin_amdgcn_raw_buffer_load_b32(xres, voff, plane, 0);
              } else {
                for (int bb = 0; bb < nvalid; ++bb)
                  val |= (unsigned)__builtin_amdgcn_raw_buffer_load_b8(xres, voff + bb, plane, 0)
                         << (8 * bb);
              }
            }
            vals[bi][rg] = val;
          }
        }
#pragma unroll
        for (int bi = 0; bi < BATCH; ++bi) {
          const int q = q0 + NW * bi;
          if (q < npairs) {
#pragma unroll
            for (int rg = 0; rg < ROWG; ++rg) {
              const int row = rg * 4 + rsub;
              if (row < NI)
                *(unsigned*)(lds + (unsigned)q * CS + row * WP + 4 * dcol) = vals[bi][rg];
            }
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- 2. input transform: wave = tile (SPW of them per wave), lane = channel ----------
  // Lanes running along channels are an odd number of dwords apart in the staging
  // area, so the aligned dword reads of a patch row hit 64 different banks.
  {
    int half[SPW][NI][NC];  // rows transformed: half[.][i][b]
#pragma unroll
    for (int it = 0; it < SPW; ++it) {
      const int tile = wave + NW * it, c = lane;
      if (tile < sp.ntiles) {
        const int s = tile / sp.tlw, tjl = tile - s * sp.tlw;
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
      if (tile < sp.ntiles) {
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
          outp[order.pos[p] * 1024] = (unsigned char)quantize_byte(v, inv_sx[p]);
        });
      }
    }
  }
  __syncthreads();

  // ---- 3. products + output transform: lane = (tile l%16, filter 4*kq + l/16) ------
  const int kfilters = sp.kgroups * 64;
  const __amdgpu_buffer_rsrc_t ures = __builtin_amdgcn_make_buffer_rsrc(
      (void*)Uf, 0, (int)((unsigned)kfilters * (unsigned)(P * 64)), kBufferFlags);
  const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)dqf, 0, (int)((unsigned)kfilters * (unsigned)(P * 4)), kBufferFlags);
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      y, 0, (int)(esz * (unsigned)(g.N * g.Cout) * (unsigned)(H * W)), kBufferFlags);
  const unsigned char* vlane = lds + (lane & 15) * 64 + (lane >> 4) * 16;  // tile l%16, channels 16*(l/16)..
  // this wave's private staging block for one output row: [filter 0..3][tile 0..15][o2]
  float* stage = (float*)(lds + sp.stage_off) + wave * (64 * M);
  // Cache policy of the y stores.  7x7 tiles divide the ResNet image widths, a
  // workgroup then writes whole image rows and the lines can stream past the L2 ("nt");
  // 6x6 tiles leave row pieces that share cache lines with a neighbouring workgroup,
  // which the L2 has to merge before they go to memory.
  constexpr int kStore = M == 7 ? kStreamStore : 0;
  constexpr int EV = VEC2 ? 2 : 1;      // elements per lane and store
  constexpr int NST = (M + EV - 1) / EV;  // stores per lane and output row (64*M elements)

#pragma unroll 1
  for (int qi = 0; qi < SPW; ++qi) {
    const int kq = blockIdx.y * 16 + wave + NW * qi;  // filter quad of this pass
    const int kcol = kq * 4 + (lane >> 4);            // this lane's filter
    const unsigned a_lane = (unsigned)lane * 16u;
    const unsigned a_wave = (unsigned)kq * (unsigned)(PG * 1024);
    const unsigned d_lane = (unsigned)kcol * (unsigned)(P * 4);
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

    // ---- 4. store: one output row at a time through the wave's staging block ------
    // store plan: the k-th store of this lane covers elements e = EV*(lane + 64*k) of
    // the staged row block, e = (filter*16 + tile)*M + o2; consecutive lanes hold
    // consecutive outputs of an image row (tiles of a strip are adjacent in y)
    unsigned yoff[NST];
    int rowlim[NST];
#pragma unroll
    for (int k = 0; k < NST; ++k) {
      const unsigned e = (unsigned)(EV * (lane + 64 * k));
      const unsigned ft = e / (unsigned)M;  // filter*16 + tile
      const int o2 = (int)(e - ft * M), f = (int)(ft >> 4), tl = (int)(ft & 15);
      const int kc = kq * 4 + f;
      const bool valid = e < 64u * M && kc < g.Cout && o2 < tile_tab[32 + tl];
      rowlim[k] = valid ? tile_tab[16 + tl] : 0;
      yoff[k] = esz * (unsigned)(tile_tab[tl] + kc * (H * W) + o2);
    }
    float* wr = stage + ((lane >> 4) * 16 + (lane & 15)) * M;
#pragma unroll
    for (int o1 = 0; o1 < M; ++o1) {
      float out[M];
      stream_row<ALG, float>(z, o1, out);
      if constexpr (M % 2 == 0) {
#pragma unroll
        for (int o2 = 0; o2 < M; o2 += 2)
          *(v2f*)(wr + o2) = v2f{out[o2] * x_scale, out[o2 + 1] * x_scale};
      } else {
#pragma unroll
        for (int o2 = 0; o2 < M; ++o2) wr[o2] = out[o2] * x_scale;
      }
      __builtin_amdgcn_wave_barrier();  // LDS accesses of one wave complete in order
      const unsigned yrow = esz * (unsigned)(o1 * W);
#pragma unroll
      for (int k = 0; k < NST; ++k) {
        float v0, v1 = 0.0f;
        if constexpr (VEC2) {
          const v2f pr = *(const v2f*)(stage + 2 * (lane + 64 * k));
          v0 = pr.x;
          v1 = pr.y;
        } else {
          v0 = (64 * k + lane < 64 * M) ? stage[lane + 64 * k] : 0.0f;
        }
        if (o1 < rowlim[k]) {
          if constexpr (OUT == 2) {
            // next layer's activation: ReLU, round half to even, clamp to [0, 127]
            constexpr float kMagic = 12582912.0f;
            float t0 = __fmaf_rn(v0, inv_y, kMagic), t1 = __fmaf_rn(v1, inv_y, kMagic);
            t0 = __builtin_amdgcn_fmed3f(t0, kMagic, kMagic + 127.0f);
            t1 = __builtin_amdgcn_fmed3f(t1, kMagic, kMagic + 127.0f);
            const unsigned q0 = __float_as_uint(t0) & 0xffu, q1 = __float_as_uint(t1) & 0xffu;
            if constexpr (VEC2)
              __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(q0 | (q1 << 8)), yres, yoff[k],
                                                    yrow, kStore);
            else
              __builtin_amdgcn_raw_buffer_store_b8((unsigned char)q0, yres, yoff[k], yrow,
                                                   kStore);
          } else {
            if constexpr (VEC2)
              __builtin_amdgcn_raw_buffer_store_b64(v2f{v0, v1}, yres, yoff[k], yrow, kStore);
            else
              __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v0), yres, yoff[k], yrow,
                                                    kStore);
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// Filter operand of the kernel above from the canonical U[p][k][c] (Cp = 64):
// block (filter quad kq, point group pg) is one KiB; lane l holds 16 channels
// 16*(l/16).. of point pt[4*pg + (l%16)%4], filter 4*kq + (l%16)/4.  Filters
// beyond Kp are zero.
template <int ALG>
__global__ __launch_bounds__(64) void repack_filter_kernel(const int8_t* __restrict__ U,
                                                           int8_t* __restrict__ Uf, Geometry g) {
  constexpr int PG = AlgTraits<ALG>::P / 4;
  constexpr Order<ALG> order{};
  const int kq = blockIdx.x / PG, pg = blockIdx.x - kq * PG;
  const int l = threadIdx.x;
  const int i = l & 15, kseg = l >> 4;
  const int p = order.pt[4 * pg + (i & 3)];
  const int k = 4 * kq + (i >> 2);
  v4i val = {0, 0, 0, 0};
  if (k < g.Kp) val = *(const v4i*)(U + ((size_t)p * g.Kp + k) * g.Cp + 16 * kseg);
  *(v4i*)(Uf + ((size_t)blockIdx.x * 64 + l) * 16) = val;
}

// waves per workgroup: the 7x7 forms carry 10x7 partial outputs per pair and need the
// 256-register budget of 8 waves
static int single_waves(int alg) { return alg_tile(alg) == 6 ? kWaves6 : 8; }

static bool make_single_plan(const Geometry& g, SinglePlan* sp) {
  if (g.Cp != 64) return false;
  const int M = alg_tile(g.alg), NI = M + 2;
  const int tlw_max = (64 - 7) / M < 16 ? (64 - 7) / M : 16;  // wp = 5 + M*tlw + 2 rounded up <= 64
  const int min_chunks = (g.tw + tlw_max - 1) / tlw_max;
  // LDS: the staged rows of S strips (later overwritten by V), the per-wave output
  // staging blocks, the per-tile store table
  const unsigned cs = (unsigned)NI * 64u + 4u;  // staged bytes per (strip, channel), as in the kernel
  const unsigned vbytes = (unsigned)g.P * 1024u;
  const unsigned sbytes = (unsigned)single_waves(g.alg) * 64u * (unsigned)M * 4u + 256u;
  const unsigned lds_max = 160u * 1024u;
  if (vbytes + 16u + sbytes > lds_max) return false;
  const int s_fit = (int)((lds_max - 16u - sbytes) / (64u * cs));
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
      sp->chunks = chunks;
      sp->tlw = tlw;
      sp->S = S;
    }
  }
  sp->kgroups = (g.Cout + 63) / 64;
  const unsigned xbytes = (unsigned)sp->S * 64u * cs;
  sp->stage_off = ((xbytes > vbytes ? xbytes : vbytes) + 15u) & ~15u;
  sp->lds_bytes = sp->stage_off + sbytes;
  sp->ntiles = sp->S * sp->tlw;
  // the reciprocal is exact while strip * th < 2^32
  if ((long long)g.strips * g.th >= (1ll << 32) || g.th < 1) return false;
  sp->th_magic = ((1ull << 32) + (unsigned long long)g.th - 1) / (unsigned long long)g.th;
  const long long xb = (long long)g.N * g.Cin * g.H * g.W;
  const long long yb = 4ll * g.N * g.Cout * g.H * g.W;
  const long long ub = (long long)sp->kgroups * 64 * g.P * 64;
  const long long lim = 1ll << 31;
  return 5 + M * sp->tlw + 2 <= 64 && sp->ntiles >= 1 && sp->ntiles <= 16 && sp->lds_bytes <= 160u * 1024u &&
         xb < lim && yb < lim && ub < lim;
}

bool single_supported(const Geometry& g) {
  SinglePlan sp;
  return make_single_plan(g, &sp);
}

size_t single_filter_bytes(const Geometry& g) {  // operand bytes; the table has kgroups*64*P floats
  return (size_t)((g.Cout + 63) / 64) * 64 * g.P * 64;
}

hipError_t launch_repack_filter(const Geometry& g, const void* U, void* Uf, hipStream_t s) {
  const int kq = ((g.Cout + 63) / 64) * 16;
  const dim3 grid((unsigned)(kq * (g.P / 4)));
  switch (g.alg) {
    case 0: hipLaunchKernelGGL(repack_filter_kernel<0>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 1: hipLaunchKernelGGL(repack_filter_kernel<1>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 2: hipLaunchKernelGGL(repack_filter_kernel<2>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    case 3: hipLaunchKernelGGL(repack_filter_kernel<3>, grid, dim3(64), 0, s, (const int8_t*)U, (int8_t*)Uf, g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// processing position -> canonical point index, for the host-built tables
void single_point_order(int alg, int* pt /*[P]*/) {
  auto copy = [&](const auto& o) {
    for (int j = 0; j < (int)(sizeof(o.pt) / sizeof(o.pt[0])); ++j) pt[j] = o.pt[j];
  };
  switch (alg) {
    case 0: { constexpr Order<0> o{}; copy(o); break; }
    case 1: { constexpr Order<1> o{}; copy(o); break; }
    case 2: { constexpr Order<2> o{}; copy(o); break; }
    default: { constexpr Order<3> o{}; copy(o); break; }
  }
}

template <int ALG, int OUT, bool VEC2, bool ALIGNED, int NW>
static hipError_t launch_single_impl(const Geometry& g, const SinglePlan& sp, const int8_t* x,
                                     const FilterViews& f, float x_scale, float inv_y, void* y,
                                     hipStream_t s) {
  auto kernel = single_conv_kernel<ALG, OUT, VEC2, ALIGNED, NW>;
  static bool attr_done = false;  // raises the dynamic LDS limit of this instantiation once
  if (!attr_done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    (void)hipGetLastError();
    attr_done = true;
  }
  const dim3 grid((unsigned)(((g.strips + sp.S - 1) / sp.S) * sp.chunks), (unsigned)sp.kgroups);
  hipLaunchKernelGGL(kernel, grid, dim3(NW * 64), sp.lds_bytes, s, x, (const int8_t*)f.U_single,
                     f.dequant_single, f.inv_sx, x_scale, inv_y, y, g, sp);
  return hipGetLastError();
}

template <int ALG, int OUT>
static hipError_t launch_single_out(const Geometry& g, const SinglePlan& sp, const int8_t* x,
                                    const FilterViews& f, float x_scale, float inv_y, void* y,
                                    hipStream_t s) {
  constexpr int NW = AlgTraits<ALG>::M == 6 ? kWaves6 : 8;
  constexpr bool kPairs = AlgTraits<ALG>::M % 2 == 0;  // pairs of an output row stay aligned
  const bool aligned = g.W % 4 == 0;  // staged dwords are aligned and never straddle a row end
  if constexpr (kPairs) {
    if (g.W % 2 == 0)
      return aligned ? launch_single_impl<ALG, OUT, true, true, NW>(g, sp, x, f, x_scale, inv_y, y, s)
                     : launch_single_impl<ALG, OUT, true, false, NW>(g, sp, x, f, x_scale, inv_y, y, s);
  }
  return aligned ? launch_single_impl<ALG, OUT, false, true, NW>(g, sp, x, f, x_scale, inv_y, y, s)
                 : launch_single_impl<ALG, OUT, false, false, NW>(g, sp, x, f, x_scale, inv_y, y, s);
}

template <int ALG>
static hipError_t launch_single_alg(int out, const Geometry& g, const SinglePlan& sp,
                                    const int8_t* x, const FilterViews& f, float x_scale,
                                    float inv_y, void* y, hipStream_t s) {
  return out == 2 ? launch_single_out<ALG, 2>(g, sp, x, f, x_scale, inv_y, y, s)
                  : launch_single_out<ALG, 0>(g, sp, x, f, x_scale, inv_y, y, s);
}

hipError_t launch_single_conv(int out, const Geometry& g, const int8_t* x, const FilterViews& f,
                              float x_scale, float inv_y, void* y, hipStream_t s) {
  SinglePlan sp;
  if (!make_single_plan(g, &sp) || out == 1) return hipErrorNotSupported;
  switch (g.alg) {
    case 0: return launch_single_alg<0>(out, g, sp, x, f, x_scale, inv_y, y, s);
    case 1: return launch_single_alg<1>(out, g, sp, x, f, x_scale, inv_y, y, s);
    case 2: return launch_single_alg<2>(out, g, sp, x, f, x_scale, inv_y, y, s);
    case 3: return launch_single_alg<3>(out, g, sp, x, f, x_scale, inv_y, y, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
