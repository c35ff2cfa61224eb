// Input-tile transform of the forms with 3x3 filters on small feature maps (the 7x7 and 14x14
// maps of the last stages), requantized mode, on the matrix cores (gfx950).
//
// The samples of a patch that are not padding lie in (NI - 1) W + NI consecutive bytes of the
// channel plane, NI the patch edge.  Where that window is at most 128 bytes, V = B^T x B (Eq. 7
// with the matrices of Sec. 4.1 / Appendix A) of a tile is a sum over the window as it lies
// in memory: k = byte of the plane, counted from the tile's first sample, and KS = 1 or 2
// int8 MFMA 16x16x64 take the sums of 16 channels (operand A: row = channel, k-bytes = the
// window of the channel plane) for 16 multiplication points (operand B: coefficients 0, +-1,
// +-2 by tile of the image and processing position, produced on the host from the add
// networks of sfc_points.hpp for the layer's H and W).
//
// A wave owns one tile and CG groups of 16 channels.  It reads the windows from global memory
// straight into operands (four dword loads per lane, group of channels and step; no staging, no
// workgroup barrier), takes the sums block by block of 16 points, rounds them (four channels
// of a point per lane: one dword), turns each block round in a small piece of LDS that only it
// uses, and writes V[p][t][c .. c + 16 CG) with 16-byte lanes: 16 CG contiguous bytes per
// point.  Waves never wait for each other.
#include <cstring>

#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_mfma_input.hpp"
#include "sfc_points.hpp"

namespace sfc {

// The table behind operand B: float inv_pos[144] (1 / s_Tx by processing position, 0 for
// positions without a point), int point[144] (canonical point of a position, -1: none), int
// base[16] (plane byte of a tile's first sample, by tile of the image), then int8
// coeff[tiles per image][rows][64 KS] ([tile][position][k]), rows = the positions padded to
// whole blocks of 16.
constexpr int kImageTabRows = 144;
constexpr unsigned kImageTabPoint = kImageTabRows * 4;
constexpr unsigned kImageTabBase = kImageTabRows * 8;
constexpr unsigned kImageTabCoeff = kImageTabBase + 64;
constexpr int kImageMaxTiles = 16;

static int image_rows(int alg) {
  const int pp = (alg_points(alg) + 3) / 4 * 4;
  return (pp + 15) / 16 * 16;
}
// bytes from a tile's first sample to its last, plus one
static int image_window(const Geometry& g) {
  const int ni = alg_tile(g.alg) + 2;  // patch edge of the 3x3-filter forms
  return (ni - 1) * g.W + ni;
}
static int image_steps(const Geometry& g) { return g.H * g.W <= 64 || image_window(g) <= 64 ? 1 : 2; }

template <int ALG, int CG, int KS>
__global__ __launch_bounds__(256, 2) void input_transform_image_kernel(
    const int8_t* __restrict__ x, int8_t* __restrict__ V, const unsigned char* __restrict__ tab,
    Geometry g) {
  using Tr = AlgTraits<ALG>;
  static_assert(Tr::R == 3, "3x3 filters");
  constexpr int P = Tr::P, PP = Order<ALG>::PP, NPB = (PP + 15) / 16;
  static_assert(16 * NPB <= kImageTabRows, "table rows");
  // LDS bytes per position of a block: the dword writes of a block fall into 64 different banks
  constexpr int kImageBlockRow = 16 * CG + 16;
  __shared__ __align__(16) unsigned char lds[4 * 16 * kImageBlockRow];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // unit = (tile, channel range), the channel range varying fastest: the waves that write the
  // parts of one row of V run next to each other, on one XCD
  const int ranges = (g.Cp + 16 * CG - 1) / (16 * CG);
  const int unit = xcd_contiguous(blockIdx.x, gridDim.x) * 4 + wave;
  const int t = unit / ranges;  // tiles are numbered image by image
  const int c0 = (unit - t * ranges) * (16 * CG);
  if (t >= g.T) return;  // (whole waves; the kernel has no workgroup barrier)
  const int tpi = g.th * g.tw;
  const int n = t / tpi, tile = t - n * tpi;

  // ---- operands A: 16 bytes from byte base + 64 s + 16 (lane / 16) of the plane of channel
  // c0 + 16 q + lane % 16
  const int hw = g.H * g.W;
  const unsigned xbytes = (unsigned)(g.N * g.Cin) * (unsigned)hw;
  const __amdgpu_buffer_rsrc_t xres =
      __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)xbytes, kBufferFlags);
  const int base = ((const int*)(tab + kImageTabBase))[tile];
  v4i a[CG][KS];
#pragma unroll
  for (int q = 0; q < CG; ++q) {
    const int ch = c0 + 16 * q + (lane & 15);
    const unsigned off = (unsigned)((n * g.Cin + ch) * hw + base + 16 * (lane >> 4));
    // (global dwords need not be aligned; bytes past the window, of the next plane, meet zero
    // coefficients; a dword that would reach past the end of the tensor is fetched byte by
    // byte; channels beyond Cin, the padding of V up to Cp, give zeros)
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const unsigned o = off + 64u * s + 4u * i;
        unsigned v = 0;
        if (ch < g.Cin) {
          if (o + 4u <= xbytes) {
            v = __builtin_amdgcn_raw_buffer_load_b32(xres, o, 0, 0);
          } else {
            for (unsigned bb = 0; o + bb < xbytes; ++bb)
              v |= (unsigned)__builtin_amdgcn_raw_buffer_load_b8(xres, o + bb, 0, 0) << (8 * bb);
          }
        }
        a[q][s][i] = (int)v;
      }
  }

  // ---- operands B and the per-position constants
  const float* inv_pos = (const float*)tab;
  const int* point = (const int*)(tab + kImageTabPoint);
  const unsigned char* ctab = tab + kImageTabCoeff + (unsigned)tile * (unsigned)(16 * NPB * 64 * KS);
  v4i coeff[NPB][KS];
  float inv[NPB];
#pragma unroll
  for (int m = 0; m < NPB; ++m) {
    const int pos = 16 * m + (lane & 15);
    inv[m] = inv_pos[pos];
#pragma unroll
    for (int s = 0; s < KS; ++s)
      coeff[m][s] = *(const v4i*)(ctab + pos * (64 * KS) + 64 * s + 16 * (lane >> 4));
  }
  // this lane's part of a store: position 16 m + RPS h + lane / CG, channels c0 + 16 (lane % CG) ..
  const unsigned vplane = (unsigned)g.Tp * (unsigned)g.Cp;
  const __amdgpu_buffer_rsrc_t vres =
      __builtin_amdgcn_make_buffer_rsrc((void*)V, 0, (int)(vplane * (unsigned)P), kBufferFlags);
  constexpr int LPR = CG;       // lanes per position row (16 bytes each)
  constexpr int RPS = 64 / CG;  // position rows per store instruction
  constexpr int NS = 16 / RPS;  // store instructions per block
  const int piece = lane % LPR, prow = lane / LPR;
  const bool cok = c0 + 16 * piece < g.Cp;
  unsigned pofs[NPB][NS];
#pragma unroll
  for (int m = 0; m < NPB; ++m)
#pragma unroll
    for (int h = 0; h < NS; ++h) {
      const int p = point[16 * m + RPS * h + prow];
      pofs[m][h] = p >= 0 && cok ? (unsigned)p * vplane + (unsigned)(c0 + 16 * piece) : 0x80000000u;
    }
  const unsigned trow = (unsigned)t * (unsigned)g.Cp;
  unsigned char* blk = lds + wave * (16 * kImageBlockRow);

  // ---- block by block of 16 positions; the matrix instructions of block m + 1 are issued
  // before block m is rounded
  auto sums = [&](int m, v4i (&d)[CG]) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < CG; ++q) {
      d[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[q][0], coeff[m][0], v4i{0, 0, 0, 0}, 0, 0, 0);
      if constexpr (KS == 2) d[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[q][1], coeff[m][1], d[q], 0, 0, 0);
    }
  };
  constexpr float kMagic = 12582912.0f;
  const float lo = kMagic - g.qmax, hi = kMagic + g.qmax;
  v4i d_cur[CG], d_nxt[CG];
  sums(0, d_cur);
#pragma unroll
  for (int m = 0; m < NPB; ++m) {
    if (m + 1 < NPB) sums(m + 1, d_nxt);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < CG; ++q) {
      unsigned b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float v = __fmaf_rn((float)d_cur[q][i], inv[m], kMagic);
        v = __builtin_amdgcn_fmed3f(v, lo, hi);
        b[i] = __float_as_uint(v);
      }
      const unsigned w = __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u) | __builtin_amdgcn_perm(b[3], b[2], 0x04000c0cu);
      *(unsigned*)(blk + (lane & 15) * kImageBlockRow + 16 * q + 4 * (lane >> 4)) = w;
    }
    __builtin_amdgcn_wave_barrier();  // LDS accesses of one wave complete in order
#pragma unroll
    for (int h = 0; h < NS; ++h) {
      const v4i d = *(const v4i*)(blk + (RPS * h + prow) * kImageBlockRow + 16 * piece);
      __builtin_amdgcn_raw_buffer_store_b128(d, vres, pofs[m][h], trow, 0);
    }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < CG; ++q) d_cur[q] = d_nxt[q];
  }
}

bool image_input_supported(const Geometry& g) {
  if (g.alg < 0 || g.alg > 5) return false;
  if (g.th * g.tw > kImageMaxTiles) return false;
  if (g.H * g.W > 64 && image_window(g) > 128) return false;
  // the SFC-4 forms on larger maps (16 tiles of a 14x14 image, each reading 128 bytes of every
  // plane) are faster through the kernel that stages whole images (256 channels on 14x14
  // maps, batch 64: 9.1 against 14.2 us)
  if (g.H * g.W > 64 && g.alg >= 4) return false;
  const long long xb = (long long)g.N * g.Cin * g.H * g.W;
  const long long vb = (long long)g.P * g.Tp * g.Cp;
  return xb < (1ll << 31) && vb < (1ll << 31);
}

unsigned image_table_offset(const Geometry& g) {
  return g.alg == 4 || g.alg == 5 ? (kInputTabBytes + 255u) & ~255u : 0u;
}

unsigned image_table_bytes(const Geometry& g) {
  if (!image_input_supported(g)) return 0u;
  return kImageTabCoeff + (unsigned)(g.th * g.tw * image_rows(g.alg) * 64 * image_steps(g));
}

// Coefficients by processing position from the add networks: the image of every unit patch
// under fwd_input (rows, then columns) and for_each_point, for the patch samples that lie in
// the image (patch row i of tile (ti, tj) = image row M ti - PAD + i).
template <int ALG>
static void fill_image_table(const Geometry& g, const float* inv_sx, unsigned char* tab) {
  using Tr = AlgTraits<ALG>;
  constexpr int NI = Tr::NI, NC = Tr::NC;
  constexpr Order<ALG> order{};
  const int ks = image_steps(g), rows = image_rows(g.alg);
  std::memset(tab, 0, image_table_bytes(g));
  float* inv_pos = reinterpret_cast<float*>(tab);
  int* point = reinterpret_cast<int*>(tab + kImageTabPoint);
  int* base = reinterpret_cast<int*>(tab + kImageTabBase);
  signed char* coeff = reinterpret_cast<signed char*>(tab) + kImageTabCoeff;
  for (int p = 0; p < Tr::P; ++p) inv_pos[order.pos[p]] = inv_sx[p];
  for (int j = 0; j < kImageTabRows; ++j) point[j] = j < Order<ALG>::PP ? order.pt[j] : -1;
  for (int tile = 0; tile < g.th * g.tw; ++tile) {
    const int r0 = Tr::M * (tile / g.tw) - Tr::PAD, q0 = Tr::M * (tile % g.tw) - Tr::PAD;
    // maps of at most 64 samples are read from their first byte whatever the tile
    const int b0 = g.H * g.W <= 64 ? 0 : (r0 > 0 ? r0 : 0) * g.W + (q0 > 0 ? q0 : 0);
    base[tile] = b0;
    signed char* ct = coeff + (size_t)tile * rows * 64 * ks;
    for (int i = 0; i < NI; ++i)
      for (int j = 0; j < NI; ++j) {
        const int h = r0 + i, w = q0 + j;
        if (h < 0 || h >= g.H || w < 0 || w >= g.W) continue;
        const int k = h * g.W + w - b0;  // 0 <= k < 64 ks (image_input_supported)
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
        for_each_point<ALG>(comp, [&](int p, int v) { ct[order.pos[p] * 64 * ks + k] = (signed char)v; });
      }
  }
}

void build_image_input_table(const Geometry& g, const float* inv_sx, unsigned char* tab) {
  switch (g.alg) {
    case 0: fill_image_table<0>(g, inv_sx, tab); break;
    case 1: fill_image_table<1>(g, inv_sx, tab); break;
    case 2: fill_image_table<2>(g, inv_sx, tab); break;
    case 3: fill_image_table<3>(g, inv_sx, tab); break;
    case 4: fill_image_table<4>(g, inv_sx, tab); break;
    case 5: fill_image_table<5>(g, inv_sx, tab); break;
    default: break;
  }
}

template <int ALG>
static hipError_t launch_image_alg(const Geometry& g, const int8_t* x, void* V,
                                   const unsigned char* tab, hipStream_t s) {
  // 64 channels per wave (128, with 128-byte pieces of V per store, measured no faster: 512
  // channels on 7x7 maps, 256 images, 7x7 tiles: 9.8 against 9.1 us)
  const int ranges = g.Cp / 64;
  const unsigned grid = (unsigned)(((long long)g.T * ranges + 3) / 4);
  auto launch = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), 0, s, x, (int8_t*)V, tab, g);
    return hipGetLastError();
  };
  return image_steps(g) == 1 ? launch(input_transform_image_kernel<ALG, 4, 1>)
                             : launch(input_transform_image_kernel<ALG, 4, 2>);
}

hipError_t launch_input_image(const Geometry& g, const int8_t* x, void* V, const unsigned char* tab,
                              hipStream_t s, bool prepare) {
  if (!image_input_supported(g)) return hipErrorNotSupported;
  if (prepare) return hipSuccess;  // static LDS only
  switch (g.alg) {
    case 0: return launch_image_alg<0>(g, x, V, tab, s);
    case 1: return launch_image_alg<1>(g, x, V, tab, s);
    case 2: return launch_image_alg<2>(g, x, V, tab, s);
    case 3: return launch_image_alg<3>(g, x, V, tab, s);
    case 4: return launch_image_alg<4>(g, x, V, tab, s);
    case 5: return launch_image_alg<5>(g, x, V, tab, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
