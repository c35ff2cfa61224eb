// Input-tile transform of the forms with 3x3 filters on feature maps of at most 64 samples
// and at most four tiles (the 7x7 maps of the last stage: one 7x7 tile of Sec. 4.2, or four
// 4x4 tiles), requantized mode, on the matrix cores (gfx950).
//
// Every sample of a patch lies in the image or is padding, so V = B^T x B (Eq. 7 with the
// matrices of Sec. 4.1 / Appendix A) of any tile is a sum over the H W <= 64 image samples:
// k = h W + w indexes them as they lie in memory, and one int8 MFMA 16x16x64 takes the sums
// of 16 channels (operand A: row = channel, 64 k-bytes = the start of the channel plane, the
// same for every tile of the image) for 16 multiplication points (operand B: coefficients
// 0, +-1, +-2 by tile of the image and processing position, produced on the host from the
// add networks of sfc_points.hpp for the layer's H and W).
//
// A wave owns one tile and CG groups of 16 channels.  It reads its planes from global memory
// straight into operands (four dword loads per lane and group of channels; no staging, no
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

// the table behind operand B: float inv_pos[144] (1 / s_Tx by processing position, 0 for
// positions without a point), int point[144] (canonical point of a position, -1: none), int8
// coeff[tiles per image][144][64] ([tile][position][k])
constexpr unsigned kImageTabPoint = kImageTabRows * 4;
constexpr unsigned kImageTabCoeff = kImageTabRows * 8;
constexpr unsigned kImageTabTile = kImageTabRows * 64;
constexpr int kImageMaxTiles = 4;


template <int ALG, int CG>
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

  // ---- operands A: 16 bytes from byte 16 (lane / 16) of the plane of channel c0 + 16 q + lane % 16
  const int hw = g.H * g.W;
  const unsigned xbytes = (unsigned)(g.N * g.Cin) * (unsigned)hw;
  const __amdgpu_buffer_rsrc_t xres =
      __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)xbytes, kBufferFlags);
  v4i a[CG];
#pragma unroll
  for (int q = 0; q < CG; ++q) {
    const int ch = c0 + 16 * q + (lane & 15);
    const unsigned off = (unsigned)((n * g.Cin + ch) * hw + 16 * (lane >> 4));
    // (global dwords need not be aligned; a dword that would reach past the end of the tensor
    // is fetched byte by byte; channels beyond Cin, the padding of V up to Cp, give zeros)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned o = off + 4u * i;
      unsigned v = 0;
      if (ch < g.Cin) {
        if (o + 4u <= xbytes) {
          v = __builtin_amdgcn_raw_buffer_load_b32(xres, o, 0, 0);
        } else {
          for (unsigned bb = 0; o + bb < xbytes; ++bb)
            v |= (unsigned)__builtin_amdgcn_raw_buffer_load_b8(xres, o + bb, 0, 0) << (8 * bb);
        }
      }
      a[q][i] = (int)v;
    }
  }

  // ---- operands B and the per-position constants
  const float* inv_pos = (const float*)tab;
  const int* point = (const int*)(tab + kImageTabPoint);
  const unsigned char* ctab = tab + kImageTabCoeff + (unsigned)tile * kImageTabTile;
  v4i coeff[NPB];
  float inv[NPB];
#pragma unroll
  for (int m = 0; m < NPB; ++m) {
    const int pos = 16 * m + (lane & 15);
    inv[m] = inv_pos[pos];
    coeff[m] = *(const v4i*)(ctab + pos * 64 + 16 * (lane >> 4));
  }
  // this lane's part of a store: position 16 m + 8 h + lane / 8, channels c0 + 16 (lane % 8) ..
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
    for (int q = 0; q < CG; ++q)
      d[q] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[q], coeff[m], v4i{0, 0, 0, 0}, 0, 0, 0);
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
        float t = __fmaf_rn((float)d_cur[q][i], inv[m], kMagic);
        t = __builtin_amdgcn_fmed3f(t, lo, hi);
        b[i] = __float_as_uint(t);
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
  if (g.th * g.tw > kImageMaxTiles || g.H * g.W > 64) return false;
  const long long xb = (long long)g.N * g.Cin * g.H * g.W;
  const long long vb = (long long)g.P * g.Tp * g.Cp;
  return xb < (1ll << 31) && vb < (1ll << 31);
}

// Coefficients by processing position from the add networks: the image of every unit patch
// under fwd_input (rows, then columns) and for_each_point, for the patch samples that lie in
// the image (patch row i = image row i - PAD).
template <int ALG>
static void fill_image_table(const Geometry& g, const float* inv_sx, unsigned char* tab) {
  using Tr = AlgTraits<ALG>;
  constexpr int NI = Tr::NI, NC = Tr::NC;
  constexpr Order<ALG> order{};
  std::memset(tab, 0, image_table_bytes(g));
  float* inv_pos = reinterpret_cast<float*>(tab);
  int* point = reinterpret_cast<int*>(tab + kImageTabPoint);
  signed char* coeff = reinterpret_cast<signed char*>(tab) + kImageTabCoeff;
  for (int p = 0; p < Tr::P; ++p) inv_pos[order.pos[p]] = inv_sx[p];
  for (int j = 0; j < kImageTabRows; ++j) point[j] = j < Order<ALG>::PP ? order.pt[j] : -1;
  for (int tile = 0; tile < g.th * g.tw; ++tile) {
    const int r0 = Tr::M * (tile / g.tw) - Tr::PAD, q0 = Tr::M * (tile % g.tw) - Tr::PAD;
    for (int i = 0; i < NI; ++i)
      for (int j = 0; j < NI; ++j) {
        const int h = r0 + i, w = q0 + j;
        if (h < 0 || h >= g.H || w < 0 || w >= g.W) continue;
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
        for_each_point<ALG>(comp, [&](int p, int v) {
          coeff[(unsigned)tile * kImageTabTile + order.pos[p] * 64 + h * g.W + w] = (signed char)v;
        });
      }
  }
}

unsigned image_table_offset(const Geometry& g) {
  return g.alg == 4 || g.alg == 5 ? (kInputTabBytes + 255u) & ~255u : 0u;
}

unsigned image_table_bytes(const Geometry& g) {
  return image_input_supported(g) ? kImageTabCoeff + (unsigned)(g.th * g.tw) * kImageTabTile : 0u;
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
  // 128 channels per wave where that leaves at least eight waves per compute unit, else 64
  const bool wide = (long long)g.T * ((g.Cp + 127) / 128) >= 2048;
  const int ranges = wide ? (g.Cp + 127) / 128 : g.Cp / 64;
  const unsigned grid = (unsigned)(((long long)g.T * ranges + 3) / 4);
  if (wide)
    hipLaunchKernelGGL((input_transform_image_kernel<ALG, 8>), dim3(grid), dim3(256), 0, s, x, (int8_t*)V, tab, g);
  else
    hipLaunchKernelGGL((input_transform_image_kernel<ALG, 4>), dim3(grid), dim3(256), 0, s, x, (int8_t*)V, tab, g);
  return hipGetLastError();
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
