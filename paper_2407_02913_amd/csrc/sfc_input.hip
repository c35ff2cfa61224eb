// Input-tile transform V = B^T x B with transform-domain requantization to int8,
// the HBM-facing first stage of the hot path (gfx950).
//
// A workgroup owns S strips (a strip = one row of tiles of one image, i.e. the
// eight input rows 6*ti-1 .. 6*ti+6) x a chunk of up to six tile columns x 64
// channels.  Wave w of the workgroup is tile w of that set, lane c is channel c.
//
//  1. Stage: the eight rows of a (strip, channel) are contiguous in NCHW, so the
//     workgroup copies them to LDS with dword loads (four rows x 16 dwords per
//     instruction), zero-filling the padding halo.  The channel stride is an odd
//     number of dwords so that lanes running along channels hit distinct banks.
//  2. Transform: each thread reads its 8x8 patch, applies the symbolic DFT-6 add
//     network along rows and columns, forms the multiplication points, rounds
//     them to int8 (one fused multiply-add and one clamp per value) and drops the
//     bytes into LDS as out[tile][p][channel].
//  3. Copy out: each wave streams its tile's P x 64 bytes to V[p][t][c0..c0+63]
//     with 16-byte lanes.
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"

namespace sfc {

struct InputPlan {
  int S;        // strips per workgroup
  int chunks;   // tile-column chunks per strip
  int tlw;      // tile columns per chunk (<= 6)
  int wp;       // LDS bytes per staged row (multiple of 4, <= 64)
  int cs;       // LDS bytes per (strip, channel): 8*wp made an odd number of dwords
  unsigned lds_bytes;
};

template <int ALG>
__global__ __launch_bounds__(384, 2) void input_transform_i8_kernel(
    const int8_t* __restrict__ x, int8_t* __restrict__ V, const float* __restrict__ inv_sx,
    Geometry g, InputPlan ip) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int P = AlgTraits<ALG>::P;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;  // = S * tlw
  // Workgroups are dealt to the 8 XCDs round-robin by id; remap so that each XCD
  // (each L2) gets a contiguous range of (strip, chunk) items: neighbours share
  // halo rows and overlapping columns.
  const int bx = xcd_contiguous(blockIdx.x, gridDim.x);
  const int chunk = bx % ip.chunks;
  const int strip0 = (bx / ip.chunks) * ip.S;
  const int c0 = blockIdx.y * 64;
  const int tj0 = chunk * ip.tlw;
  const int colbase = (6 * tj0) & ~3;       // image column held at LDS byte 4 of a row
  const int halo = 6 * tj0 - 1 - colbase + 4;  // LDS byte of the chunk's first patch column
  const int W = g.W, H = g.H;

  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)x, 0, (int)((unsigned)(g.N * g.Cin) * (unsigned)(H * W)), kBufferFlags);

  // ---- 1. stage ---------------------------------------------------------------
  // One instruction covers four rows x 16 dwords of a (strip, channel): lane =
  // (row within the half, dword).  Everything that depends on the lane or the
  // strip is hoisted; per channel only a scalar plane offset changes.  A batch
  // of up to 16 channels per wave keeps up to 32 loads in flight before the first LDS
  // write.  Global dwords need not be aligned (W may be odd); a dword that
  // straddles the end of an image row is assembled from its valid bytes.
  {
    const int dpr = ip.wp >> 2;  // dwords per staged row, <= 16
    const int rsub = lane >> 4, dcol = lane & 15;
    const int col = colbase + 4 * dcol - 4;  // image column of this lane's dword
    const int nvalid = col < 0 ? 0 : min(4, max(0, W - col));
    const unsigned plane_stride = (unsigned)(H * W);
    constexpr int BATCH = 16;
    for (int s = 0; s < ip.S; ++s) {
      const int strip = strip0 + s;
      const bool strip_live = strip < g.strips;
      const int n = strip / g.th, ti = strip - n * g.th;
      bool ok[2];
      unsigned voff[2], loff[2];
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int h = 6 * ti - 1 + half * 4 + rsub;
        ok[half] = strip_live && dcol < dpr && h >= 0 && h < H && nvalid > 0;
        voff[half] = (unsigned)(h * W + col);
        loff[half] = (unsigned)(s * 64 * ip.cs + (half * 4 + rsub) * ip.wp + 4 * dcol);
      }
      const unsigned plane0 = (unsigned)(n * g.Cin + c0) * plane_stride;
      for (int cb = wave; cb < 64; cb += BATCH * nwaves) {
        unsigned vals[BATCH][2];
#pragma unroll
        for (int bi = 0; bi < BATCH; ++bi) {
          const int c = cb + bi * nwaves;
          const bool live = c < 64 && c0 + c < g.Cin;
          const unsigned plane = plane0 + (unsigned)c * plane_stride;
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            unsigned val = 0;
            if (live && ok[half]) {
              if (nvalid == 4) {
                val = __builtin_amdgcn_raw_buffer_load_b32(xres, voff[half], plane, 0);
              } else {
                for (int bb = 0; bb < nvalid; ++bb)
                  val |= (unsigned)__builtin_amdgcn_raw_buffer_load_b8(xres, voff[half] + bb, plane, 0)
                         << (8 * bb);
              }
            }
            vals[bi][half] = val;
          }
        }
#pragma unroll
        for (int bi = 0; bi < BATCH; ++bi) {
          const int c = cb + bi * nwaves;
          if (c < 64 && dcol < dpr) {
#pragma unroll
            for (int half = 0; half < 2; ++half)
              *(unsigned*)(lds + loff[half] + c * ip.cs) = vals[bi][half];
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- 2. transform -------------------------------------------------------------
  const int s = wave / ip.tlw, tjl = wave - s * ip.tlw;
  const int tj = tj0 + tjl;
  const int strip = strip0 + s;
  const bool tile_live = strip < g.strips && tj < g.tw;
  int comp[8][8];
  {
    const signed char* src = (const signed char*)lds + (s * 64 + lane) * ip.cs + halo + 6 * tjl;
    int half[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int row[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) row[j] = (int)src[i * ip.wp + j];
      fwd_input<8, 8>(row, half[i]);
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      int col[8], cc[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) col[i] = half[i][b];
      fwd_input<8, 8>(col, cc);
#pragma unroll
      for (int a = 0; a < 8; ++a) comp[a][b] = cc[a];
    }
  }
  __syncthreads();  // every patch is in registers: the staging area becomes the output area

  unsigned char* outp = lds + (unsigned)wave * (P * 64) + lane;
  constexpr float kMagic = 12582912.0f;  // 1.5 * 2^23: the sum's low mantissa bits are the integer
  for_each_point<ALG>(comp, [&](int p, int v) {
    float t = __fmaf_rn((float)v, inv_sx[p], kMagic);  // rounds the exact product, ties to even
    t = __builtin_amdgcn_fmed3f(t, kMagic - 127.0f, kMagic + 127.0f);
    outp[p * 64] = (unsigned char)__float_as_uint(t);
  });
  __syncthreads();

  // ---- 3. copy out ---------------------------------------------------------------
  if (tile_live) {
    const unsigned t = (unsigned)strip * g.tw + tj;
    const unsigned vplane = (unsigned)g.Tp * g.Cp;
    const __amdgpu_buffer_rsrc_t vres = __builtin_amdgcn_make_buffer_rsrc(
        (void*)V, 0, (int)(vplane * (unsigned)P), kBufferFlags);
    const unsigned lane_off = t * g.Cp + c0 + (lane & 3) * 16;
    const unsigned char* inp = lds + (unsigned)wave * (P * 64) + lane * 16;
#pragma unroll
    for (int it = 0; it < (P + 15) / 16; ++it) {
      const int p = it * 16 + (lane >> 2);
      if (p < P) {
        const v4i d = *(const v4i*)(inp + it * 1024);
        __builtin_amdgcn_raw_buffer_store_b128(d, vres, lane_off + p * vplane, 0, 0);
      }
    }
  }
}

static bool make_input_plan(const Geometry& g, InputPlan* ip) {
  if (g.alg > 1) return false;  // 6x6 tiles only
  ip->chunks = (g.tw + 5) / 6;
  ip->tlw = (g.tw + ip->chunks - 1) / ip->chunks;
  ip->S = ip->chunks > 1 ? 1 : (6 / ip->tlw > 0 ? 6 / ip->tlw : 1);
  if (ip->S > g.strips) ip->S = g.strips;
  // widest staged row: halo byte (3 or 5) + 6*tlw + 2 patch columns
  ip->wp = ((5 + 6 * ip->tlw + 2) + 3) / 4 * 4;
  int dw = 8 * ip->wp / 4;
  if ((dw & 1) == 0) dw += 1;
  ip->cs = 4 * dw;
  const unsigned in_bytes = (unsigned)ip->S * 64u * ip->cs;
  const unsigned out_bytes = (unsigned)ip->S * ip->tlw * g.P * 64u;
  ip->lds_bytes = in_bytes > out_bytes ? in_bytes : out_bytes;
  const long long xbytes = (long long)g.N * g.Cin * g.H * g.W;
  const long long vbytes = (long long)g.P * g.Tp * g.Cp;
  return ip->wp <= 64 && ip->S * ip->tlw <= 6 && ip->lds_bytes <= 64 * 1024 &&
         xbytes < (1ll << 31) && vbytes < (1ll << 31);
}

// Returns hipErrorNotSupported when the geometry is outside this kernel's limits;
// the caller then uses the generic kernel.
hipError_t launch_input_transform_i8(const Geometry& g, const int8_t* x, void* V,
                                     const float* inv_sx, hipStream_t s) {
  InputPlan ip;
  if (!make_input_plan(g, &ip)) return hipErrorNotSupported;
  dim3 grid(((g.strips + ip.S - 1) / ip.S) * ip.chunks, g.Cp / 64);
  dim3 block(64 * ip.S * ip.tlw);
  if (g.alg == 0)
    hipLaunchKernelGGL(input_transform_i8_kernel<0>, grid, block, ip.lds_bytes, s, x, (int8_t*)V,
                       inv_sx, g, ip);
  else
    hipLaunchKernelGGL(input_transform_i8_kernel<1>, grid, block, ip.lds_bytes, s, x, (int8_t*)V,
                       inv_sx, g, ip);
  return hipGetLastError();
}

}  // namespace sfc
