// HIP kernels of the staged path on gfx950 (wave64), every algorithm of sfc_points.hpp.
//
//   filter_transform_kernel   U = G f G^T               (once per layer)
//   input_transform_kernel    V = B^T x B               (NCHW int8 -> [P][Tp][Cp])
//   product_i16_kernel        M_p = V_p . U_p^T, exact mode (int16 operands, vector ALU)
//   output_transform_kernel   y = A^T M A, corrections, NCHW store, exact mode
// (the requantized-mode products and output transform are in sfc_gemm.hip)
//
// Layouts (element strides): V[p][t][c] = (p*Tp + t)*Cp + c, U[p][k][c] =
// (p*Kp + k)*Cp + c, M[p][t][k] = (p*Tp + t)*Kp + k.  Channels c >= Cin and
// filters k >= Cout are zero in U, so padding never contributes to a sum.
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"

namespace sfc {


// round-half-even(v * inv) clamped to [-qmax, qmax].  Adding 1.5 * 2^23 inside one
// fused multiply-add rounds the exact product once, to an integer, ties to even;
// the integer then sits in the low mantissa bits.
__device__ __forceinline__ int quantize_i8(int v, float inv, float qmax) {
  constexpr float kMagic = 12582912.0f;  // 0x4B400000
  float t = __fmaf_rn((float)v, inv, kMagic);
  t = fminf(fmaxf(t, kMagic - qmax), kMagic + qmax);
  return __float_as_int(t) - 0x4B400000;
}

// R x R filter taps of one (k, c) -> NC x NC components (rows, then columns)
template <int ALG>
__device__ __forceinline__ void filter_components(
    const int (&f)[AlgTraits<ALG>::R][AlgTraits<ALG>::R],
    int (&comp)[AlgTraits<ALG>::NC][AlgTraits<ALG>::NC]) {
  constexpr int NC = AlgTraits<ALG>::NC, R = AlgTraits<ALG>::R;
  int half[R][NC];
#pragma unroll
  for (int r = 0; r < R; ++r) fwd_filter<R, NC>(f[r], half[r]);
#pragma unroll
  for (int b = 0; b < NC; ++b) {
    int col[R];
#pragma unroll
    for (int r = 0; r < R; ++r) col[r] = half[r][b];
    int cc[NC];
    fwd_filter<R, NC>(col, cc);
#pragma unroll
    for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
  }
}

// ---------------------------------------------------------------------------
// filter transform: one thread per (k, c) of the padded [Kp][Cp] domain
// ---------------------------------------------------------------------------
template <int ALG, int MODE>
__global__ __launch_bounds__(256) void filter_transform_kernel(const int8_t* __restrict__ w,
                                                               void* __restrict__ U,
                                                               const float* __restrict__ inv_sw,
                                                               Geometry g) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  const int k = blockIdx.y;
  if (c >= g.Cp) return;
  constexpr int R = AlgTraits<ALG>::R;
  int f[R][R];
  const bool valid = (k < g.Cout) && (c < g.Cin);
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int s = 0; s < R; ++s)
      f[r][s] = valid ? (int)w[((size_t)k * g.Cin + c) * (R * R) + r * R + s] : 0;
  int comp[AlgTraits<ALG>::NC][AlgTraits<ALG>::NC];
  filter_components<ALG>(f, comp);
  for_each_point<ALG>(comp, [&](int p, int v) {
    const size_t idx = ((size_t)p * g.Kp + k) * g.Cp + c;
    if constexpr (MODE == 1) {
      ((int8_t*)U)[idx] = (int8_t)quantize_i8(v, inv_sw[p * g.Kp + k], g.qmax);
    } else {
      ((int16_t*)U)[idx] = (int16_t)v;
    }
  });
}

// abs-max over Cin of every transformed filter value: one block per k
template <int ALG>
__global__ __launch_bounds__(256) void filter_absmax_kernel(const int8_t* __restrict__ w,
                                                            int32_t* __restrict__ maxima,
                                                            Geometry g) {
  __shared__ int smax[AlgTraits<ALG>::P];
  const int k = blockIdx.x;
  for (int i = threadIdx.x; i < AlgTraits<ALG>::P; i += blockDim.x) smax[i] = 0;
  __syncthreads();
  for (int c = threadIdx.x; c < g.Cin; c += blockDim.x) {
    constexpr int R = AlgTraits<ALG>::R;
    int f[R][R];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int s = 0; s < R; ++s) f[r][s] = (int)w[((size_t)k * g.Cin + c) * (R * R) + r * R + s];
    int comp[AlgTraits<ALG>::NC][AlgTraits<ALG>::NC];
    filter_components<ALG>(f, comp);
    for_each_point<ALG>(comp, [&](int p, int v) { atomicMax(&smax[p], v < 0 ? -v : v); });
  }
  __syncthreads();
  for (int i = threadIdx.x; i < AlgTraits<ALG>::P; i += blockDim.x)
    maxima[(size_t)i * g.Cout + k] = smax[i];
}

// ---------------------------------------------------------------------------
// input transform
//
// One workgroup owns S consecutive strips (a strip = one row of tiles of one
// image, i.e. the NI = M+R-1 input rows from M*ti-PAD on) for 64 channels -- whole
// strips, or, when their rows do not fit in LDS (wide images), one chunk of tlw tile
// columns of them, staged byte by byte with its halo columns.  The whole input
// rows of a (strip, channel) are one contiguous run of NI*W bytes in NCHW, so the
// workgroup copies them to LDS with coalesced loads, then each thread transforms
// one (tile, channel) patch with lanes running along channels, which makes the
// V stores contiguous.  MODE: 0 int16 out, 1 int8 requantized out, 2 abs-max.
// ---------------------------------------------------------------------------
struct StripParams {
  int S;         // strips per workgroup
  int cs;        // LDS bytes per (strip, channel): NI*pitch padded to 4*(odd)
  int vec4;      // 1: whole rows with W % 4 == 0, staged as dwords
  int chunks;    // tile-column chunks per strip (1: whole rows)
  int tlw;       // tile columns per chunk
  int pitch;     // staged bytes per row: W, or M*tlw + 2*PAD for a chunk
};

template <int ALG, int MODE>
__global__ __launch_bounds__(256) void input_transform_kernel(const int8_t* __restrict__ x,
                                                              void* __restrict__ V,
                                                              const float* __restrict__ inv_sx,
                                                              int32_t* __restrict__ maxima,
                                                              Geometry g, StripParams sp) {
  extern __shared__ __align__(16) unsigned char lds[];
  constexpr int P = AlgTraits<ALG>::P, M = AlgTraits<ALG>::M, NI = AlgTraits<ALG>::NI,
                NC = AlgTraits<ALG>::NC, PAD = AlgTraits<ALG>::PAD;
  __shared__ int smax[MODE == 2 ? P : 1];
  if constexpr (MODE == 2) {
    for (int i = threadIdx.x; i < P; i += blockDim.x) smax[i] = 0;
  }
  const int strip0 = blockIdx.x * sp.S;
  const int c0 = blockIdx.y * 64;
  const int W = g.W, H = g.H;
  const int pitch = sp.pitch;
  const int seg = NI * pitch;  // bytes per (strip, channel)
  const int tjc0 = blockIdx.z * sp.tlw;                       // first tile column of the chunk
  const int colstart = sp.chunks > 1 ? M * tjc0 - PAD : 0;    // image column of staged byte 0

  // ---- stage the raw rows -------------------------------------------------
  if (sp.vec4) {
    const int segw = seg >> 2;
    const int total = sp.S * 64 * segw;
    for (int i = threadIdx.x; i < total; i += blockDim.x) {
      const int e = i % segw;
      const int sc = i / segw;
      const int c = sc & 63, s = sc >> 6;
      const int strip = strip0 + s;
      unsigned val = 0;
      if (strip < g.strips && c0 + c < g.Cin) {
        const int n = strip / g.th, ti = strip - n * g.th;
        const int row = (4 * e) / W;
        const int h = M * ti - PAD + row;
        if (h >= 0 && h < H) {
          const size_t base = (((size_t)n * g.Cin + c0 + c) * H + h) * W + (4 * e - row * W);
          val = *(const unsigned*)(x + base);
        }
      }
      *(unsigned*)(lds + (size_t)sc * sp.cs + 4 * e) = val;
    }
  } else {
    const int total = sp.S * 64 * seg;
    for (int i = threadIdx.x; i < total; i += blockDim.x) {
      const int e = i % seg;
      const int sc = i / seg;
      const int c = sc & 63, s = sc >> 6;
      const int strip = strip0 + s;
      unsigned char val = 0;
      if (strip < g.strips && c0 + c < g.Cin) {
        const int n = strip / g.th, ti = strip - n * g.th;
        const int row = e / pitch;
        const int h = M * ti - PAD + row;
        const int col = colstart + (e - row * pitch);
        if (h >= 0 && h < H && col >= 0 && col < W) {
          const size_t base = (((size_t)n * g.Cin + c0 + c) * H + h) * W + col;
          val = (unsigned char)x[base];
        }
      }
      lds[(size_t)sc * sp.cs + e] = val;
    }
  }
  __syncthreads();

  // ---- transform: item = (strip s, tile column tj, channel c), c fastest ----
  const int items = sp.S * sp.tlw * 64;
  for (int item = threadIdx.x; item < items; item += blockDim.x) {
    const int c = item & 63;
    const int rest = item >> 6;
    const int tj = tjc0 + rest % sp.tlw;
    const int s = rest / sp.tlw;
    const int strip = strip0 + s;
    if (strip >= g.strips || tj >= g.tw) continue;
    const signed char* src = (const signed char*)lds + (size_t)(s * 64 + c) * sp.cs;
    int half[NI][NC];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      int row[NI];
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int col = M * tj - PAD + j;
        row[j] = (col >= 0 && col < W) ? (int)src[i * pitch + col - colstart] : 0;
      }
      fwd_input<NI, NC>(row, half[i]);  // horizontal axis: half[i][b]
    }
    int comp[NC][NC];
#pragma unroll
    for (int b = 0; b < NC; ++b) {
      int col[NI], cc[NC];
#pragma unroll
      for (int i = 0; i < NI; ++i) col[i] = half[i][b];
      fwd_input<NI, NC>(col, cc);
#pragma unroll
      for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
    }
    const size_t t = (size_t)strip * g.tw + tj;
    const size_t row_off = t * g.Cp + c0 + c;
    const size_t pstride = (size_t)g.Tp * g.Cp;
    for_each_point<ALG>(comp, [&](int p, int v) {
      if constexpr (MODE == 1) {
        ((int8_t*)V)[p * pstride + row_off] = (int8_t)quantize_i8(v, inv_sx[p], g.qmax);
      } else if constexpr (MODE == 0) {
        ((int16_t*)V)[p * pstride + row_off] = (int16_t)v;
      } else {
        atomicMax(&smax[p], v < 0 ? -v : v);
      }
    });
  }
  if constexpr (MODE == 2) {
    __syncthreads();
    for (int i = threadIdx.x; i < P; i += blockDim.x)
      if (smax[i] > 0) atomicMax(&maxima[i], smax[i]);
  }
}

// plain streaming copy, 16 bytes per lane, grid-stride
__global__ __launch_bounds__(256) void stream_copy_kernel(const v4i* __restrict__ src,
                                                          v4i* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}

hipError_t launch_stream_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 16;
  size_t blocks = (n + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const v4i*)src,
                     (v4i*)dst, n);
  return hipGetLastError();
}

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// exact mode: int16 operands, int32 sums on the vector ALU, 16x16 block per workgroup
__global__ __launch_bounds__(256) void product_i16_kernel(const int16_t* __restrict__ V,
                                                          const int16_t* __restrict__ U,
                                                          int32_t* __restrict__ M, Geometry g) {
  __shared__ int16_t sv[16][66];
  __shared__ int16_t su[16][66];
  const int kblocks = g.Kp >> 4;
  const int kb = blockIdx.x % kblocks, tb = blockIdx.x / kblocks;
  const int p = blockIdx.y;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  unsigned acc = 0;  // sums modulo 2^32: wrap-around is defined, exact while the true sum fits
  for (int kc = 0; kc < g.Cp; kc += 64) {
    for (int i = threadIdx.x; i < 16 * 64; i += 256) {
      const int r = i >> 6, c = i & 63;
      sv[r][c] = V[((size_t)p * g.Tp + tb * 16 + r) * g.Cp + kc + c];
      su[r][c] = U[((size_t)p * g.Kp + kb * 16 + r) * g.Cp + kc + c];
    }
    __syncthreads();
#pragma unroll 16
    for (int c = 0; c < 64; ++c) acc += (unsigned)((int)sv[ty][c] * (int)su[tx][c]);
    __syncthreads();
  }
  M[((size_t)p * g.Tp + tb * 16 + ty) * g.Kp + kb * 16 + tx] = (int32_t)acc;
}

// ---------------------------------------------------------------------------
// output transform, exact mode: one thread per (tile, filter), lanes along filters;
// the integer sums are divided by 36 (16 for SFC-4) exactly
// ---------------------------------------------------------------------------
template <int ALG, int OUT>
__global__ __launch_bounds__(256) void output_transform_kernel(const int32_t* __restrict__ M,
                                                               const float* __restrict__ wscale,
                                                               float x_scale, void* __restrict__ y,
                                                               Geometry g, int kx) {
  const int k = blockIdx.y * kx + (threadIdx.x % kx);
  const int t = blockIdx.x * (256 / kx) + (threadIdx.x / kx);
  if (k >= g.Cout || t >= g.T) return;
  const size_t pstride = (size_t)g.Tp * g.Kp;
  const int32_t* m = M + (size_t)t * g.Kp + k;
  const int tiles_per_image = g.th * g.tw;
  const int n = t / tiles_per_image;
  const int rem = t - n * tiles_per_image;
  const int ti = rem / g.tw, tj = rem - ti * g.tw;
  const size_t ybase = ((size_t)n * g.Cout + k) * g.H * g.W;

  constexpr int MT = AlgTraits<ALG>::M;
  {
    // unsigned: the add network runs modulo 2^32 (the division by 3 of the Hermitian forms
    // is a multiplication by the inverse of 3), so only the final kDen-fold sums -- and, for
    // SFC-4, the sums it halves -- have to fit 32 bits
    unsigned out[MT][MT];
    output_transform<ALG, unsigned>([&](int p) { return (unsigned)m[p * pstride]; }, out);
    const float scale = x_scale * wscale[k];
#pragma unroll
    for (int o1 = 0; o1 < MT; ++o1) {
      const int h = MT * ti + o1;
      if (h >= g.H) continue;
#pragma unroll
      for (int o2 = 0; o2 < MT; ++o2) {
        const int w = MT * tj + o2;
        if (w >= g.W) continue;
        const int acc = (int)out[o1][o2] / AlgTraits<ALG>::kDen;  // exact: the sum is a multiple of it
        if constexpr (OUT == 1)
          ((int32_t*)y)[ybase + (size_t)h * g.W + w] = acc;
        else
          ((float*)y)[ybase + (size_t)h * g.W + w] = (float)acc * scale;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------

static StripParams strip_params(const Geometry& g) {
  StripParams sp;
  const int M = alg_tile(g.alg), PAD = (alg_taps(g.alg) - 1) / 2, NI = M + 2 * PAD;
  // odd dword stride between channels: lanes along channels hit distinct banks
  auto channel_bytes = [&](int pitch) {
    int seg4 = (NI * pitch + 3) / 4;
    if ((seg4 & 1) == 0) seg4 += 1;
    return 4 * seg4;
  };
  sp.chunks = 1;
  sp.tlw = g.tw;
  sp.pitch = g.W;
  sp.cs = channel_bytes(g.W);
  sp.vec4 = (g.W % 4 == 0) ? 1 : 0;
  if (64 * sp.cs > 64 * 1024) {
    // wide rows: chunks of tile columns with their halo, at most 48 KB per strip
    int tlw = g.tw;
    while (tlw > 1 && 64 * channel_bytes(M * tlw + 2 * PAD) > 48 * 1024) --tlw;
    sp.tlw = tlw;
    sp.chunks = (g.tw + tlw - 1) / tlw;
    sp.pitch = M * tlw + 2 * PAD;
    sp.cs = channel_bytes(sp.pitch);
    sp.vec4 = 0;
  }
  // aim at >= 256 (tile, channel) items and <= 32 KB of LDS per workgroup
  int S = 1;
  while (S < 16 && S * 2 * 64 * sp.cs <= 32 * 1024 && S * sp.tlw * 64 < 512) S *= 2;
  sp.S = S;
  return sp;
}

template <int ALG, int MODE>
static hipError_t launch_input_impl(const Geometry& g, const int8_t* x, void* V,
                                    const float* inv_sx, int32_t* maxima, hipStream_t s) {
  const StripParams sp = strip_params(g);
  const size_t lds = (size_t)sp.S * 64 * sp.cs;
  if (lds > 64 * 1024) return hipErrorInvalidValue;
  dim3 grid((g.strips + sp.S - 1) / sp.S, g.Cp / 64, sp.chunks);
  hipLaunchKernelGGL((input_transform_kernel<ALG, MODE>), grid, dim3(256), lds, s, x, V, inv_sx,
                     maxima, g, sp);
  return hipGetLastError();
}

template <int MODE>
static hipError_t launch_input_alg(const Geometry& g, const int8_t* x, void* V, const float* inv_sx,
                                   int32_t* maxima, hipStream_t s) {
  switch (g.alg) {
    case 0: return launch_input_impl<0, MODE>(g, x, V, inv_sx, maxima, s);
    case 1: return launch_input_impl<1, MODE>(g, x, V, inv_sx, maxima, s);
    case 2: return launch_input_impl<2, MODE>(g, x, V, inv_sx, maxima, s);
    case 3: return launch_input_impl<3, MODE>(g, x, V, inv_sx, maxima, s);
    case 4: return launch_input_impl<4, MODE>(g, x, V, inv_sx, maxima, s);
    case 5: return launch_input_impl<5, MODE>(g, x, V, inv_sx, maxima, s);
    case 6: return launch_input_impl<6, MODE>(g, x, V, inv_sx, maxima, s);
    case 7: return launch_input_impl<7, MODE>(g, x, V, inv_sx, maxima, s);
    case 8: return launch_input_impl<8, MODE>(g, x, V, inv_sx, maxima, s);
    case 9: return launch_input_impl<9, MODE>(g, x, V, inv_sx, maxima, s);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_input_transform(int mode, const Geometry& g, const int8_t* x, void* V,
                                  const float* inv_sx, const unsigned char* input_tab,
                                  hipStream_t s) {
  if (mode == 1) {
    const hipError_t e = launch_input_transform_i8(g, x, V, inv_sx, input_tab, s);
    if (e != hipErrorNotSupported) return e;
    return launch_input_alg<1>(g, x, V, inv_sx, nullptr, s);
  }
  return launch_input_alg<0>(g, x, V, inv_sx, nullptr, s);
}

hipError_t prepare_kernels(int path, int out, const Geometry& g) {
  const FilterViews none{};
  if (path == 2) {
    if (single16_supported(g)) return launch_single16(out, g, nullptr, none, 1.0f, 1.0f, nullptr, nullptr, true);
    if (single16k_supported(g)) return launch_single16k(out, g, nullptr, none, 1.0f, 1.0f, nullptr, nullptr, true);
    return launch_single_conv(out, g, nullptr, none, 1.0f, 1.0f, nullptr, nullptr, true);
  }
  // the generic input kernel (geometries the int8 one does not take) stays under 64 KB
  hipError_t e = launch_input_transform_i8(g, nullptr, nullptr, nullptr, nullptr, nullptr, true);
  if (e != hipSuccess && e != hipErrorNotSupported) return e;
  if (path == 1)
    return quad16_supported(g)   ? launch_quad16(out, g, nullptr, none, 1.0f, 1.0f, nullptr, nullptr, true)
           : splitk_supported(g) ? launch_splitk(out, g, nullptr, none, 1.0f, 1.0f, nullptr, nullptr, true)
                                 : launch_fused_quad(out, g, nullptr, none, 1.0f, 1.0f, nullptr, nullptr, true);
  return launch_output_sums(out, g, nullptr, none, 1.0f, 1.0f, nullptr, nullptr, true);
}

hipError_t launch_act_absmax(const Geometry& g, const int8_t* x, int32_t* maxima, hipStream_t s) {
  hipLaunchKernelGGL(fill_i32_kernel, dim3((g.P + 255) / 256), dim3(256), 0, s, maxima, g.P, 0);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_input_alg<2>(g, x, nullptr, nullptr, maxima, s);
}

hipError_t launch_filter_absmax(const Geometry& g, const int8_t* w, int32_t* maxima,
                                hipStream_t s) {
#define SFC_LAUNCH_FMAX(A) \
  hipLaunchKernelGGL(filter_absmax_kernel<A>, dim3(g.Cout), dim3(256), 0, s, w, maxima, g)
  switch (g.alg) {
    case 0: SFC_LAUNCH_FMAX(0); break;
    case 1: SFC_LAUNCH_FMAX(1); break;
    case 2: SFC_LAUNCH_FMAX(2); break;
    case 3: SFC_LAUNCH_FMAX(3); break;
    case 4: SFC_LAUNCH_FMAX(4); break;
    case 5: SFC_LAUNCH_FMAX(5); break;
    case 6: SFC_LAUNCH_FMAX(6); break;
    case 7: SFC_LAUNCH_FMAX(7); break;
    case 8: SFC_LAUNCH_FMAX(8); break;
    case 9: SFC_LAUNCH_FMAX(9); break;
    default: return hipErrorInvalidValue;
  }
#undef SFC_LAUNCH_FMAX
  return hipGetLastError();
}

hipError_t launch_filter_transform(int mode, const Geometry& g, const int8_t* w,
                                   const FilterViews& f, hipStream_t s) {
  dim3 grid((g.Cp + 255) / 256, g.Kp);
  dim3 block(256);
#define SFC_LAUNCH_FT(A)                                                                          \
  do {                                                                                            \
    if (mode == 1)                                                                                \
      hipLaunchKernelGGL((filter_transform_kernel<A, 1>), grid, block, 0, s, w, f.U, f.inv_sw, g); \
    else                                                                                          \
      hipLaunchKernelGGL((filter_transform_kernel<A, 0>), grid, block, 0, s, w, f.U, f.inv_sw, g); \
  } while (0)
  switch (g.alg) {
    case 0: SFC_LAUNCH_FT(0); break;
    case 1: SFC_LAUNCH_FT(1); break;
    case 2: SFC_LAUNCH_FT(2); break;
    case 3: SFC_LAUNCH_FT(3); break;
    case 4: SFC_LAUNCH_FT(4); break;
    case 5: SFC_LAUNCH_FT(5); break;
    case 6: SFC_LAUNCH_FT(6); break;
    case 7: SFC_LAUNCH_FT(7); break;
    case 8: SFC_LAUNCH_FT(8); break;
    case 9: SFC_LAUNCH_FT(9); break;
    default: return hipErrorInvalidValue;
  }
#undef SFC_LAUNCH_FT
  return hipGetLastError();
}

hipError_t launch_product(int mode, const Geometry& g, const void* V, const void* U, int32_t* M,
                          hipStream_t s) {
  const int blocks = (g.Tp / 16) * (g.Kp / 16);
  if (mode == 1) return launch_product_gemm_i8(g, V, U, M, s);
  hipLaunchKernelGGL(product_i16_kernel, dim3(blocks, g.P), dim3(256), 0, s, (const int16_t*)V,
                     (const int16_t*)U, M, g);
  return hipGetLastError();
}

template <int ALG>
static hipError_t launch_output_alg(int mode, int out, const Geometry& g, const int32_t* M,
                                    const FilterViews& f, float x_scale, float inv_y, void* y,
                                    hipStream_t s) {
  if (mode == 1) return launch_output_sums(out, g, M, f, x_scale, inv_y, y, s);
  int kx = 64;
  while (kx > g.Kp) kx >>= 1;  // Kp is a multiple of 16
  dim3 grid((g.T + (256 / kx) - 1) / (256 / kx), (g.Cout + kx - 1) / kx);
  dim3 block(256);
  if (out == 1)
    hipLaunchKernelGGL((output_transform_kernel<ALG, 1>), grid, block, 0, s, M, f.wscale, x_scale,
                       y, g, kx);
  else
    hipLaunchKernelGGL((output_transform_kernel<ALG, 0>), grid, block, 0, s, M, f.wscale, x_scale,
                       y, g, kx);
  return hipGetLastError();
}

hipError_t launch_output_transform(int mode, int out, const Geometry& g, const int32_t* M,
                                   const FilterViews& f, float x_scale, float inv_y, void* y,
                                   hipStream_t s) {
  switch (g.alg) {
    case 0: return launch_output_alg<0>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 1: return launch_output_alg<1>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 2: return launch_output_alg<2>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 3: return launch_output_alg<3>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 4: return launch_output_alg<4>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 5: return launch_output_alg<5>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 6: return launch_output_alg<6>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 7: return launch_output_alg<7>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 8: return launch_output_alg<8>(mode, out, g, M, f, x_scale, inv_y, y, s);
    case 9: return launch_output_alg<9>(mode, out, g, M, f, x_scale, inv_y, y, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
