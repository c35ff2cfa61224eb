// Fused transform-domain product + output transform for SFC-6(6x6,3x3), gfx950.
//
// One wave owns a block of 16 tiles x 16 filters.  For every multiplication
// point it runs the int8 MFMA 16x16x64 over the input channels, scales the
// int32 sums by the point's dequantization factor and feeds them straight into
// the output transform, so the products M never leave the registers.
//
// Result layout of the 16x16 MFMA: lane l holds filter column l%16 of tile rows
// 4*(l/16)..+3.  A lane therefore owns four (tile, filter) pairs and the output
// transform is lane-local; the four pairs ride in a 4-vector so that the add
// networks of sfc_points.hpp are reused unchanged.
//
// Points are consumed grouped by their horizontal row class so that each group
// collapses at once (product rule post-additions, Hermitian recombination,
// inverse symbolic DFT along the vertical axis) into z[b][o1]; only z (8x6 values
// per pair) stays live.  The last step runs the inverse along the horizontal axis
// one output row at a time, stages the row block in LDS and stores it with
// contiguous lanes.
#include "sfc_internal.hpp"
#include "sfc_points.hpp"

namespace sfc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

template <>
struct Third<v4f> {
  static __device__ __forceinline__ v4f apply(v4f v) { return v * (1.0f / 3.0f); }
};

// canonical index of the kept nested point (r1, r2) in the 88-point order
__host__ __device__ constexpr int kept_index(int r1, int r2) {
  int n = 0;
  for (int a = 0; a < 10; ++a)
    for (int b = 0; b < 10; ++b) {
      if (row_is_complex(a) && row_is_complex(b)) continue;
      if (a == r1 && b == r2) return n;
      ++n;
    }
  return -1;
}

// Processing order (canonical point indices), grouped by horizontal class.
template <int ALG>
struct Order {
  static constexpr int P = AlgTraits<ALG>::P;
  int pt[P];
  constexpr Order() : pt{} {
    constexpr int real_rows[4] = {0, 7, 8, 9};
    int n = 0;
    // real columns: all ten vertical rows
    for (int j = 0; j < 4; ++j)
      for (int r1 = 0; r1 < 10; ++r1)
        pt[n++] = ALG == 1 ? 10 * r1 + real_rows[j] : kept_index(r1, real_rows[j]);
    // complex column groups
    for (int g2 = 0; g2 < 2; ++g2) {
      if (ALG == 1) {
        for (int r1 = 0; r1 < 10; ++r1)
          for (int i = 0; i < 3; ++i) pt[n++] = 10 * r1 + 1 + 3 * g2 + i;
      } else {
        for (int j = 0; j < 4; ++j)
          for (int i = 0; i < 3; ++i) pt[n++] = kept_index(real_rows[j], 1 + 3 * g2 + i);
        for (int g1 = 0; g1 < 2; ++g1)
          for (int i = 0; i < 6; ++i) pt[n++] = 64 + 6 * (2 * g1 + g2) + i;
      }
    }
  }
};

constexpr int kRing = 8;        // operand slots in flight (64-channel chunks)
constexpr int kStageStride = 98;  // floats per filter row of the staging block (16 tiles x 6 + 2)

template <int ALG, int KC>
__global__ __launch_bounds__(256) void fused_product_output_kernel(
    const int8_t* __restrict__ V, const int8_t* __restrict__ U, const float* __restrict__ dequant,
    float x_scale, float* __restrict__ y, Geometry g) {
  constexpr int P = AlgTraits<ALG>::P;
  constexpr Order<ALG> order{};
  constexpr int NS = P * KC;  // chunk steps

  __shared__ __align__(16) float stage[4][16 * kStageStride];
  __shared__ int tile_off[16];   // y offset of the tile's first output, -1: padding row
  __shared__ int tile_ext[16];   // valid rows | valid cols << 8

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int t0 = blockIdx.x * 16;
  const int kb = blockIdx.y * 4 + wave;
  const bool active = kb * 16 < g.Kp;
  const int k = kb * 16 + (lane & 15);

  if (threadIdx.x < 16) {
    const int t = t0 + threadIdx.x;
    int off = -1, ext = 0;
    if (t < g.T) {
      const int per = g.th * g.tw;
      const int n = t / per, rem = t - n * per;
      const int ti = rem / g.tw, tj = rem - ti * g.tw;
      off = ((n * g.Cout) * g.H + 6 * ti) * g.W + 6 * tj;
      const int rows = min(6, g.H - 6 * ti), cols = min(6, g.W - 6 * tj);
      ext = rows | (cols << 8);
    }
    tile_off[threadIdx.x] = off;
    tile_ext[threadIdx.x] = ext;
  }
  __syncthreads();

  const size_t vstride = (size_t)g.Tp * g.Cp;  // per point
  const size_t ustride = (size_t)g.Kp * g.Cp;
  const int8_t* a_base = V + (size_t)(t0 + (lane & 15)) * g.Cp + (lane >> 4) * 16;
  const int8_t* b_base = U + (size_t)(active ? k : 0) * g.Cp + (lane >> 4) * 16;
  const float* d_base = dequant + (active ? k : 0);

  v4i a[kRing], b[kRing];
  float dq[kRing];
  auto load_chunk = [&](int s) {  // s is a compile-time constant at every call site
    const int q = s / KC, kc = s % KC;
    const int p = order.pt[q];
    a[s % kRing] = *(const v4i*)(a_base + p * vstride + kc * 64);
    b[s % kRing] = *(const v4i*)(b_base + p * ustride + kc * 64);
    if (kc == 0) dq[q % kRing] = d_base[(size_t)p * g.Kp];
  };
#pragma unroll
  for (int s = 0; s < kRing && s < NS; ++s) load_chunk(s);

  int q = 0;  // folds to a constant: the code below is straight-line after unrolling
  v4i pending = {0, 0, 0, 0};
  float pending_d = 0.0f;
  auto issue = [&](int qq) {  // MFMA chain of point qq, refilling the ring behind it
    pending_d = dq[qq % kRing];  // read before the slot is refilled below
    v4i acc = {0, 0, 0, 0};
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int s = qq * KC + kc;
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s % kRing], b[s % kRing], acc, 0, 0, 0);
      if (s + kRing < NS) load_chunk(s + kRing);
    }
    pending = acc;
  };
  issue(0);
  // product of the next point in processing order, dequantized; overlaps the
  // following point's MFMA chain with the caller's additions
  auto next = [&]() -> v4f {
    const v4i acc = pending;
    const float d = pending_d;
    if (q + 1 < P) issue(q + 1);
    ++q;
    return v4f{(float)acc.x * d, (float)acc.y * d, (float)acc.z * d, (float)acc.w * d};
  };

  // z[b][o1]: horizontal component b, vertical output o1 (times 6)
  v4f z[8][6];
  constexpr int real_comp[4] = {0, 5, 6, 7};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    v4f col[10], cc[8];
#pragma unroll
    for (int r1 = 0; r1 < 10; ++r1) col[r1] = next();
    collapse10(col, cc);
    inv8(cc, z[real_comp[j]]);
  }
#pragma unroll
  for (int g2 = 0; g2 < 2; ++g2) {
    v4f c0[8], c1[8];  // components along the vertical axis for horizontal a0 / a1
    if constexpr (ALG == 1) {
      v4f h0[10], h1[10];
#pragma unroll
      for (int r1 = 0; r1 < 10; ++r1) {
        const v4f m0 = next(), m1 = next(), m2 = next();
        h0[r1] = m0 - m1;
        h1[r1] = m2 - m0;
      }
      collapse10(h0, c0);
      collapse10(h1, c1);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const v4f m0 = next(), m1 = next(), m2 = next();
        c0[real_comp[j]] = m0 - m1;
        c1[real_comp[j]] = m2 - m0;
      }
#pragma unroll
      for (int g1 = 0; g1 < 2; ++g1) {
        v4f m[6];
#pragma unroll
        for (int i = 0; i < 6; ++i) m[i] = next();
        // o[i][j]: i along the vertical axis (component a), j along the horizontal one
        hermitian_collapse(m, c0[1 + 2 * g1], c0[2 + 2 * g1], c1[1 + 2 * g1], c1[2 + 2 * g1]);
      }
    }
    inv8(c0, z[1 + 2 * g2]);
    inv8(c1, z[2 + 2 * g2]);
  }

  // ---- inverse along the horizontal axis, one output row per phase ----------
  float* st = stage[wave];
  const int wr_base = (lane & 15) * kStageStride + (lane >> 4) * 24;  // + j*6 + o2
#pragma unroll
  for (int o1 = 0; o1 < 6; ++o1) {
    v4f zc[8], out[6];
#pragma unroll
    for (int bb = 0; bb < 8; ++bb) zc[bb] = z[bb][o1];
    inv8(zc, out);
    if (active) {
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int o2 = 0; o2 < 6; o2 += 2) {
          v2f pr = {out[o2][j] * x_scale, out[o2 + 1][j] * x_scale};
          *(v2f*)(st + wr_base + j * 6 + o2) = pr;
        }
    }
    __syncthreads();
    if (active) {
      // 16 filters x 48 float pairs, lanes contiguous along (tile, o2)
#pragma unroll
      for (int i = 0; i < 12; ++i) {
        const int e = i * 64 + lane;
        const int kk = e / 48, r = e - kk * 48;
        const int tl = r / 3, o2 = 2 * (r - tl * 3);
        const int kcol = kb * 16 + kk;
        const int off = tile_off[tl], ext = tile_ext[tl];
        const v2f val = *(const v2f*)(st + kk * kStageStride + tl * 6 + o2);
        if (off >= 0 && kcol < g.Cout && o1 < (ext & 0xff)) {
          const int cols = ext >> 8;
          float* dst = y + (size_t)off + ((size_t)kcol * g.H + o1) * g.W + o2;
          if (o2 + 1 < cols) {
            if ((g.W & 1) == 0) {
              *(v2f*)dst = val;
            } else {
              dst[0] = val.x;
              dst[1] = val.y;
            }
          } else if (o2 < cols) {
            dst[0] = val.x;
          }
        }
      }
    }
    __syncthreads();
  }
}

template <int ALG>
static hipError_t launch_fused_alg(const Geometry& g, const void* V, const FilterViews& f,
                                   float x_scale, float* y, hipStream_t s) {
  const int kblocks = g.Kp / 16;
  dim3 grid(g.Tp / 16, (kblocks + 3) / 4);
  dim3 block(256);
  const int8_t* v = (const int8_t*)V;
  const int8_t* u = (const int8_t*)f.U;
  switch (g.Cp / 64) {
    case 1:
      hipLaunchKernelGGL((fused_product_output_kernel<ALG, 1>), grid, block, 0, s, v, u, f.dequant, x_scale, y, g);
      break;
    case 2:
      hipLaunchKernelGGL((fused_product_output_kernel<ALG, 2>), grid, block, 0, s, v, u, f.dequant, x_scale, y, g);
      break;
    case 4:
      hipLaunchKernelGGL((fused_product_output_kernel<ALG, 4>), grid, block, 0, s, v, u, f.dequant, x_scale, y, g);
      break;
    case 8:
      hipLaunchKernelGGL((fused_product_output_kernel<ALG, 8>), grid, block, 0, s, v, u, f.dequant, x_scale, y, g);
      break;
    default:
      return hipErrorNotSupported;
  }
  return hipGetLastError();
}

bool fused_supported(const Geometry& g) {
  const int kc = g.Cp / 64;
  // y offsets are kept in 32 bits inside the kernel
  const long long ysize = (long long)g.N * g.Cout * g.H * g.W;
  return (kc == 1 || kc == 2 || kc == 4 || kc == 8) && ysize < (1ll << 31);
}

hipError_t launch_fused_product_output(int alg, const Geometry& g, const void* V,
                                       const FilterViews& f, float x_scale, float* y,
                                       hipStream_t s) {
  if (!fused_supported(g)) return hipErrorNotSupported;
  return alg == 0 ? launch_fused_alg<0>(g, V, f, x_scale, y, s)
                  : launch_fused_alg<1>(g, V, f, x_scale, y, s);
}

}  // namespace sfc
