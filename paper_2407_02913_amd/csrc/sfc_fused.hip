// Fused transform-domain product + output transform for SFC-6(6x6,3x3), gfx950.
//
// A workgroup of four waves owns a block of 16 tiles x 16 filters.  For every
// multiplication point one of its waves runs the int8 MFMA 16x16x64 over the input
// channels and scales the int32 sums by the point's dequantization factor; the
// products M go through LDS to the thread that owns the (tile, filter) pair and
// straight into the output transform, so M never reaches HBM.
//
// Result layout of the 16x16 MFMA: lane l holds filter column l%16 of tile rows
// 4*(l/16)..+3; written as one 16-byte LDS store per lane, pair (t, k) sits at
// float ((t/4)*16 + k)*4 + t%4.
//
// Points are consumed grouped by their horizontal row class so that each group
// collapses at once (product rule post-additions, Hermitian recombination,
// inverse symbolic DFT along the vertical axis) into z[b][o1]; only z (8x6 values
// per pair) stays live.  The last step runs the inverse along the horizontal axis
// one output row at a time, stages the row block in LDS and stores it with
// contiguous lanes (consecutive tiles of a strip form full image rows).
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"

namespace sfc {


constexpr int kRing = 4;          // operand slots in flight (64-channel chunks)
constexpr int kStageStride = 98;  // floats per filter row of the staging block (16 tiles x 6 + 2)

// ---------------------------------------------------------------------------
// Points are handled in rounds of PPR; in a round every wave runs
// the MFMA chains of PPR/4 points, scales the sums and leaves them in LDS in the
// MFMA's own layout; after one barrier every thread reads the PPR values of its
// single (tile, filter) pair and feeds the output transform.  One pair per thread
// keeps the register count low enough for four waves per SIMD.  Nothing in the
// prologue waits on global memory: operands and dequantization factors stream
// through a register ring that is filled before the first barrier.
// ---------------------------------------------------------------------------
// VEC2: W is even, so float pairs (or byte pairs) of an output row stay aligned.
// OUT8: write the next layer's int8 activations (ReLU, round, clamp) instead of float32.
template <int ALG, int KC, bool VEC2, bool OUT8>
__global__ __launch_bounds__(256, 4) void fused_product_output_kernel(
    const int8_t* __restrict__ V, const int8_t* __restrict__ U, const float* __restrict__ dequant,
    float x_scale, float inv_y, void* __restrict__ y, Geometry g) {
  constexpr int P = AlgTraits<ALG>::P;
  constexpr Order<ALG> order{};
  constexpr int PPR = (P % 8 == 0) ? 8 : 4;  // points per round
  constexpr int PW = PPR / 4;                // points per wave and round
  constexpr int ROUNDS = P / PPR;
  constexpr int NJ = P / 4;                  // points of one wave
  constexpr int NS = NJ * KC;                // chunk steps of one wave

  __shared__ __align__(16) float mx[2][PPR][256];  // [buffer][point of the round][MFMA layout]
  __shared__ __align__(16) float stage[2][16 * kStageStride];
  __shared__ int tile_off[16];
  __shared__ int tile_ext[16];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int t0 = blockIdx.x * 16;
  const int kb = blockIdx.y;
  const int kcol = kb * 16 + (lane & 15);  // < Kp

  if (threadIdx.x < 16) {
    const int t = t0 + threadIdx.x;
    int off = 0, ext = 0;
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

  const unsigned vstride = (unsigned)g.Tp * g.Cp;
  const unsigned ustride = (unsigned)g.Kp * g.Cp;
  const unsigned aoff = (unsigned)(t0 + (lane & 15)) * g.Cp + (lane >> 4) * 16;
  const unsigned boff = (unsigned)kcol * g.Cp + (lane >> 4) * 16;
  const __amdgpu_buffer_rsrc_t vres =
      __builtin_amdgcn_make_buffer_rsrc((void*)V, 0, (int)(vstride * (unsigned)P), kBufferFlags);
  const __amdgpu_buffer_rsrc_t ures =
      __builtin_amdgcn_make_buffer_rsrc((void*)U, 0, (int)(ustride * (unsigned)P), kBufferFlags);
  const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)dequant, 0, (int)(4u * (unsigned)P * (unsigned)g.Kp), kBufferFlags);

  // This wave's j-th point is the (4j + wave)-th of the processing order: one of
  // four compile-time constants chosen by the uniform wave index, so the plane
  // offsets stay scalar.  Chunk step s = j*KC + kc.
  auto point_of = [&](int j) {
    const int p0 = order.pt[4 * j], p1 = order.pt[4 * j + 1], p2 = order.pt[4 * j + 2],
              p3 = order.pt[4 * j + 3];
    return wave_u == 0 ? p0 : wave_u == 1 ? p1 : wave_u == 2 ? p2 : p3;
  };
  v4i a[kRing], b[kRing];
  float dq[kRing];
  auto load_chunk = [&](int s) {
    const int j = s / KC, kc = s % KC;
    const int p = point_of(j);
    a[s % kRing] = __builtin_amdgcn_raw_buffer_load_b128(vres, aoff, p * vstride + kc * 64, 0);
    b[s % kRing] = __builtin_amdgcn_raw_buffer_load_b128(ures, boff, p * ustride + kc * 64, 0);
    if (kc == 0)
      dq[j % kRing] = __builtin_bit_cast(
          float, __builtin_amdgcn_raw_buffer_load_b32(dres, 4u * (unsigned)kcol, 4u * (unsigned)(p * g.Kp), 0));
  };
#pragma unroll
  for (int s = 0; s < kRing && s < NS; ++s) load_chunk(s);

  // MFMA chain of this wave's point j, already scaled (the factor is read before
  // its ring slot is refilled)
  auto product = [&](int j) -> v4f {
    const float d = dq[j % kRing];
    v4i acc = {0, 0, 0, 0};
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int s = j * KC + kc;
      acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[s % kRing], b[s % kRing], acc, 0, 0, 0);
      if (s + kRing < NS) load_chunk(s + kRing);
    }
    return v4f{(float)acc.x * d, (float)acc.y * d, (float)acc.z * d, (float)acc.w * d};
  };
  // round r: this wave's points j = r*PW .. r*PW + PW-1 land in slots 4*(j % PW) + wave
  auto publish_round = [&](int r) {
#pragma unroll
    for (int i = 0; i < PW; ++i)
      *(v4f*)(&mx[r & 1][4 * i + wave][lane * 4]) = product(r * PW + i);
  };

  publish_round(0);
  __syncthreads();

  // consumer side: this thread's pair is tile row 4*wave + lane/16, filter lane%16
  const int rd_idx = (wave * 16 + (lane & 15)) * 4 + (lane >> 4);
  int q = 0;  // folds to a constant
  float cur[PPR];
  auto next = [&]() -> float {
    const int r = q / PPR, i = q % PPR;
    if (i == 0) {
#pragma unroll
      for (int j = 0; j < PPR; ++j) cur[j] = mx[r & 1][j][rd_idx];
      if (r + 1 < ROUNDS) publish_round(r + 1);
    }
    const float v = cur[i];
    if (i == PPR - 1) __syncthreads();
    ++q;
    return v;
  };

  float z[8][6];
  stream_vertical<ALG, float>(next, z);

  // ---- store plan, fixed over the six output rows --------------------------------
  // float32: 16 filters x 48 float pairs (or 96 floats) over 256 threads, lanes
  // contiguous along (tile, o2).  int8: one (filter, tile) row of six bytes per thread.
  constexpr int SLOTS = OUT8 ? 1 : (VEC2 ? 3 : 6);
  unsigned yo[SLOTS];
  int rows[SLOTS];
  int rd[SLOTS];
  int cols8 = 0;
  const unsigned esz = OUT8 ? 1u : 4u;
#pragma unroll
  for (int i = 0; i < SLOTS; ++i) {
    const int e = i * 256 + threadIdx.x;
    constexpr int per_k = OUT8 ? 16 : (VEC2 ? 48 : 96), per_t = OUT8 ? 1 : (VEC2 ? 3 : 6),
                  step = VEC2 ? 2 : 1;
    const int kk = e / per_k, r = e - kk * per_k;
    const int tl = r / per_t, o2 = OUT8 ? 0 : step * (r - tl * per_t);
    const int kc2 = kb * 16 + kk;
    const int ext = tile_ext[tl];
    const bool ok = kc2 < g.Cout && o2 < (ext >> 8);
    rows[i] = ok ? (ext & 0xff) : 0;
    yo[i] = esz * ((unsigned)tile_off[tl] + (unsigned)(kc2 * g.H) * g.W + o2);
    rd[i] = kk * kStageStride + tl * 6 + o2;
    if constexpr (OUT8) cols8 = ext >> 8;
  }
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      y, 0, (int)(esz * (unsigned)(g.N * g.Cout) * (unsigned)(g.H * g.W)), kBufferFlags);
  const int wr_base = (lane & 15) * kStageStride + (4 * wave + (lane >> 4)) * 6;
  // one barrier per output row: the staging block is double buffered
#pragma unroll
  for (int o1 = 0; o1 < 6; ++o1) {
    float out[6];
    stream_row<ALG, float>(z, o1, out);
    float* st = stage[o1 & 1];
#pragma unroll
    for (int o2 = 0; o2 < 6; o2 += 2) {
      v2f pr = {out[o2] * x_scale, out[o2 + 1] * x_scale};
      *(v2f*)(st + wr_base + o2) = pr;
    }
    __syncthreads();
    const unsigned yrow = esz * (unsigned)(o1 * g.W);
    if constexpr (OUT8) {
      // ReLU + round-half-even + clamp to [0, 127]: adding 1.5 * 2^23 in one fused
      // multiply-add leaves the integer in the low mantissa bits
      constexpr float kMagic = 12582912.0f;
      unsigned q[6];
#pragma unroll
      for (int o2 = 0; o2 < 6; ++o2) {
        float t = __fmaf_rn(st[rd[0] + o2], inv_y, kMagic);
        t = __builtin_amdgcn_fmed3f(t, kMagic, kMagic + 127.0f);
        q[o2] = __float_as_uint(t) & 0xffu;
      }
      if (o1 < rows[0]) {
#pragma unroll
        for (int o2 = 0; o2 < 6; o2 += 2) {
          if constexpr (VEC2) {
            if (o2 < cols8)
              __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(q[o2] | (q[o2 + 1] << 8)), yres,
                                                    yo[0] + o2, yrow, kStreamStore);
          } else {
            if (o2 < cols8)
              __builtin_amdgcn_raw_buffer_store_b8((unsigned char)q[o2], yres, yo[0] + o2, yrow,
                                                   kStreamStore);
            if (o2 + 1 < cols8)
              __builtin_amdgcn_raw_buffer_store_b8((unsigned char)q[o2 + 1], yres, yo[0] + o2 + 1,
                                                   yrow, kStreamStore);
          }
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < SLOTS; ++i) {
        if constexpr (VEC2) {
          const v2f val = *(const v2f*)(st + rd[i]);
          if (o1 < rows[i]) __builtin_amdgcn_raw_buffer_store_b64(val, yres, yo[i], yrow, kStreamStore);
        } else {
          const float val = st[rd[i]];
          if (o1 < rows[i])
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(val), yres, yo[i], yrow, kStreamStore);
        }
      }
    }
  }
}

template <int ALG, bool VEC2, bool OUT8>
static hipError_t launch_fused_alg(const Geometry& g, const void* V, const FilterViews& f,
                                   float x_scale, float inv_y, void* y, hipStream_t s) {
  const int kblocks = g.Kp / 16;
  dim3 grid(g.Tp / 16, kblocks);
  dim3 block(256);
  const int8_t* v = (const int8_t*)V;
  const int8_t* u = (const int8_t*)f.U;
#define SFC_LAUNCH_FUSED(KC)                                                                  \
  hipLaunchKernelGGL((fused_product_output_kernel<ALG, KC, VEC2, OUT8>), grid, block, 0, s, v, \
                     u, f.dequant, x_scale, inv_y, y, g)
  switch (g.Cp / 64) {
    case 1: SFC_LAUNCH_FUSED(1); break;
    case 2: SFC_LAUNCH_FUSED(2); break;
    case 4: SFC_LAUNCH_FUSED(4); break;
    case 8: SFC_LAUNCH_FUSED(8); break;
    default: return hipErrorNotSupported;
  }
#undef SFC_LAUNCH_FUSED
  return hipGetLastError();
}

bool fused_supported(const Geometry& g) {
  if (g.alg > 1) return false;  // 6x6 tiles only
  const int kc = g.Cp / 64;
  // V, U and y are addressed through buffer descriptors with 32-bit byte offsets
  const long long ybytes = 4ll * g.N * g.Cout * g.H * g.W;
  const long long vbytes = (long long)g.P * g.Tp * g.Cp, ubytes = (long long)g.P * g.Kp * g.Cp;
  const long long lim = 1ll << 31;
  return (kc == 1 || kc == 2 || kc == 4 || kc == 8) && ybytes < lim && vbytes < lim && ubytes < lim;
}

template <int ALG>
static hipError_t launch_fused_out(int out, const Geometry& g, const void* V, const FilterViews& f,
                                   float x_scale, float inv_y, void* y, hipStream_t s) {
  const bool vec2 = (g.W % 2) == 0;  // pairs of an output row stay aligned in y
  if (out == 2)
    return vec2 ? launch_fused_alg<ALG, true, true>(g, V, f, x_scale, inv_y, y, s)
                : launch_fused_alg<ALG, false, true>(g, V, f, x_scale, inv_y, y, s);
  return vec2 ? launch_fused_alg<ALG, true, false>(g, V, f, x_scale, inv_y, y, s)
              : launch_fused_alg<ALG, false, false>(g, V, f, x_scale, inv_y, y, s);
}

hipError_t launch_fused_product_output(int out, const Geometry& g, const void* V,
                                       const FilterViews& f, float x_scale, float inv_y, void* y,
                                       hipStream_t s) {
  if (!fused_supported(g) || out == 1) return hipErrorNotSupported;
  return g.alg == 0 ? launch_fused_out<0>(out, g, V, f, x_scale, inv_y, y, s)
                  : launch_fused_out<1>(out, g, V, f, x_scale, inv_y, y, s);
}

}  // namespace sfc
