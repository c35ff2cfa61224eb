// Staged path, requantized mode (gfx950): the transform-domain products as P batched int8
// GEMMs on the matrix cores, and the output transform that reads their int32 sums back.
//
//   product_gemm_i8_kernel   M_p[tiles x Cout] = V_p[tiles x Cin] . U_p[Cout x Cin]^T  for
//                            every point p (the element-wise product of Eq. (1) summed over
//                            Cin), int8 MFMA 16x16x64 with int32 accumulation
//   output_sums_kernel       y = A^T M A with the correction terms, dequantization, NCHW store
//
// Layouts (element strides): V[p][t][c] = (p*Tp + t)*Cp + c, U[p][k][c] = (p*Kp + k)*Cp + c.
// M is kept in blocks of 16 tiles x 4 filters, M[p][t/16][k/4][t%16][k%4]: the 64 sums
// (256 contiguous bytes) that one wave of the output transform needs per point, and that
// a quarter wave of the GEMM holds in one accumulator register quad.
#include "sfc_device.hpp"
#include "sfc_internal.hpp"
#include "sfc_points.hpp"
#include "sfc_store.hpp"

namespace sfc {

// ---------------------------------------------------------------------------------------
// Batched GEMM.  A workgroup of four waves computes a 128-filter x 128-tile block of one
// point; each wave a 64 x 64 quarter as 4 x 4 MFMA blocks (A operand = filters, B operand =
// tiles, so that a lane ends up with four consecutive filters of one tile: 16 contiguous
// bytes of M).  Per 64-channel chunk the workgroup stages 128 x 64 bytes of U and of V in
// LDS through registers, the next chunk's loads in flight while the current one is
// multiplied.  LDS rows are 80 bytes apart: the 16 rows a quarter wave reads as one MFMA
// operand (16 bytes each) then fall into different banks.
// ---------------------------------------------------------------------------------------
constexpr int kGemmBlock = 128;  // filters and tiles per workgroup
constexpr int kGemmPitch = 80;   // LDS bytes per operand row (64 + padding)

__global__ __launch_bounds__(256) void product_gemm_i8_kernel(const int8_t* __restrict__ V,
                                                              const int8_t* __restrict__ U,
                                                              int32_t* __restrict__ M, Geometry g,
                                                              int nbt, int nbf, int stream_m,
                                                              int m_bytes) {
  constexpr int BL = kGemmBlock, PITCH = kGemmPitch;
  constexpr int TILE_BYTES = BL * PITCH;  // one staged operand
  __shared__ __align__(16) unsigned char lds[4 * TILE_BYTES];  // [buffer][U, V]
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1;  // quarter: filters 64*wm.., tiles 64*wn..
  // Workgroups that share an XCD (an L2) take consecutive positions, i.e. the blocks of the
  // same few points: V_p and U_p are then fetched from memory once per XCD.
  const int pos = xcd_contiguous(blockIdx.x, gridDim.x);
  const int per_point = nbt * nbf;
  const int p = pos / per_point, rem = pos - p * per_point;
  const int bt = rem / nbf, bf = rem - bt * nbf;
  const int KC = g.Cp >> 6;

  const __amdgpu_buffer_rsrc_t ures = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(U + (size_t)p * g.Kp * g.Cp), 0, g.Kp * g.Cp, kBufferFlags);
  const __amdgpu_buffer_rsrc_t vres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(V + (size_t)p * g.Tp * g.Cp), 0, g.Tp * g.Cp, kBufferFlags);

  // loader: piece q = tid + 256*i is 16 bytes of operand row q/4, segment q%4; rows beyond
  // the tensor get an offset outside the buffer (the load returns zero)
  constexpr unsigned kOutOfRange = 0x80000000u;
  unsigned usrc[2], vsrc[2], ldst[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int q = (int)threadIdx.x + 256 * i;
    const int row = q >> 2, seg = q & 3;
    const int k = bf * BL + row, t = bt * BL + row;
    usrc[i] = k < g.Kp ? (unsigned)(k * g.Cp + seg * 16) : kOutOfRange;
    vsrc[i] = t < g.Tp ? (unsigned)(t * g.Cp + seg * 16) : kOutOfRange;
    ldst[i] = (unsigned)(row * PITCH + seg * 16);
  }
  v4i ureg[2], vreg[2];
  auto load_regs = [&](int kc) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      ureg[i] = __builtin_amdgcn_raw_buffer_load_b128(ures, usrc[i], (unsigned)kc * 64u, 0);
      vreg[i] = __builtin_amdgcn_raw_buffer_load_b128(vres, vsrc[i], (unsigned)kc * 64u, 0);
    }
  };
  auto store_lds = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *(v4i*)(lds + (2 * buf) * TILE_BYTES + ldst[i]) = ureg[i];
      *(v4i*)(lds + (2 * buf + 1) * TILE_BYTES + ldst[i]) = vreg[i];
    }
  };

  v4i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = v4i{0, 0, 0, 0};

  const unsigned a_lane = (unsigned)((wm * 64 + (lane & 15)) * PITCH + (lane >> 4) * 16);
  const unsigned b_lane = (unsigned)((wn * 64 + (lane & 15)) * PITCH + (lane >> 4) * 16);

  load_regs(0);
  store_lds(0);
  __syncthreads();
  for (int kc = 0; kc < KC; ++kc) {
    const int buf = kc & 1;
    if (kc + 1 < KC) load_regs(kc + 1);
    v4i a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[i] = *(const v4i*)(lds + (2 * buf) * TILE_BYTES + a_lane + i * 16 * PITCH);
      b[i] = *(const v4i*)(lds + (2 * buf + 1) * TILE_BYTES + b_lane + i * 16 * PITCH);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    if (kc + 1 < KC) store_lds(buf ^ 1);
    __syncthreads();
  }

  // lane: filter quad (k0 + 16*i)/4 + lane/16, tile block (t0 + 16*j)/16, tile lane%16 of it:
  // the four sums of an accumulator are 16 contiguous bytes of M (12 when the sums are kept
  // in three bytes each, m_sum_bytes), a wave writes 1 KiB (768 bytes)
  const size_t plane = (size_t)g.Tp * g.Kp * (size_t)m_bytes;
  const __amdgpu_buffer_rsrc_t mres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)((unsigned char*)M + (size_t)p * plane), 0, (int)plane, kBufferFlags);
  const int k0 = bf * BL + wm * 64, t0 = bt * BL + wn * 64;
  const int kquads = g.Kp >> 2;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int tb = (t0 >> 4) + j;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int kq = ((k0 + 16 * i) >> 2) + (lane >> 4);
      if (tb * 16 < g.Tp && kq < kquads) {
        // a wave writes whole cache lines; stream_m: past the L2 ("nt")
        const unsigned elem = (unsigned)((tb * kquads + kq) * 64 + (lane & 15) * 4);
        const v4i a = acc[i][j];
        if (m_bytes == 3) {
          v3i d;
          d[0] = (int)__builtin_amdgcn_perm((unsigned)a[1], (unsigned)a[0], 0x04020100u);
          d[1] = (int)__builtin_amdgcn_perm((unsigned)a[2], (unsigned)a[1], 0x05040201u);
          d[2] = (int)__builtin_amdgcn_perm((unsigned)a[3], (unsigned)a[2], 0x06050402u);
          if (stream_m)
            __builtin_amdgcn_raw_buffer_store_b96(d, mres, elem * 3u, 0, kStreamStore);
          else
            __builtin_amdgcn_raw_buffer_store_b96(d, mres, elem * 3u, 0, 0);
        } else if (stream_m) {
          __builtin_amdgcn_raw_buffer_store_b128(a, mres, elem * 4u, 0, kStreamStore);
        } else {
          __builtin_amdgcn_raw_buffer_store_b128(a, mres, elem * 4u, 0, 0);
        }
      }
    }
  }
}

// Bytes per sum of M.  A sum of Cp products of operands within +-qmax is below 2^23 in
// magnitude when Cp qmax^2 < 2^23 (int8 operands: up to 512 channels); it is then stored as a
// little-endian 24-bit two's complement integer, which takes a quarter off the largest tensor
// of the staged path (512 channels on 7x7 maps, 256 images: M 69 -> 52 MB).
int m_sum_bytes(const Geometry& g) {
  return (double)g.Cp * (double)g.qmax * (double)g.qmax < 8388608.0 ? 3 : 4;
}

hipError_t launch_product_gemm_i8(const Geometry& g, const void* V, const void* U, int32_t* M,
                                  hipStream_t s) {
  const int nbt = (g.Tp + kGemmBlock - 1) / kGemmBlock, nbf = (g.Kp + kGemmBlock - 1) / kGemmBlock;
  const long long total = (long long)g.P * nbt * nbf;
  // 32-bit byte offsets inside one point's V, U and M
  if (total > 0x7fffffffll || (long long)g.Tp * g.Cp >= (1ll << 31) ||
      (long long)g.Kp * g.Cp >= (1ll << 31) || (long long)g.Tp * g.Kp * 4 >= (1ll << 31))
    return hipErrorNotSupported;
  // An M larger than the L2s together (8 x 4 MB; threshold 48 MB) is written with streaming
  // stores: the L2 then holds no dirty lines for the end of the kernel to write back (512
  // channels on 7x7 maps, 256 images, M = 69 MB: 23.4 instead of 27.6 us; the output
  // transform that follows reads M from memory either way once several batches are in flight).
  const int m_bytes = m_sum_bytes(g);
  const int stream_m = (long long)g.P * g.Tp * g.Kp * m_bytes > (48ll << 20) ? 1 : 0;
  hipLaunchKernelGGL(product_gemm_i8_kernel, dim3((unsigned)total), dim3(256), 0, s,
                     (const int8_t*)V, (const int8_t*)U, M, g, nbt, nbf, stream_m, m_bytes);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Output transform from M.  Wave w of a workgroup owns filters 4w..4w+3 of a 4*NW-filter
// group and 16 consecutive tiles, lane l the pair (tile l%16, filter 4w + l/16) -- the
// arrangement of the fused kernels, so the streaming output transform and the LDS-staged
// NCHW store are theirs.  The int32 sums of the pair are read point by point in
// processing order, a ring of loads ahead; no barrier, no LDS besides the store staging.
// The kernel moves M and y once each and runs at the rate the memory system delivers them.
// PLANES: whole tiles cover the feature map and the 16 tiles of a wave are whole images
// (whole_image_tiles); y is then written image by image (store_planes) from a staging
// block of M*M floats per pair.
// ---------------------------------------------------------------------------------------
// Points in flight per lane: 12 where a compute unit holds many waves; 32 for the forms
// whose partial outputs allow few (7x7 tiles, 5x5 and 7x7 filters: four-wave workgroups), so
// that the eight waves a compute unit has on a small layer keep some 64 KB of M on the way
// (512 channels on 7x7 maps, 256 images: the same 23 us either way when measured alone; the
// kernel there is bound by the bytes of M, see m_sum_bytes).
template <int ALG>
constexpr int sum_ring() { return AlgTraits<ALG>::NC <= 8 ? 12 : 32; }

template <int ALG, bool PLANES, int NW>
constexpr unsigned sums_stage_bytes() {
  return (unsigned)(NW * 64 * AlgTraits<ALG>::M * (PLANES ? AlgTraits<ALG>::M : 1) * 4);
}

template <int ALG, int OUT, bool VEC2, int NW, bool PLANES>
__global__ __launch_bounds__(NW * 64) void output_sums_kernel(const int32_t* __restrict__ M,
                                                              const float* __restrict__ dequant,
                                                              float x_scale, float inv_y,
                                                              void* __restrict__ y, Geometry g,
                                                              int m_bytes) {
  using Tr = AlgTraits<ALG>;
  constexpr int P = Tr::P, Mo = Tr::M, NC = Tr::NC, D = sum_ring<ALG>();
  constexpr Order<ALG> order{};
  extern __shared__ __align__(16) unsigned char lds[];  // staging blocks, then the tile table
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  float* stage = (float*)lds + wave * (64 * Mo * (PLANES ? Mo : 1));
  int* tile_tab = (int*)(lds + sums_stage_bytes<ALG, PLANES, NW>());
  const int t0 = blockIdx.x * 16;
  const int kq = blockIdx.y * NW + wave;
  const int kcol = kq * 4 + (lane >> 4);
  if (threadIdx.x < 16) {
    const int tl = threadIdx.x, t = t0 + tl;
    const int per = g.th * g.tw;
    const int n = t / per, rem = t - n * per;
    const int ti = rem / g.tw, tj = rem - ti * g.tw;
    write_tile_entry<Mo>(tile_tab, tl, t < g.T, n, ti, tj, g.Cout, g.H, g.W);
  }
  __syncthreads();

  // bytes of one point of M; three-byte sums are read as the low bytes of a dword (the last
  // one reaches a byte past the tensor, inside the 256-byte rounding of its buffer)
  const unsigned mplane = (unsigned)g.Tp * (unsigned)g.Kp * (unsigned)m_bytes;
  const unsigned msh = m_bytes == 3 ? 8u : 0u;
  const __amdgpu_buffer_rsrc_t mres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)M, 0, (int)(mplane * (unsigned)P + (4u - (unsigned)m_bytes)), kBufferFlags);
  const __amdgpu_buffer_rsrc_t dres = __builtin_amdgcn_make_buffer_rsrc(
      (void*)dequant, 0, Order<ALG>::PP * g.Kp * 4, kBufferFlags);
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(
      y, 0, (int)(esz * (unsigned)(g.N * g.Cout) * (unsigned)(g.H * g.W)), kBufferFlags);
  // filters beyond the padded count read nothing (zeros) and store nothing
  const bool kvalid = kcol < g.Kp;
  const unsigned m_lane =
      kvalid ? (unsigned)((blockIdx.x * (g.Kp >> 2) + kq) * 64 + (lane & 15) * 4 + (lane >> 4)) *
                   (unsigned)m_bytes
             : 0x80000000u;
  // dequantization factors: [filter][processing position], one 16-byte load per four points
  static_assert(D % 4 == 0, "the ring holds whole groups of four points");
  const unsigned d_lane = kvalid ? (unsigned)kcol * (unsigned)(Order<ALG>::PP * 4) : 0x80000000u;

  int mring[D];
  v4f dring[D / 4];
  auto load_point = [&](int j) {
    const unsigned p = (unsigned)order.pt[j];
    mring[j % D] = (int)__builtin_amdgcn_raw_buffer_load_b32(mres, m_lane, p * mplane, 0);
  };
  auto load_factors = [&](int grp) {  // positions 4*grp .. 4*grp + 3
    dring[grp % (D / 4)] = __builtin_bit_cast(
        v4f, __builtin_amdgcn_raw_buffer_load_b128(dres, d_lane, (unsigned)grp * 16u, 0));
  };
#pragma unroll
  for (int grp = 0; grp < D / 4 && 4 * grp < P; ++grp) load_factors(grp);
#pragma unroll
  for (int j = 0; j < D && j < P; ++j) load_point(j);
  int j = 0;  // folds to a constant after unrolling
  auto next = [&]() -> float {
    float v = (float)((mring[j % D] << msh) >> msh) * dring[(j >> 2) % (D / 4)][j & 3];
    asm volatile("" : "+v"(v));  // the slot is free from here on
    if (j + D < P) load_point(j + D);
    // the factor slot of a group is free once its fourth product has been taken
    if ((j & 3) == 3 && 4 * ((j >> 2) + D / 4) < P) load_factors((j >> 2) + D / 4);
    ++j;
    return v;
  };
  float z[NC][Mo];
  stream_vertical<ALG, float>(next, z);
  if constexpr (PLANES)
    store_planes<ALG, OUT>(z, stage, tile_tab, lane, kq, x_scale, inv_y, yres, g.Cout, g.th, g.tw);
  else
    store_pairs<ALG, OUT, VEC2>(z, stage, tile_tab, lane, kq, x_scale, inv_y, yres, g.Cout, g.H, g.W);
}

template <int ALG, int OUT, bool VEC2, bool PLANES = false>
static hipError_t launch_sums_impl(const Geometry& g, const int32_t* M, const FilterViews& f,
                                   float x_scale, float inv_y, void* y, hipStream_t s,
                                   bool prepare) {
  // the 7x7 forms carry 10x7 partial outputs per pair, the 5x5- and 7x7-filter forms 12x6 or
  // 12x4: they need the 256-register budget; four waves per workgroup, so that a small layer
  // still has several workgroups per compute unit, reading M and writing y out of phase (512
  // channels on 7x7 maps at batch 64, 7x7 tiles: staged path 38.9 us against 47.3 with eight).
  // The 6x6 forms (8x6 partial outputs) take eight waves: with sixteen, 128 registers, they spill.
  constexpr int NW = AlgTraits<ALG>::NC <= 6 ? 16 : AlgTraits<ALG>::NC <= 8 ? 8 : 4;
  constexpr unsigned lds_bytes = sums_stage_bytes<ALG, PLANES, NW>() + 256;
  static_assert(lds_bytes <= 160u * 1024u, "staging blocks exceed the LDS of a compute unit");
  auto kernel = output_sums_kernel<ALG, OUT, VEC2, NW, PLANES>;
  if (prepare)
    return lds_bytes > 64u * 1024u ? raise_lds_limit(reinterpret_cast<const void*>(kernel))
                                   : hipSuccess;
  const dim3 grid((unsigned)(g.Tp / 16), (unsigned)((g.Cout + 4 * NW - 1) / (4 * NW)));
  hipLaunchKernelGGL(kernel, grid, dim3(NW * 64), lds_bytes, s, M, f.dequant_single, x_scale,
                     inv_y, y, g, m_sum_bytes(g));
  return hipGetLastError();
}

template <int ALG>
static hipError_t launch_sums_alg(int out, const Geometry& g, const int32_t* M,
                                  const FilterViews& f, float x_scale, float inv_y, void* y,
                                  hipStream_t s, bool prepare) {
  constexpr bool kPairs = AlgTraits<ALG>::M % 2 == 0;
  // 7x7 tiles on 7x7, 14x14, 28x28 ... maps, 4x4 tiles on 4x4, 8x8, 16x16 ...: a wave's
  // pairs are whole planes of y
  if constexpr (AlgTraits<ALG>::M == 7 || AlgTraits<ALG>::M == 4) {
    if (whole_image_tiles(AlgTraits<ALG>::M, g.H, g.W, g.th, g.tw, g.Cout))
      return out == 2 ? launch_sums_impl<ALG, 2, false, true>(g, M, f, x_scale, inv_y, y, s, prepare)
                      : launch_sums_impl<ALG, 0, false, true>(g, M, f, x_scale, inv_y, y, s, prepare);
  }
  if constexpr (kPairs) {
    if (g.W % 2 == 0)
      return out == 2 ? launch_sums_impl<ALG, 2, true>(g, M, f, x_scale, inv_y, y, s, prepare)
                      : launch_sums_impl<ALG, 0, true>(g, M, f, x_scale, inv_y, y, s, prepare);
  }
  return out == 2 ? launch_sums_impl<ALG, 2, false>(g, M, f, x_scale, inv_y, y, s, prepare)
                  : launch_sums_impl<ALG, 0, false>(g, M, f, x_scale, inv_y, y, s, prepare);
}

// out: 0 float32, 2 int8 with ReLU.  hipErrorNotSupported beyond the 32-bit offset limits.
hipError_t launch_output_sums(int out, const Geometry& g, const int32_t* M, const FilterViews& f,
                              float x_scale, float inv_y, void* y, hipStream_t s, bool prepare) {
  const long long mbytes = 4ll * g.P * g.Tp * g.Kp, ybytes = 4ll * g.N * g.Cout * g.H * g.W;
  if (mbytes >= (1ll << 31) || ybytes >= (1ll << 31) || out == 1) return hipErrorNotSupported;
  switch (g.alg) {
    case 0: return launch_sums_alg<0>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 1: return launch_sums_alg<1>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 2: return launch_sums_alg<2>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 3: return launch_sums_alg<3>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 4: return launch_sums_alg<4>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 5: return launch_sums_alg<5>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 6: return launch_sums_alg<6>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 7: return launch_sums_alg<7>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 8: return launch_sums_alg<8>(out, g, M, f, x_scale, inv_y, y, s, prepare);
    case 9: return launch_sums_alg<9>(out, g, M, f, x_scale, inv_y, y, s, prepare);
  }
  return hipErrorInvalidValue;
}

}  // namespace sfc
