// Output side shared by the fused kernels (gfx950): the per-tile store table and the
// store of one (tile, filter) pair per lane through a wave-private LDS block.
#pragma once
#include "sfc_device.hpp"
#include "sfc_points.hpp"

namespace sfc {

// Per-tile store data, 48 ints: [tile] output offset (elements) of the tile's first
// element for filter 0, [16 + tile] valid rows (0: no such tile), [32 + tile] valid columns.
template <int M>
__device__ __forceinline__ void write_tile_entry(int* tile_tab, int tl, bool live, int n, int ti,
                                                 int tj, int Cout, int H, int W) {
  tile_tab[tl] = ((n * Cout) * H + M * ti) * W + M * tj;
  tile_tab[16 + tl] = live ? min(M, H - M * ti) : 0;
  tile_tab[32 + tl] = min(M, W - M * tj);
}

// Lane l holds z (vertical outputs of every horizontal component, see stream_vertical)
// of the pair (tile l%16, filter 4*kq + l/16).  One output row at a time: the
// inverse along the horizontal axis, the wave's staging block [filter 0..3][tile
// 0..15][o2] (64*M floats), then stores in which consecutive lanes hold consecutive
// outputs of an image row (tiles of a strip are adjacent in y).
// OUT: 0 float32, 2 int8 with ReLU (inv_y = 1 / output scale).  VEC2: M and W even,
// pairs of outputs stay aligned.
template <int ALG, int OUT, bool VEC2>
__device__ __forceinline__ void store_pairs(
    const float (&z)[AlgTraits<ALG>::NC][AlgTraits<ALG>::M], float* stage, const int* tile_tab,
    int lane, int kq, float x_scale, float inv_y, __amdgpu_buffer_rsrc_t yres, int Cout, int H,
    int W) {
  constexpr int M = AlgTraits<ALG>::M;
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  // Cache policy of the y stores.  7x7 and 4x4 tiles divide the ResNet image widths; on wide
  // images a workgroup then writes long whole rows and the lines can stream past the L2
  // ("nt"): nothing is left dirty in the L2 for the end of the kernel to write back, which
  // shortened a 4x4 single kernel on 56x56 maps from 19.6 to 17.0 us.  Everywhere else (6x6
  // tiles, or short rows of small feature maps, where a line is completed by several stores
  // or several workgroups) the L2 has to merge the pieces before they go to memory:
  // streaming those costs up to 2.5x the bytes in HBM writes.
  const bool stream = (M == 7 || M == 4) && W >= 48;
  constexpr int EV = VEC2 ? 2 : 1;        // elements per lane and store
  constexpr int NST = (M + EV - 1) / EV;  // stores per lane and output row (64*M elements)
  // store plan: the k-th store of this lane covers elements e = EV*(lane + 64*k) of the
  // staged row block, e = (filter*16 + tile)*M + o2
  unsigned yoff[NST];
  int rowlim[NST];
#pragma unroll
  for (int k = 0; k < NST; ++k) {
    const unsigned e = (unsigned)(EV * (lane + 64 * k));
    const unsigned ft = e / (unsigned)M;  // filter*16 + tile
    const int o2 = (int)(e - ft * M), f = (int)(ft >> 4), tl = (int)(ft & 15);
    const int kc = kq * 4 + f;
    const bool valid = e < 64u * M && kc < Cout && o2 < tile_tab[32 + tl];
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
          if constexpr (VEC2) {
            const unsigned short q = (unsigned short)(q0 | (q1 << 8));
            if (stream) __builtin_amdgcn_raw_buffer_store_b16(q, yres, yoff[k], yrow, kStreamStore);
            else __builtin_amdgcn_raw_buffer_store_b16(q, yres, yoff[k], yrow, 0);
          } else {
            if (stream) __builtin_amdgcn_raw_buffer_store_b8((unsigned char)q0, yres, yoff[k], yrow, kStreamStore);
            else __builtin_amdgcn_raw_buffer_store_b8((unsigned char)q0, yres, yoff[k], yrow, 0);
          }
        } else {
          if constexpr (VEC2) {
            if (stream) __builtin_amdgcn_raw_buffer_store_b64(v2f{v0, v1}, yres, yoff[k], yrow, kStreamStore);
            else __builtin_amdgcn_raw_buffer_store_b64(v2f{v0, v1}, yres, yoff[k], yrow, 0);
          } else {
            if (stream) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v0), yres, yoff[k], yrow, kStreamStore);
            else __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v0), yres, yoff[k], yrow, 0);
          }
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

// The same for feature maps that whole tiles cover exactly (H = M*th, W = M*tw) with th*tw
// a divisor of 16: the 16 tiles of a wave are then 16/(th*tw) whole images, and the four
// filter planes of an image are one run of 4*H*W elements of y.  The wave stages all M rows
// of its 64 pairs as [image][filter][row][column], the order of y, and writes them with four
// elements per lane, 1 KB of consecutive addresses per store instruction.  Row-by-row stores
// put a 128-byte line together from pieces of 4*M bytes issued M row transforms apart, and
// the L2 wrote such lines to memory about twice (WRITE_SIZE 45.8 MB for 25.7 MB of y on 7x7
// maps).  Used by the 7x7 and the 4x4 forms.  Needs Cout % 4 == 0 (runs stay 16-byte aligned)
// and a staging block of 64*M*M floats per wave.  The float32 runs go out as streaming stores: nothing stays dirty in
// the L2 for the end of the kernel (output transform from M on 7x7 maps 25.3 instead of
// 27.1 us, fused kernel on 14x14 maps 40.5 instead of 42.3 us).
inline bool whole_image_tiles(int M, int H, int W, int th, int tw, int Cout) {
  const int per = th * tw;
  return H == M * th && W == M * tw && per <= 16 && 16 % per == 0 && Cout % 4 == 0;
}

template <int ALG, int OUT>
__device__ __forceinline__ void store_planes(
    const float (&z)[AlgTraits<ALG>::NC][AlgTraits<ALG>::M], float* stage, const int* tile_tab,
    int lane, int kq, float x_scale, float inv_y, __amdgpu_buffer_rsrc_t yres, int Cout, int th,
    int tw) {
  constexpr int M = AlgTraits<ALG>::M, MM = M * M;
  constexpr unsigned esz = OUT == 2 ? 1u : 4u;
  const int per = th * tw, W = M * tw, HW = per * MM;
  {
    const int tl = lane & 15, f = lane >> 4;
    const int il = tl / per, rem = tl - il * per;  // image of the wave, tile of the image
    const int ti = rem / tw, tj = rem - ti * tw;
    float* wr = stage + (il * 4 + f) * HW + (M * ti) * W + M * tj;
#pragma unroll
    for (int o1 = 0; o1 < M; ++o1) {
      float out[M];
      stream_row<ALG, float>(z, o1, out);
      if constexpr (M % 4 == 0) {  // rows of whole 16-byte groups
#pragma unroll
        for (int o2 = 0; o2 < M; o2 += 4)
          *(v4f*)(wr + o1 * W + o2) = v4f{out[o2] * x_scale, out[o2 + 1] * x_scale,
                                          out[o2 + 2] * x_scale, out[o2 + 3] * x_scale};
      } else {
#pragma unroll
        for (int o2 = 0; o2 < M; ++o2) wr[o1 * W + o2] = out[o2] * x_scale;
      }
    }
  }
  __builtin_amdgcn_wave_barrier();  // LDS accesses of one wave complete in order
  constexpr int NQ = 16 * MM;       // groups of four elements in the wave's block
  const bool kvalid = 4 * kq < Cout;
#pragma unroll
  for (int k = 0; k < (NQ + 63) / 64; ++k) {
    const int q = lane + 64 * k;
    if (q < NQ) {
      const int il = q / HW, r = q - il * HW;  // image, group within its four planes
      const v4f v = *(const v4f*)(stage + 4 * q);
      if (kvalid && tile_tab[16 + il * per] > 0) {
        const unsigned off = esz * (unsigned)(tile_tab[il * per] + 4 * kq * HW + 4 * r);
        if constexpr (OUT == 2) {
          // next layer's activation: ReLU, round half to even, clamp to [0, 127]
          constexpr float kMagic = 12582912.0f;
          unsigned word = 0;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float t = __fmaf_rn(v[i], inv_y, kMagic);
            t = __builtin_amdgcn_fmed3f(t, kMagic, kMagic + 127.0f);
            word |= (__float_as_uint(t) & 0xffu) << (8 * i);
          }
          __builtin_amdgcn_raw_buffer_store_b32(word, yres, off, 0, 0);
        } else {
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4i, v), yres, off, 0, kStreamStore);
        }
      }
    }
  }
}

}  // namespace sfc
