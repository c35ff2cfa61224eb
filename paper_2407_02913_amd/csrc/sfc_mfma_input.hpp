// Input-tile transform of the SFC-4(4x4,3x3) forms on the matrix cores (gfx950).
//
// V = B^T x B of a 6 x 6 patch is 46 / 49 sums of patch samples with coefficients 0, +1, -1
// (the four-point symbolic DFT with its correction rows, Appendix A).  On the vector ALU that
// is 110 additions per (tile, channel) plus a conversion per point; here the same sums are
// taken by int8 MFMA 16x16x64 instructions: operand A holds the patches of 16 channels (row =
// channel; the 64 k-bytes are the patch rows of 8 bytes each, k = 8 i + j, of which j < 6 and
// i < 6 carry samples), operand B the coefficients of 16 multiplication points (column = point
// in processing order).  The coefficient table is produced on the host by running the add
// networks of sfc_points.hpp on unit patches, so both forms compute the same integers.  Lane l
// ends with the sums of channels 4(l/16) .. 4(l/16)+3 for point l%16 of the block: after
// rounding, four bytes that go to V as one dword.
#pragma once
#include "sfc_device.hpp"
#include "sfc_points.hpp"

namespace sfc {

constexpr int kInputTabRows = 64;  // positions padded to whole blocks of 16
// the table behind the filter operand: float inv_pos[64] (1 / s_Tx by processing position, 0
// for positions without a point), then int8 coeff[64][64] ([position][k]), then int
// point[64] (canonical point of a processing position, -1: none)
constexpr unsigned kInputTabPoints = kInputTabRows * 4 + kInputTabRows * 64;  // offset of point[]
constexpr unsigned kInputTabBytes = kInputTabPoints + kInputTabRows * 4;

// Host: fills the table for one algorithm from the add networks (inv_sx by canonical point).
void build_input_table(int alg, const float* inv_sx, unsigned char* tab);


// The SFC-6 forms (8x8, 9x9 and 10x10 patches) outside small feature maps: k = 16 i + j over
// two or three matrix steps of 64 (patch rows 4 s .. 4 s + 3 in step s; columns and rows past
// the patch carry no coefficient).  Table, at the start of FilterViews::input_tab:
// float inv_pos[208], int point[208], int8 coeff[208][192] ([position][k]).
constexpr int kRowsTabRows = 208;
constexpr unsigned kRowsTabPoint = kRowsTabRows * 4;
constexpr unsigned kRowsTabCoeff = kRowsTabRows * 8;
constexpr unsigned kRowsTabBytes = kRowsTabCoeff + kRowsTabRows * 192;
void build_rows_table(int alg, const float* inv_sx, unsigned char* tab);

#ifdef __HIPCC__

// Operand A of step s from the staged rows of a tile rectangle (sfc_tile_input.hpp): lane =
// (channel l%16 of the group of 16 starting at ch0, patch row 4 s + l/16), 16 bytes from LDS
// byte o of the row (o = strip * 64 * CS + byte of the tile's first patch column).  Rows past
// the patch repeat its last row, bytes past it belong to the next row: both meet zero
// coefficients.
template <int CS, int NI>
__device__ __forceinline__ v4i operand_rows16(const unsigned char* in, int ch0, int o, int lane, int s) {
  const int ch = ch0 + (lane & 15), row = min(4 * s + (lane >> 4), NI - 1);
  const unsigned* src = (const unsigned*)(in + (unsigned)ch * CS + row * 64 + (o & ~3));
  const unsigned sh = (unsigned)(o & 3);
  unsigned d[5];
#pragma unroll
  for (int i = 0; i < 5; ++i) d[i] = src[i];
  v4i a;
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = (int)__builtin_amdgcn_alignbyte(d[i + 1], d[i], sh);
  return a;
}

template <int ALG>
struct MfmaInput {
  static constexpr int PP = Order<ALG>::PP;
  static constexpr int NPB = (PP + 15) / 16;  // blocks of 16 points
  v4i coeff[NPB];
  float inv[NPB];

  __device__ __forceinline__ void load(const unsigned char* __restrict__ tab, int lane) {
    const float* inv_pos = (const float*)tab;
    const unsigned char* c = tab + kInputTabRows * 4;
#pragma unroll
    for (int m = 0; m < NPB; ++m) {
      const int pos = 16 * m + (lane & 15);
      inv[m] = inv_pos[pos];
      coeff[m] = *(const v4i*)(c + pos * 64 + 16 * (lane >> 4));
    }
  }

  // Operand A from the staged rows of a tile rectangle (sfc_tile_input.hpp: 64 bytes per
  // image row, six rows per channel, CS bytes per channel): lane = (channel l%16 of the group
  // of 16 starting at ch0, patch rows 2(l/16), 2(l/16)+1); o = LDS byte of the tile's first
  // patch column.  Lanes 48..63 (k >= 48, coefficients zero) repeat rows 4, 5.
  template <int CS>
  static __device__ __forceinline__ v4i operand_rect(const unsigned char* in, int s, int ch0, int o,
                                                     int lane) {
    return operand_rect<CS>(in, ch0, s * 64 * CS + o, lane);
  }
  // (the same with the strip folded into the offset: o = strip * 64 * CS + LDS byte of the
  // tile's first patch column, which lies in the first 64 bytes)
  template <int CS>
  static __device__ __forceinline__ v4i operand_rect(const unsigned char* in, int ch0, int o, int lane) {
    const int ch = ch0 + (lane & 15), rp = min(lane >> 4, 2);
    const unsigned* src = (const unsigned*)(in + (unsigned)ch * CS + (2 * rp) * 64 + (o & ~3));
    const unsigned sh = (unsigned)(o & 3);
    v4i a;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const unsigned d0 = src[r * 16], d1 = src[r * 16 + 1], d2 = src[r * 16 + 2];
      a[2 * r] = (int)__builtin_amdgcn_alignbyte(d1, d0, sh);
      a[2 * r + 1] = (int)__builtin_amdgcn_alignbyte(d2, d1, sh);
    }
    return a;
  }

  // Operand A from whole channel planes (small feature maps): sample (r0 + i, q0 + j) of the
  // plane of channel ch0 + l%16, zero outside the image.  The tile position (r0, q0) is the
  // same for the whole wave.  A patch row is cut out of three aligned dwords; its columns
  // outside the image are masked (the same mask for every lane), a row outside the image is
  // replaced by zeros.  The dwords may reach up to 4 bytes before the first plane and 8 bytes
  // past the last one: the caller keeps that much LDS around the planes.
  // (the per-tile part of that, the same for every lane, channel group and chunk)
  struct PlaneTile {
    int boff[2];        // byte offset of the lane's two patch rows from plane - 4 (rows clamped)
    bool rok[2];        // whether they lie inside the image
    unsigned cmask[2];  // bytes of a row's two dwords that are image columns
  };
  static __device__ __forceinline__ PlaneTile plane_tile(int r0, int q0, int H, int W, int lane) {
    PlaneTile t;
    const int rp = min(lane >> 4, 2);
    t.cmask[0] = t.cmask[1] = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if ((unsigned)(q0 + j) < (unsigned)W) t.cmask[j >> 2] |= 0xffu << (8 * (j & 3));
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int h = r0 + 2 * rp + r;
      t.rok[r] = (unsigned)h < (unsigned)H;
      t.boff[r] = min(max(h, 0), H - 1) * W + q0 + 4;  // >= 3
    }
    return t;
  }
  static __device__ __forceinline__ v4i operand_plane(const unsigned char* planes, int cs, int ch0,
                                                      const PlaneTile& t, int lane) {
    const unsigned char* plane = planes + (ch0 + (lane & 15)) * cs;
    v4i a;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const unsigned* src = (const unsigned*)(plane - 4 + (t.boff[r] & ~3));
      const unsigned sh = (unsigned)(t.boff[r] & 3);
      const unsigned d0 = src[0], d1 = src[1], d2 = src[2];
      const unsigned w0 = __builtin_amdgcn_alignbyte(d1, d0, sh) & t.cmask[0];
      const unsigned w1 = __builtin_amdgcn_alignbyte(d2, d1, sh) & t.cmask[1];
      a[2 * r] = t.rok[r] ? (int)w0 : 0;
      a[2 * r + 1] = t.rok[r] ? (int)w1 : 0;
    }
    return a;
  }
  static __device__ __forceinline__ v4i operand_plane(const unsigned char* planes, int cs, int ch0,
                                                      int r0, int q0, int H, int W, int lane) {
    return operand_plane(planes, cs, ch0, plane_tile(r0, q0, H, W, lane), lane);
  }

  // The sums of the lane's four channels for its point of every block (matrix instructions
  // only: a caller can issue those of the next patch before it rounds the current one) ...
  __device__ __forceinline__ void sums(v4i a, v4i (&d)[NPB]) const {
#pragma unroll
    for (int m = 0; m < NPB; ++m)
      d[m] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, coeff[m], v4i{0, 0, 0, 0}, 0, 0, 0);
  }
  // ... and their rounding to int8 (clamp(round-half-even(v / s_Tx), +-qmax)), packed: byte i =
  // channel 4(l/16) + i.
  __device__ __forceinline__ void round(const v4i (&d)[NPB], float qmax, unsigned (&packed)[NPB]) const {
    constexpr float kMagic = 12582912.0f;
#pragma unroll
    for (int m = 0; m < NPB; ++m) {
      unsigned q[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float t = __fmaf_rn((float)d[m][i], inv[m], kMagic);
        t = __builtin_amdgcn_fmed3f(t, kMagic - qmax, kMagic + qmax);
        q[i] = __float_as_uint(t);
      }
      // low bytes of q[0..3] -> one dword
      const unsigned lo = __builtin_amdgcn_perm(q[1], q[0], 0x0c0c0400u);
      const unsigned hi = __builtin_amdgcn_perm(q[3], q[2], 0x04000c0cu);
      packed[m] = lo | hi;
    }
  }
  __device__ __forceinline__ void transform(v4i a, float qmax, unsigned (&packed)[NPB]) const {
    v4i d[NPB];
    sums(a, d);
    round(d, qmax, packed);
  }
};

#endif  // __HIPCC__

}  // namespace sfc
