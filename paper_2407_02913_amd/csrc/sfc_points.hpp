// Add networks of SFC-6(6x6,3x3): forward transforms to the multiplication
// points and the output transform back, as straight-line device code.
//
// A 1-D signal of 8 samples becomes 8 "components" (Sec. 4.1-4.2):
//   c0  X0            (real, k = 0)
//   c1  X1.a0   c2  X1.a1     X1 = a0 + a1 s,  s = exp(j pi/3), s^2 = s - 1
//   c3  X2.a0   c4  X2.a1
//   c5  X3            (real, k = 3)
//   c6  x0 - x6       correction input for output 0   (Sec. 4.2)
//   c7  x7 - x1       correction input for output 5
// The 3-multiplication product rule (Eq. DFT6M) adds a row a0 + a1 per complex
// point, giving the 10 rows of Appendix A's B^T and G:
//   r0=c0 r1=c1 r2=c2 r3=c1+c2 r4=c3 r5=c4 r6=c3+c4 r7=c5 r8=c6 r9=c7.
// In 2-D the components form an 8x8 array C[a][b] (a: vertical axis).
//   P = 100: every (r_a, r_b) pair.
//   P = 88 : the 64 pairs that are not complex x complex, then for each pair of
//            complex frequencies the two independent 2-D DFT values
//              U = (a00 - a11) + (a10 + a01 + a11) s
//              V = (a00 + a01 + a11) + (a10 - a01) s
//            each as (x0, x1, x0 + x1).
#pragma once
#include <hip/hip_runtime.h>

// host + device so that the add networks can also be checked on the CPU
#define SFC_HD __host__ __device__ __forceinline__

namespace sfc {

constexpr int kTileOut = 6;
constexpr int kTileIn = 8;

template <int ALG>
struct AlgTraits;
template <>
struct AlgTraits<0> {
  static constexpr int P = 88;
};
template <>
struct AlgTraits<1> {
  static constexpr int P = 100;
};

// ---- forward, 1-D ----------------------------------------------------------

// Eight samples -> eight components (14 additions for the symbolic DFT-6 of the
// inner six samples, 2 for the correction inputs).
template <typename T>
SFC_HD void fwd8(const T (&x)[8], T (&c)[8]) {
  const T e0 = x[1] + x[4], e1 = x[2] + x[5], e2 = x[3] + x[6];
  const T d0 = x[1] - x[4], d1 = x[2] - x[5], d2 = x[3] - x[6];
  c[0] = e0 + e1 + e2;
  c[1] = d0 + d1;
  c[2] = -d1 - d2;
  c[3] = e0 - e2;
  c[4] = e2 - e1;
  c[5] = d0 - d1 + d2;
  c[6] = x[0] - x[6];
  c[7] = x[7] - x[1];
}

// Three filter taps -> eight components (rows of Appendix A's G without the sum rows).
template <typename T>
SFC_HD void fwd3(const T (&f)[3], T (&c)[8]) {
  c[0] = f[0] + f[1] + f[2];
  c[1] = f[1] + f[2];
  c[2] = -f[0] - f[1];
  c[3] = f[2] - f[0];
  c[4] = f[0] - f[1];
  c[5] = f[0] - f[1] + f[2];
  c[6] = f[0];
  c[7] = f[2];
}

// component index -> which components a 1-D row adds (second = -1: none)
SFC_HD constexpr int row_c0(int r) {
  return r == 0 ? 0 : r == 1 ? 1 : r == 2 ? 2 : r == 3 ? 1 : r == 4 ? 3 : r == 5 ? 4 : r == 6 ? 3 : r == 7 ? 5 : r == 8 ? 6 : 7;
}
SFC_HD constexpr int row_c1(int r) { return r == 3 ? 2 : r == 6 ? 4 : -1; }
SFC_HD constexpr bool row_is_complex(int r) { return r >= 1 && r <= 6; }

// ---- forward, 2-D: components -> multiplication points ----------------------

template <typename T>
SFC_HD T nested_point(const T (&c)[8][8], int r1, int r2) {
  const int a0 = row_c0(r1), a1 = row_c1(r1), b0 = row_c0(r2), b1 = row_c1(r2);
  T v = c[a0][b0];
  if (b1 >= 0) v += c[a0][b1];
  if (a1 >= 0) {
    v += c[a1][b0];
    if (b1 >= 0) v += c[a1][b1];
  }
  return v;
}

// The six Hermitian points of the frequency pair (g1, g2), g in {0,1} -> k = g + 1.
template <typename T>
SFC_HD void hermitian_points(const T (&c)[8][8], int g1, int g2, T (&out)[6]) {
  const int a = 1 + 2 * g1, b = 1 + 2 * g2;
  const T a00 = c[a][b], a10 = c[a + 1][b], a01 = c[a][b + 1], a11 = c[a + 1][b + 1];
  const T u0 = a00 - a11, u1 = a10 + a01 + a11;
  const T v0 = a00 + a01 + a11, v1 = a10 - a01;
  out[0] = u0;
  out[1] = u1;
  out[2] = u0 + u1;
  out[3] = v0;
  out[4] = v1;
  out[5] = v0 + v1;
}

// Calls f(p, value) for every point in canonical order.  Fully unrolled: p is a
// compile-time constant at each call site after inlining.
template <int ALG, typename T, typename F>
SFC_HD void for_each_point(const T (&c)[8][8], F&& f) {
  if constexpr (ALG == 1) {
#pragma unroll
    for (int r1 = 0; r1 < 10; ++r1)
#pragma unroll
      for (int r2 = 0; r2 < 10; ++r2) f(10 * r1 + r2, nested_point(c, r1, r2));
  } else {
    int p = 0;
#pragma unroll
    for (int r1 = 0; r1 < 10; ++r1)
#pragma unroll
      for (int r2 = 0; r2 < 10; ++r2) {
        if (row_is_complex(r1) && row_is_complex(r2)) continue;
        f(p++, nested_point(c, r1, r2));
      }
#pragma unroll
    for (int g1 = 0; g1 < 2; ++g1)
#pragma unroll
      for (int g2 = 0; g2 < 2; ++g2) {
        T h[6];
        hermitian_points(c, g1, g2, h);
#pragma unroll
        for (int i = 0; i < 6; ++i) f(p++, h[i]);
      }
  }
}

// ---- output transform --------------------------------------------------------

// Ten 1-D products -> eight components: o0 = m0 - m1, o1 = m2 - m0 (Eq. DFT6M).
template <typename T>
SFC_HD void collapse10(const T (&r)[10], T (&c)[8]) {
  c[0] = r[0];
  c[1] = r[1] - r[2];
  c[2] = r[3] - r[1];
  c[3] = r[4] - r[5];
  c[4] = r[6] - r[4];
  c[5] = r[7];
  c[6] = r[8];
  c[7] = r[9];
}

template <typename T>
struct Third;
template <>
struct Third<int> {
  // exact division of a multiple of 3: multiply by the inverse of 3 modulo 2^32
  static SFC_HD int apply(int v) { return (int)((unsigned)v * 0xAAAAAAABu); }
};
template <>
struct Third<float> {
  static SFC_HD float apply(float v) { return v * (1.0f / 3.0f); }
};

// Six Hermitian products of one frequency pair -> the four product components
// o[i][j] (i: power of s along the vertical axis, j: along the horizontal axis).
template <typename T>
SFC_HD void hermitian_collapse(const T (&m)[6], T& o00, T& o10, T& o01, T& o11) {
  const T uo0 = m[0] - m[1], uo1 = m[2] - m[0];
  const T vo0 = m[3] - m[4], vo1 = m[5] - m[3];
  const T du = uo1 - vo1, dv = vo0 - uo0;
  o01 = Third<T>::apply(du + du - dv);
  o11 = Third<T>::apply(dv + dv - du);
  o00 = uo0 + o11;
  o10 = vo1 + o01;
}

// Eight components -> six outputs, times 6 (the inverse symbolic DFT-6 through its
// DFT-2 x DFT-3 structure, plus the two correction products with weight 6).
template <typename T>
SFC_HD void inv8(const T (&c)[8], T (&y)[6]) {
  // even harmonics k = 0, 2 repeat with period 3; odd harmonics k = 1, 3 flip sign
  const T t = c[0] - c[3];
  const T e0 = t - c[4] - c[4];
  const T e1 = t + c[4];
  const T e2 = c[0] + c[3] + c[3] + c[4];
  const T d0 = c[1] - c[2] - c[5];
  const T d1 = c[5] - c[1] - c[2] - c[2];
  const T d2 = -c[1] - c[1] - c[2] - c[5];
  y[0] = e0 + d0 + T(6) * c[6];
  y[1] = e1 + d1;
  y[2] = e2 + d2;
  y[3] = e0 - d0;
  y[4] = e1 - d1;
  y[5] = e2 - d2 + T(6) * c[7];
}

// All P products of one (tile, Cout) pair -> 36 outputs times 36.
// get(p) returns product p (already scaled in the dequantizing case).
template <int ALG, typename T, typename G>
SFC_HD void output_transform(G&& get, T (&out)[6][6]) {
  T comp[8][8];
  if constexpr (ALG == 1) {
    T half[10][8];
#pragma unroll
    for (int r1 = 0; r1 < 10; ++r1) {
      T row[10];
#pragma unroll
      for (int r2 = 0; r2 < 10; ++r2) row[r2] = get(10 * r1 + r2);
      collapse10(row, half[r1]);
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      T col[10], cc[8];
#pragma unroll
      for (int r1 = 0; r1 < 10; ++r1) col[r1] = half[r1][b];
      collapse10(col, cc);
#pragma unroll
      for (int a = 0; a < 8; ++a) comp[a][b] = cc[a];
    }
  } else {
    // the 64 kept points: rows where r1 is real hold all ten r2; rows where r1
    // is complex hold only the four real r2 (0, 7, 8, 9)
    T kept[10][10];
    int p = 0;
#pragma unroll
    for (int r1 = 0; r1 < 10; ++r1)
#pragma unroll
      for (int r2 = 0; r2 < 10; ++r2) {
        if (row_is_complex(r1) && row_is_complex(r2)) {
          kept[r1][r2] = T(0);
          continue;
        }
        kept[r1][r2] = get(p++);
      }
    // real r1: collapse along the horizontal axis
    constexpr int real_rows[4] = {0, 7, 8, 9};
    constexpr int real_comp[4] = {0, 5, 6, 7};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      T cc[8];
      collapse10(kept[real_rows[i]], cc);
#pragma unroll
      for (int b = 0; b < 8; ++b) comp[real_comp[i]][b] = cc[b];
    }
    // complex r1, real r2: collapse along the vertical axis
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      T col[10], cc[8];
#pragma unroll
      for (int r1 = 0; r1 < 10; ++r1) col[r1] = kept[r1][real_rows[j]];
      collapse10(col, cc);
#pragma unroll
      for (int a = 1; a <= 4; ++a) comp[a][real_comp[j]] = cc[a];
    }
    // complex x complex from the Hermitian blocks
#pragma unroll
    for (int g1 = 0; g1 < 2; ++g1)
#pragma unroll
      for (int g2 = 0; g2 < 2; ++g2) {
        T m[6];
#pragma unroll
        for (int i = 0; i < 6; ++i) m[i] = get(p++);
        const int a = 1 + 2 * g1, b = 1 + 2 * g2;
        hermitian_collapse(m, comp[a][b], comp[a + 1][b], comp[a][b + 1], comp[a + 1][b + 1]);
      }
  }
  // separable inverse: along the horizontal axis, then the vertical one
  T z[8][6];
#pragma unroll
  for (int a = 0; a < 8; ++a) inv8(comp[a], z[a]);
#pragma unroll
  for (int o2 = 0; o2 < 6; ++o2) {
    T col[8], y[6];
#pragma unroll
    for (int a = 0; a < 8; ++a) col[a] = z[a][o2];
    inv8(col, y);
#pragma unroll
    for (int o1 = 0; o1 < 6; ++o1) out[o1][o2] = y[o1];
  }
}

}  // namespace sfc
