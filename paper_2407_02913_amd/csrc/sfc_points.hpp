// Add networks of SFC-6(6x6,3x3), SFC-6(7x7,3x3), SFC-4(4x4,3x3), SFC-6(6x6,5x5) and SFC-6(4x4,7x7):
// forward transforms to the multiplication points and the output transform back, as
// straight-line code.
//
// 3x3 filters: a 1-D signal of M+2 samples (M = 6 or 7 outputs) becomes NC "components"
// (Sec. 4.1-4.2):
//   c0  X0            (real, k = 0)
//   c1  X1.a0   c2  X1.a1     X1 = a0 + a1 s,  s = exp(j pi/3), s^2 = s - 1
//   c3  X2.a0   c4  X2.a1
//   c5  X3            (real, k = 3)
//   c6  x0 - x6       correction input for output 0, paired with f0   (Sec. 4.2)
//   c7  x7 - x1       correction input for output 5, paired with f2
//   c8  x7 - x1       M = 7 only: correction for output 6, paired with f1
//   c9  x8 - x2       M = 7 only: correction for output 6, paired with f2
// The 3-multiplication product rule (Eq. DFT6M) adds a row a0 + a1 per complex
// point, giving the NR = NC + 2 rows of Appendix A's B^T and G:
//   r0=c0 r1=c1 r2=c2 r3=c1+c2 r4=c3 r5=c4 r6=c3+c4 r7=c5 r8=c6 r9=c7 (r10=c8 r11=c9).
// SFC-6(6x6,5x5) (Appendix A): ten samples, the symbolic DFT-6 works on x2..x7, the filter's
// as G_k = sum_r f_r s^(k (r - 4)); six corrections (wanted sample minus the one the cyclic
// convolution supplies, times one tap):
//   c6  x0 - x6 with f0 -> output 0     c7  x1 - x7 with f0 -> output 1     c8  x1 - x7 with f1 -> output 0
//   c9  x8 - x2 with f3 -> output 5     c10 x8 - x2 with f4 -> output 4     c11 x9 - x3 with f4 -> output 5
// With this alignment the inverse symbolic DFT delivers the cyclic result rotated by one
// position.  NC = 12 components, NR = 14 rows, 196 nested / 184 Hermitian points.
// SFC-6(4x4,7x7) (Table 1; derived with the same steps): the same ten samples, window and
// differences on the input side, so the same input transform; the filter's symbolic DFT is
// G_k = sum_r f_r s^(k r) (aligned on the seventh tap, s^6 = 1); six corrections:
//   c6  x0 - x6 with f0 -> output 0     c7  x1 - x7 with f0 -> output 1     c8  x1 - x7 with f1 -> output 0
//   c9  x8 - x2 with f5 -> output 3     c10 x8 - x2 with f6 -> output 2     c11 x9 - x3 with f6 -> output 3
// and the inverse delivers the cyclic result rotated by three positions.  Also NC = 12,
// NR = 14, 196 / 184 points.
// In 2-D the components form an NC x NC array C[a][b] (a: vertical axis).
//   nested   : every (r_a, r_b) pair, NR^2 points (100 / 144).
//   Hermitian: the pairs that are not complex x complex, then for each pair of
//              complex frequencies the two independent 2-D DFT values
//                U = (a00 - a11) + (a10 + a01 + a11) s
//                V = (a00 + a01 + a11) + (a10 - a01) s
//              each as (x0, x1, x0 + x1): NR^2 - 12 points (88 / 132).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

// host + device so that the add networks can also be checked on the CPU
#define SFC_HD __host__ __device__ __forceinline__

namespace sfc {

// SFC-4(4x4,3x3) (Appendix A, s = j): a signal of 6 samples becomes 6 components
//   c0  X0    c1  -X2   (real, as printed)    c2  X1.a0   c3  X1.a1   (X1 = a0 + a1 j)
//   c4  x0 - x4  (correction for output 0, with f0)     c5  x5 - x1  (for output 3, with f2)
// and the 7 rows of the printed matrices are r0=c0 r1=c1 r2=c2+c3 r3=c3 r4=c2 r5=c4 r6=c5.
// Product rule (Eq. DFT4M): o0 = m0 - m1, o1 = m2 - m0 - m1.  Hermitian form: the one
// complex x complex block (9 points) becomes U = (a00 - a11) + (a10 + a01) s and
// V = (a00 + a11) + (a10 - a01) s, each as (x0, x1, x0 + x1): 46 points instead of 49.
//
// ALG: 0 = 6x6 Hermitian (88), 1 = 6x6 nested (100), 2 = 7x7 Hermitian (132), 3 = 7x7 nested (144),
//      4 = 4x4 Hermitian (46), 5 = 4x4 nested (49), all for 3x3 filters;
//      6 = 6x6 outputs with a 5x5 filter, Hermitian (184), 7 = the same, nested (196);
//      8 = 4x4 outputs with a 7x7 filter, Hermitian (184), 9 = the same, nested (196)
template <int ALG>
struct AlgTraits {
  static_assert(ALG >= 0 && ALG < 10, "unknown algorithm");
  static constexpr int kFamily = (ALG < 4 || ALG >= 6) ? 6 : 4;  // points of the symbolic DFT
  static constexpr bool kHermitian = ALG % 2 == 0;
  static constexpr int M = ALG < 2 ? 6 : ALG < 4 ? 7 : ALG < 6 ? 4 : ALG < 8 ? 6 : 4;  // outputs per tile edge
  static constexpr int R = ALG < 6 ? 3 : ALG < 8 ? 5 : 7;                // filter taps per axis
  static constexpr int PAD = (R - 1) / 2;                                // zero padding
  static constexpr int NI = M + R - 1;                                   // input samples per tile edge
  static constexpr int NC = ALG < 2 ? 8 : ALG < 4 ? 10 : ALG < 6 ? 6 : 12;  // components per axis
  // rows of the printed 1-D matrices: one more than components per complex point
  static constexpr int NR = kFamily == 6 ? NC + 2 : NC + 1;
  static constexpr int NREAL = kFamily == 6 ? NR - 6 : NR - 3;  // rows outside a complex point
  static constexpr int P = !kHermitian ? NR * NR : kFamily == 6 ? NR * NR - 12 : NR * NR - 3;
  static constexpr int kDen = kFamily == 6 ? 36 : 16;  // the output transform yields kDen * y
};

constexpr int kNumAlgs = 10;
__host__ __device__ constexpr int alg_points(int alg) {
  return alg == 0 ? 88 : alg == 1 ? 100 : alg == 2 ? 132 : alg == 3 ? 144 : alg == 4 ? 46
       : alg == 5 ? 49 : (alg == 6 || alg == 8) ? 184 : 196;
}
__host__ __device__ constexpr int alg_tile(int alg) {
  return alg < 2 ? 6 : alg < 4 ? 7 : alg < 6 ? 4 : alg < 8 ? 6 : 4;
}
__host__ __device__ constexpr int alg_taps(int alg) { return alg < 6 ? 3 : alg < 8 ? 5 : 7; }

// ---- row bookkeeping ----------------------------------------------------------

// row -> the component(s) it adds (second = -1: none)
SFC_HD constexpr int row_c0(int r) {
  return r == 0 ? 0 : r == 1 ? 1 : r == 2 ? 2 : r == 3 ? 1 : r == 4 ? 3 : r == 5 ? 4 : r == 6 ? 3 : r == 7 ? 5 : r - 2;
}
SFC_HD constexpr int row_c1(int r) { return r == 3 ? 2 : r == 6 ? 4 : -1; }
SFC_HD constexpr bool row_is_complex(int r) { return r >= 1 && r <= 6; }
// i-th real row (0, 7, 8, 9, ...) and the component it carries (0, 5, 6, 7, ...)
SFC_HD constexpr int real_row(int i) { return i == 0 ? 0 : 6 + i; }
SFC_HD constexpr int real_comp(int i) { return i == 0 ? 0 : 4 + i; }

// canonical index of the kept nested point (r1, r2) of a Hermitian point set
template <int NR>
SFC_HD constexpr int kept_index(int r1, int r2) {
  int n = 0;
  for (int a = 0; a < NR; ++a)
    for (int b = 0; b < NR; ++b) {
      if (row_is_complex(a) && row_is_complex(b)) continue;
      if (a == r1 && b == r2) return n;
      ++n;
    }
  return -1;
}

// SFC-4: row -> component(s), in the printed row order
SFC_HD constexpr int row4_c0(int r) { return r == 0 ? 0 : r == 1 ? 1 : r == 2 ? 2 : r == 3 ? 3 : r == 4 ? 2 : r - 1; }
SFC_HD constexpr int row4_c1(int r) { return r == 2 ? 3 : -1; }
SFC_HD constexpr bool row4_is_complex(int r) { return r >= 2 && r <= 4; }

// SFC-4: i-th real row (0, 1, 5, 6) and the component it carries (0, 1, 4, 5)
SFC_HD constexpr int real_row4(int i) { return i < 2 ? i : i + 3; }
SFC_HD constexpr int real_comp4(int i) { return i < 2 ? i : i + 2; }
// SFC-4: canonical index of the kept nested point (r1, r2) of the Hermitian point set
SFC_HD constexpr int kept_index4(int r1, int r2) {
  int n = 0;
  for (int a = 0; a < 7; ++a)
    for (int b = 0; b < 7; ++b) {
      if (row4_is_complex(a) && row4_is_complex(b)) continue;
      if (a == r1 && b == r2) return n;
      ++n;
    }
  return -1;
}

// Processing order of the fused kernels: canonical point indices grouped by
// horizontal class (first the real columns with all their vertical rows, then the
// complex column groups), so that each group can be collapsed as soon as its
// products exist.  pt[j] = canonical index of the j-th point, pos = its inverse.
// The kernels take points in groups of four: PP is P rounded up to a multiple of four,
// positions P .. PP-1 hold no point (pt = -1; only the SFC-4 forms have any).
template <int ALG>
struct Order {
  using Tr = AlgTraits<ALG>;
  static constexpr int P = Tr::P, NR = Tr::NR, NREAL = Tr::NREAL;
  static constexpr int PP = (P + 3) / 4 * 4;
  int pt[PP];
  int pos[P];
  constexpr Order() : pt{}, pos{} {
    int n = 0;
    if constexpr (Tr::kFamily == 4) {
      // real columns 0, 1, 5, 6: all seven vertical rows
      for (int j = 0; j < NREAL; ++j)
        for (int r1 = 0; r1 < NR; ++r1)
          pt[n++] = Tr::kHermitian ? kept_index4(r1, real_row4(j)) : NR * r1 + real_row4(j);
      // the complex column group: rows 2, 3, 4 = (a0 + a1, a1, a0)
      if (!Tr::kHermitian) {
        for (int r1 = 0; r1 < NR; ++r1)
          for (int i = 0; i < 3; ++i) pt[n++] = NR * r1 + 2 + i;
      } else {
        for (int j = 0; j < NREAL; ++j)
          for (int i = 0; i < 3; ++i) pt[n++] = kept_index4(real_row4(j), 2 + i);
        for (int i = 0; i < 6; ++i) pt[n++] = (NR * NR - 9) + i;
      }
    } else {
      // real columns: all vertical rows
      for (int j = 0; j < NREAL; ++j)
        for (int r1 = 0; r1 < NR; ++r1)
          pt[n++] = Tr::kHermitian ? kept_index<NR>(r1, real_row(j)) : NR * r1 + real_row(j);
      // complex column groups
      for (int g2 = 0; g2 < 2; ++g2) {
        if (!Tr::kHermitian) {
          for (int r1 = 0; r1 < NR; ++r1)
            for (int i = 0; i < 3; ++i) pt[n++] = NR * r1 + 1 + 3 * g2 + i;
        } else {
          for (int j = 0; j < NREAL; ++j)
            for (int i = 0; i < 3; ++i) pt[n++] = kept_index<NR>(real_row(j), 1 + 3 * g2 + i);
          for (int g1 = 0; g1 < 2; ++g1)
            for (int i = 0; i < 6; ++i) pt[n++] = (NR * NR - 36) + 6 * (2 * g1 + g2) + i;
        }
      }
    }
    for (int j = 0; j < P; ++j) pos[pt[j]] = j;
    for (int j = P; j < PP; ++j) pt[j] = -1;
  }
};

// ---- forward, 1-D ----------------------------------------------------------

// NI samples -> NC components (14 additions for the symbolic DFT-6 of the inner
// six samples, one per correction input).
template <int NI, int NC, typename T>
SFC_HD void fwd_input(const T (&x)[NI], T (&c)[NC]) {
  if constexpr (NC == 12) {
    // 5-tap and 7-tap filters: ten samples, the inner six are x2..x7
    static_assert(NI == 10, "SFC-6(6,5) and SFC-6(4,7) take ten samples");
    const T e0 = x[2] + x[5], e1 = x[3] + x[6], e2 = x[4] + x[7];
    const T d0 = x[2] - x[5], d1 = x[3] - x[6], d2 = x[4] - x[7];
    c[0] = e0 + e1 + e2;
    c[1] = d0 + d1;
    c[2] = -d1 - d2;
    c[3] = e0 - e2;
    c[4] = e2 - e1;
    c[5] = d0 - d1 + d2;
    c[6] = x[0] - x[6];
    c[7] = x[1] - x[7];
    c[8] = c[7];
    c[9] = x[8] - x[2];
    c[10] = c[9];
    c[11] = x[9] - x[3];
    return;
  } else if constexpr (NI == 6) {
    // SFC-4: 6 samples -> 6 components, 8 additions
    const T s02 = x[1] + x[3], s13 = x[2] + x[4];
    c[0] = s02 + s13;
    c[1] = s13 - s02;
    c[2] = x[1] - x[3];
    c[3] = x[4] - x[2];
    c[4] = x[0] - x[4];
    c[5] = x[5] - x[1];
    return;
  } else {
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
  if constexpr (NC == 10) {
    c[8] = c[7];
    c[9] = x[8] - x[2];
  }
  }
}

// R filter taps -> NC components (rows of Appendix A's G without the sum rows).
template <int R, int NC, typename T>
SFC_HD void fwd_filter(const T (&f)[R], T (&c)[NC]) {
  if constexpr (NC == 12 && R == 7) {
    // G_k = sum_r f_r s^(k r): s^0..s^6 = 1, s, s - 1, -1, -s, 1 - s, 1
    const T a = f[0] + f[6], b = f[2] + f[5], d = f[1] + f[4];
    const T e = f[2] - f[5], h = f[1] - f[4];
    c[0] = a + b + d + f[3];
    c[1] = a - f[3] - e;
    c[2] = h + e;
    c[3] = a + f[3] - d;
    c[4] = d - b;
    c[5] = a - f[3] + e - h;
    c[6] = f[0];
    c[7] = f[0];
    c[8] = f[1];
    c[9] = f[5];
    c[10] = f[6];
    c[11] = f[6];
    return;
  } else if constexpr (NC == 12) {
    static_assert(R == 5, "SFC-6(6,5) takes five taps");
    const T p = f[3] + f[4], q = f[0] + f[1];
    c[0] = q + f[2] + p;
    c[1] = p - q;
    c[2] = f[0] - f[2] - f[3];
    c[3] = f[1] - f[2] + f[4];
    c[4] = f[2] - f[0] - f[3];
    c[5] = f[0] - f[1] + f[2] - f[3] + f[4];
    c[6] = f[0];
    c[7] = f[0];
    c[8] = f[1];
    c[9] = f[3];
    c[10] = f[4];
    c[11] = f[4];
    return;
  } else if constexpr (NC == 6) {
    // SFC-4 (rows of Appendix A's G without the sum row)
    const T s = f[0] + f[2];
    c[0] = s + f[1];
    c[1] = s - f[1];
    c[2] = -f[1];
    c[3] = f[0] - f[2];
    c[4] = f[0];
    c[5] = f[2];
    return;
  } else {
  c[0] = f[0] + f[1] + f[2];
  c[1] = f[1] + f[2];
  c[2] = -f[0] - f[1];
  c[3] = f[2] - f[0];
  c[4] = f[0] - f[1];
  c[5] = f[0] - f[1] + f[2];
  c[6] = f[0];
  c[7] = f[2];
  if constexpr (NC == 10) {
    c[8] = f[1];
    c[9] = f[2];
  }
  }
}

// ---- forward, 2-D: components -> multiplication points ----------------------

template <int NC, typename T>
SFC_HD T nested_point(const T (&c)[NC][NC], int r1, int r2) {
  constexpr bool k4 = NC == 6;  // SFC-4
  const int a0 = k4 ? row4_c0(r1) : row_c0(r1), a1 = k4 ? row4_c1(r1) : row_c1(r1);
  const int b0 = k4 ? row4_c0(r2) : row_c0(r2), b1 = k4 ? row4_c1(r2) : row_c1(r2);
  T v = c[a0][b0];
  if (b1 >= 0) v += c[a0][b1];
  if (a1 >= 0) {
    v += c[a1][b0];
    if (b1 >= 0) v += c[a1][b1];
  }
  return v;
}

// The six Hermitian points of the frequency pair (g1, g2), g in {0,1} -> k = g + 1.
template <int NC, typename T>
SFC_HD void hermitian_points(const T (&c)[NC][NC], int g1, int g2, T (&out)[6]) {
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

// SFC-4: the six Hermitian points of the single complex frequency pair (components 2, 3).
template <typename T>
SFC_HD void hermitian4_points(const T (&c)[6][6], T (&out)[6]) {
  const T a00 = c[2][2], a10 = c[3][2], a01 = c[2][3], a11 = c[3][3];
  const T u0 = a00 - a11, u1 = a10 + a01;
  const T v0 = a00 + a11, v1 = a10 - a01;
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
SFC_HD void for_each_point(const T (&c)[AlgTraits<ALG>::NC][AlgTraits<ALG>::NC], F&& f) {
  constexpr int NR = AlgTraits<ALG>::NR;
  if constexpr (!AlgTraits<ALG>::kHermitian) {
#pragma unroll
    for (int r1 = 0; r1 < NR; ++r1)
#pragma unroll
      for (int r2 = 0; r2 < NR; ++r2) f(NR * r1 + r2, nested_point(c, r1, r2));
  } else {
    int p = 0;
#pragma unroll
    for (int r1 = 0; r1 < NR; ++r1)
#pragma unroll
      for (int r2 = 0; r2 < NR; ++r2) {
        if constexpr (AlgTraits<ALG>::kFamily == 4) {
          if (row4_is_complex(r1) && row4_is_complex(r2)) continue;
        } else {
          if (row_is_complex(r1) && row_is_complex(r2)) continue;
        }
        f(p++, nested_point(c, r1, r2));
      }
    if constexpr (AlgTraits<ALG>::kFamily == 4) {
      T h[6];
      hermitian4_points(c, h);
#pragma unroll
      for (int i = 0; i < 6; ++i) f(p++, h[i]);
    } else {
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
}

// ---- output transform --------------------------------------------------------

// NR 1-D products -> NC components: o0 = m0 - m1, o1 = m2 - m0 (Eq. DFT6M).
template <int NR, typename T>
SFC_HD void collapse_rows(const T (&r)[NR], T (&c)[NR - 2]) {
  c[0] = r[0];
  c[1] = r[1] - r[2];
  c[2] = r[3] - r[1];
  c[3] = r[4] - r[5];
  c[4] = r[6] - r[4];
  c[5] = r[7];
#pragma unroll
  for (int i = 8; i < NR; ++i) c[i - 2] = r[i];
}

template <typename T>
struct Third;
template <>
struct Third<int> {
  // exact division of a multiple of 3: multiply by the inverse of 3 modulo 2^32
  static SFC_HD int apply(int v) { return (int)((unsigned)v * 0xAAAAAAABu); }
};
template <>
struct Third<unsigned> {  // the same modulo 2^32, wrap-around defined
  static SFC_HD unsigned apply(unsigned v) { return v * 0xAAAAAAABu; }
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

// NC components -> M outputs, times 6 (the inverse symbolic DFT-6 through its
// DFT-2 x DFT-3 structure, plus the correction products with weight 6).  For
// M = 7 the seventh output is the cyclic output 0 with its own two corrections.
// For the 5-tap form the cyclic result arrives rotated by one position and six
// corrections are added; for the 7-tap form (four outputs) rotated by three positions.
template <int NC, int MO, typename T>
SFC_HD void inv_outputs(const T (&c)[NC], T (&y)[MO]) {
  static_assert((NC == 8 && MO == 6) || (NC == 10 && MO == 7) || (NC == 12 && (MO == 6 || MO == 4)),
                "components and outputs of one of the SFC-6 algorithms");
  // even harmonics k = 0, 2 repeat with period 3; odd harmonics k = 1, 3 flip sign
  const T t = c[0] - c[3];
  const T e0 = t - c[4] - c[4];
  const T e1 = t + c[4];
  const T e2 = c[0] + c[3] + c[3] + c[4];
  const T d0 = c[1] - c[2] - c[5];
  const T d1 = c[5] - c[1] - c[2] - c[2];
  const T d2 = -c[1] - c[1] - c[2] - c[5];
  if constexpr (NC == 12 && MO == 4) {
    y[0] = e0 - d0 + T(6) * (c[6] + c[8]);
    y[1] = e1 - d1 + T(6) * c[7];
    y[2] = e2 - d2 + T(6) * c[10];
    y[3] = e0 + d0 + T(6) * (c[9] + c[11]);
  } else if constexpr (NC == 12) {
    y[0] = e1 + d1 + T(6) * (c[6] + c[8]);
    y[1] = e2 + d2 + T(6) * c[7];
    y[2] = e0 - d0;
    y[3] = e1 - d1;
    y[4] = e2 - d2 + T(6) * c[10];
    y[5] = e0 + d0 + T(6) * (c[9] + c[11]);
  } else {
    const T y0 = e0 + d0;
    y[0] = y0 + T(6) * c[6];
    y[1] = e1 + d1;
    y[2] = e2 + d2;
    y[3] = e0 - d0;
    y[4] = e1 - d1;
    y[5] = e2 - d2 + T(6) * c[7];
    if constexpr (NC == 10) y[6] = y0 + T(6) * (c[8] + c[9]);
  }
}

template <typename T>
struct Half;
template <>
struct Half<int> {
  static SFC_HD int apply(int v) { return v >> 1; }  // exact: the argument is even
};
template <>
struct Half<unsigned> {  // two's-complement value halved (exact while it fits 32 bits)
  static SFC_HD unsigned apply(unsigned v) { return (unsigned)((int)v >> 1); }
};
template <>
struct Half<float> {
  static SFC_HD float apply(float v) { return v * 0.5f; }
};

// SFC-4: 7 1-D products -> 6 components (Eq. DFT4M: o0 = m0 - m1, o1 = m2 - m0 - m1, with
// the rows a0+a1, a1, a0 at positions 2, 3, 4).
template <typename T>
SFC_HD void collapse4_rows(const T (&r)[7], T (&c)[6]) {
  c[0] = r[0];
  c[1] = r[1];
  c[2] = r[4] - r[3];
  c[3] = r[2] - r[4] - r[3];
  c[4] = r[5];
  c[5] = r[6];
}

// SFC-4: 6 components -> 4 outputs, times 4 (inverse symbolic DFT-4 plus the corrections).
template <typename T>
SFC_HD void inv4_outputs(const T (&c)[6], T (&y)[4]) {
  const T s = c[0] + c[1], d = c[0] - c[1];
  const T re2 = c[2] + c[2], im2 = c[3] + c[3];
  y[0] = s - re2 + T(4) * c[4];
  y[1] = d + im2;
  y[2] = s + re2;
  y[3] = d - im2 + T(4) * c[5];
}

// SFC-4: all P products of one (tile, Cout) pair -> 4 x 4 outputs times 16.
template <int ALG, typename T, typename G>
SFC_HD void output_transform4(G&& get, T (&out)[4][4]) {
  constexpr int NR = 7, NC = 6;
  T comp[NC][NC];
  if constexpr (!AlgTraits<ALG>::kHermitian) {
    T half[NR][NC];
#pragma unroll
    for (int r1 = 0; r1 < NR; ++r1) {
      T row[NR];
#pragma unroll
      for (int r2 = 0; r2 < NR; ++r2) row[r2] = get(NR * r1 + r2);
      collapse4_rows(row, half[r1]);
    }
#pragma unroll
    for (int b = 0; b < NC; ++b) {
      T col[NR], cc[NC];
#pragma unroll
      for (int r1 = 0; r1 < NR; ++r1) col[r1] = half[r1][b];
      collapse4_rows(col, cc);
#pragma unroll
      for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
    }
  } else {
    T kept[NR][NR];
    int p = 0;
#pragma unroll
    for (int r1 = 0; r1 < NR; ++r1)
#pragma unroll
      for (int r2 = 0; r2 < NR; ++r2) {
        if (row4_is_complex(r1) && row4_is_complex(r2)) {
          kept[r1][r2] = T(0);
          continue;
        }
        kept[r1][r2] = get(p++);
      }
    // real r1 (rows 0, 1, 5, 6 -> components 0, 1, 4, 5): collapse along the horizontal axis
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r1 = i < 2 ? i : i + 3, a = i < 2 ? i : i + 2;
      T cc[NC];
      collapse4_rows(kept[r1], cc);
#pragma unroll
      for (int b = 0; b < NC; ++b) comp[a][b] = cc[b];
    }
    // complex r1, real r2: collapse along the vertical axis
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r2 = j < 2 ? j : j + 3, b = j < 2 ? j : j + 2;
      T col[NR], cc[NC];
#pragma unroll
      for (int r1 = 0; r1 < NR; ++r1) col[r1] = kept[r1][r2];
      collapse4_rows(col, cc);
      comp[2][b] = cc[2];
      comp[3][b] = cc[3];
    }
    // complex x complex from the Hermitian block
    T m[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) m[i] = get(p++);
    const T uo0 = m[0] - m[1], uo1 = m[2] - m[0] - m[1];
    const T vo0 = m[3] - m[4], vo1 = m[5] - m[3] - m[4];
    comp[2][2] = Half<T>::apply(uo0 + vo0);  // o00
    comp[3][3] = Half<T>::apply(vo0 - uo0);  // o11
    comp[3][2] = Half<T>::apply(uo1 + vo1);  // o10
    comp[2][3] = Half<T>::apply(uo1 - vo1);  // o01
  }
  T z[NC][4];
#pragma unroll
  for (int a = 0; a < NC; ++a) inv4_outputs(comp[a], z[a]);
#pragma unroll
  for (int o2 = 0; o2 < 4; ++o2) {
    T col[NC], y[4];
#pragma unroll
    for (int a = 0; a < NC; ++a) col[a] = z[a][o2];
    inv4_outputs(col, y);
#pragma unroll
    for (int o1 = 0; o1 < 4; ++o1) out[o1][o2] = y[o1];
  }
}

// All P products of one (tile, Cout) pair -> M x M outputs times 36 (16 for SFC-4).
// get(p) returns product p (already scaled in the dequantizing case).
template <int ALG, typename T, typename G>
SFC_HD void output_transform(G&& get, T (&out)[AlgTraits<ALG>::M][AlgTraits<ALG>::M]) {
  using Tr = AlgTraits<ALG>;
  if constexpr (Tr::kFamily == 4) {
    output_transform4<ALG, T>(get, out);
    return;
  } else {
  constexpr int NR = Tr::NR, NC = Tr::NC, M = Tr::M, NREAL = Tr::NREAL;
  T comp[NC][NC];
  if constexpr (!Tr::kHermitian) {
    T half[NR][NC];
#pragma unroll
    for (int r1 = 0; r1 < NR; ++r1) {
      T row[NR];
#pragma unroll
      for (int r2 = 0; r2 < NR; ++r2) row[r2] = get(NR * r1 + r2);
      collapse_rows(row, half[r1]);
    }
#pragma unroll
    for (int b = 0; b < NC; ++b) {
      T col[NR], cc[NC];
#pragma unroll
      for (int r1 = 0; r1 < NR; ++r1) col[r1] = half[r1][b];
      collapse_rows(col, cc);
#pragma unroll
      for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
    }
  } else {
    // kept points: rows where r1 is real hold all r2; rows where r1 is complex
    // hold only the real r2
    T kept[NR][NR];
    int p = 0;
#pragma unroll
    for (int r1 = 0; r1 < NR; ++r1)
#pragma unroll
      for (int r2 = 0; r2 < NR; ++r2) {
        if (row_is_complex(r1) && row_is_complex(r2)) {
          kept[r1][r2] = T(0);
          continue;
        }
        kept[r1][r2] = get(p++);
      }
    // real r1: collapse along the horizontal axis
#pragma unroll
    for (int i = 0; i < NREAL; ++i) {
      T cc[NC];
      collapse_rows(kept[real_row(i)], cc);
#pragma unroll
      for (int b = 0; b < NC; ++b) comp[real_comp(i)][b] = cc[b];
    }
    // complex r1, real r2: collapse along the vertical axis
#pragma unroll
    for (int j = 0; j < NREAL; ++j) {
      T col[NR], cc[NC];
#pragma unroll
      for (int r1 = 0; r1 < NR; ++r1) col[r1] = kept[r1][real_row(j)];
      collapse_rows(col, cc);
#pragma unroll
      for (int a = 1; a <= 4; ++a) comp[a][real_comp(j)] = cc[a];
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
  T z[NC][M];
#pragma unroll
  for (int a = 0; a < NC; ++a) inv_outputs(comp[a], z[a]);
#pragma unroll
  for (int o2 = 0; o2 < M; ++o2) {
    T col[NC], y[M];
#pragma unroll
    for (int a = 0; a < NC; ++a) col[a] = z[a][o2];
    inv_outputs(col, y);
#pragma unroll
    for (int o1 = 0; o1 < M; ++o1) out[o1][o2] = y[o1];
  }
  }
}

// ---- output transform, streaming form ------------------------------------------

// f(integral_constant<int, 0>), ..., f(integral_constant<int, N-1>): a loop whose index is a
// compile-time constant inside the body
template <typename F, int... I>
SFC_HD void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
SFC_HD void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}
// The product at processing position J: next(integral_constant<int, J>) if the source takes
// its position as a compile-time constant, else next() (sources that count for themselves).
template <int J, typename F>
SFC_HD auto take_product(F&& next) {
  if constexpr (std::is_invocable_v<F, std::integral_constant<int, J>>)
    return next(std::integral_constant<int, J>{});
  else
    return next();
}

// Consumes the P products of one (tile, filter) pair in the processing order of
// Order<ALG> (next() returns the following product, already scaled) and leaves
// z[b][o1]: horizontal component b, vertical output o1, times 6.  Each group
// collapses at once: product-rule post-additions, Hermitian recombination, inverse
// symbolic DFT-6 with the corrections along the vertical axis.
// SFC-4, first part: the products of the four real columns (7 each, processing positions
// 0 .. 27) give z[0], z[1], z[4], z[5].
template <int ALG, typename T, typename F>
SFC_HD void stream_vertical4_real(F&& next, T (&z)[6][4]) {
  constexpr int NR = 7, NC = 6;
  static_for<4>([&](auto jc) {
    constexpr int j = decltype(jc)::value;
    T col[NR], cc[NC];
    static_for<NR>([&](auto rc) {
      constexpr int r1 = decltype(rc)::value;
      col[r1] = take_product<NR * j + r1>(next);
    });
    collapse4_rows(col, cc);
    inv4_outputs(cc, z[real_comp4(j)]);
  });
}

// SFC-4, second part: the products of the complex column group (positions 28 on; Eq. DFT4M)
// give z[2], z[3].
template <int ALG, typename T, typename F>
SFC_HD void stream_vertical4_complex(F&& next, T (&z)[6][4]) {
  constexpr int NR = 7, NC = 6, NREAL = 4;
  constexpr int J0 = NR * NREAL;  // positions of the real columns come first
  T c0[NC], c1[NC];
  if constexpr (!AlgTraits<ALG>::kHermitian) {
    T h0[NR], h1[NR];
    static_for<NR>([&](auto rc) {
      constexpr int r1 = decltype(rc)::value;
      const T m2 = take_product<J0 + 3 * r1>(next), m1 = take_product<J0 + 3 * r1 + 1>(next),
              m0 = take_product<J0 + 3 * r1 + 2>(next);  // rows a0 + a1, a1, a0
      h0[r1] = m0 - m1;
      h1[r1] = m2 - m0 - m1;
    });
    collapse4_rows(h0, c0);
    collapse4_rows(h1, c1);
  } else {
    static_for<NREAL>([&](auto jc) {
      constexpr int j = decltype(jc)::value;
      const T m2 = take_product<J0 + 3 * j>(next), m1 = take_product<J0 + 3 * j + 1>(next),
              m0 = take_product<J0 + 3 * j + 2>(next);
      c0[real_comp4(j)] = m0 - m1;
      c1[real_comp4(j)] = m2 - m0 - m1;
    });
    T m[6];
    static_for<6>([&](auto ic) {
      constexpr int i = decltype(ic)::value;
      m[i] = take_product<J0 + 3 * NREAL + i>(next);
    });
    const T uo0 = m[0] - m[1], uo1 = m[2] - m[0] - m[1];
    const T vo0 = m[3] - m[4], vo1 = m[5] - m[3] - m[4];
    c0[2] = Half<T>::apply(uo0 + vo0);  // o00
    c0[3] = Half<T>::apply(uo1 + vo1);  // o10
    c1[2] = Half<T>::apply(uo1 - vo1);  // o01
    c1[3] = Half<T>::apply(vo0 - uo0);  // o11
  }
  inv4_outputs(c0, z[2]);
  inv4_outputs(c1, z[3]);
}

template <int ALG, typename T, typename F>
SFC_HD void stream_vertical(F&& next, T (&z)[AlgTraits<ALG>::NC][AlgTraits<ALG>::M]) {
  using Tr = AlgTraits<ALG>;
  constexpr int NR = Tr::NR, NC = Tr::NC, NREAL = Tr::NREAL;
  if constexpr (Tr::kFamily == 4) {
    // SFC-4: four real columns, then the one complex column group
    stream_vertical4_real<ALG, T>(next, z);
    stream_vertical4_complex<ALG, T>(next, z);
    return;
  } else {
  static_for<NREAL>([&](auto jc) {
    constexpr int j = decltype(jc)::value;
    T col[NR], cc[NC];
    static_for<NR>([&](auto rc) {
      constexpr int r1 = decltype(rc)::value;
      col[r1] = take_product<NR * j + r1>(next);
    });
    collapse_rows(col, cc);
    inv_outputs(cc, z[real_comp(j)]);
  });
  // the two complex column groups: 3 NR positions each (nested), or 3 NREAL + 12 (Hermitian)
  constexpr int GSZ = Tr::kHermitian ? 3 * NREAL + 12 : 3 * NR;
  static_for<2>([&](auto gc) {
    constexpr int g2 = decltype(gc)::value;
    constexpr int J0 = NREAL * NR + g2 * GSZ;
    T c0[NC], c1[NC];
    if constexpr (!Tr::kHermitian) {
      T h0[NR], h1[NR];
      static_for<NR>([&](auto rc) {
        constexpr int r1 = decltype(rc)::value;
        const T m0 = take_product<J0 + 3 * r1>(next), m1 = take_product<J0 + 3 * r1 + 1>(next),
                m2 = take_product<J0 + 3 * r1 + 2>(next);
        h0[r1] = m0 - m1;
        h1[r1] = m2 - m0;
      });
      collapse_rows(h0, c0);
      collapse_rows(h1, c1);
    } else {
      static_for<NREAL>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const T m0 = take_product<J0 + 3 * j>(next), m1 = take_product<J0 + 3 * j + 1>(next),
                m2 = take_product<J0 + 3 * j + 2>(next);
        c0[real_comp(j)] = m0 - m1;
        c1[real_comp(j)] = m2 - m0;
      });
      static_for<2>([&](auto g1c) {
        constexpr int g1 = decltype(g1c)::value;
        T m[6];
        static_for<6>([&](auto ic) {
          constexpr int i = decltype(ic)::value;
          m[i] = take_product<J0 + 3 * NREAL + 6 * g1 + i>(next);
        });
        hermitian_collapse(m, c0[1 + 2 * g1], c0[2 + 2 * g1], c1[1 + 2 * g1], c1[2 + 2 * g1]);
      });
    }
    inv_outputs(c0, z[1 + 2 * g2]);
    inv_outputs(c1, z[2 + 2 * g2]);
  });
  }
}

// Output row o1 of the pair: the inverse along the horizontal axis (times 36 overall).
template <int ALG, typename T>
SFC_HD void stream_row(const T (&z)[AlgTraits<ALG>::NC][AlgTraits<ALG>::M], int o1,
                       T (&out)[AlgTraits<ALG>::M]) {
  constexpr int NC = AlgTraits<ALG>::NC;
  T zc[NC];
#pragma unroll
  for (int b = 0; b < NC; ++b) zc[b] = z[b][o1];
  if constexpr (AlgTraits<ALG>::kFamily == 4)
    inv4_outputs(zc, out);
  else
    inv_outputs(zc, out);
}

}  // namespace sfc
