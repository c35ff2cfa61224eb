// Host-side dump of the linear maps realized by the kernels' add networks
// (sfc_points.hpp), so that a CPU test can compare them with the oracle's
// matrices.  Prints, for ALG 0 (88 points) and 1 (100 points):
//   B <alg> <p> <64 ints>   input transform row p  (impulse responses)
//   G <alg> <p> <9 ints>    filter transform row p
//   A <alg> <p> <36 ints>   output transform row p (times 36)
#include <cmath>
#include <cstdio>

#include "../../paper_2407_02913_amd/csrc/sfc_points.hpp"

using namespace sfc;

template <int ALG>
void dump() {
  constexpr int P = AlgTraits<ALG>::P;
  static int B[P][64], G[P][9], A[P][36];
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 8; ++j) {
      int x[8][8] = {};
      x[i][j] = 1;
      int half[8][8], comp[8][8];
      for (int r = 0; r < 8; ++r) fwd8(x[r], half[r]);
      for (int b = 0; b < 8; ++b) {
        int col[8], cc[8];
        for (int r = 0; r < 8; ++r) col[r] = half[r][b];
        fwd8(col, cc);
        for (int a = 0; a < 8; ++a) comp[a][b] = cc[a];
      }
      for_each_point<ALG>(comp, [&](int p, int v) { B[p][i * 8 + j] = v; });
    }
  for (int i = 0; i < 3; ++i)
    for (int j = 0; j < 3; ++j) {
      int f[3][3] = {};
      f[i][j] = 1;
      int half[3][8], comp[8][8];
      for (int r = 0; r < 3; ++r) fwd3(f[r], half[r]);
      for (int b = 0; b < 8; ++b) {
        int col[3] = {half[0][b], half[1][b], half[2][b]}, cc[8];
        fwd3(col, cc);
        for (int a = 0; a < 8; ++a) comp[a][b] = cc[a];
      }
      for_each_point<ALG>(comp, [&](int p, int v) { G[p][i * 3 + j] = v; });
    }
  for (int q = 0; q < P; ++q) {
    float out[6][6];
    output_transform<ALG, float>([&](int p) { return p == q ? 3.0f : 0.0f; }, out);
    for (int o = 0; o < 36; ++o) A[q][o] = (int)std::lround(out[o / 6][o % 6] / 3.0f);
  }
  for (int p = 0; p < P; ++p) {
    std::printf("B %d %d", ALG, p);
    for (int i = 0; i < 64; ++i) std::printf(" %d", B[p][i]);
    std::printf("\nG %d %d", ALG, p);
    for (int i = 0; i < 9; ++i) std::printf(" %d", G[p][i]);
    std::printf("\nA %d %d", ALG, p);
    for (int i = 0; i < 36; ++i) std::printf(" %d", A[p][i]);
    std::printf("\n");
  }
  // integer path of the output transform on a valid product vector: a random
  // integer image of the forward maps must come back exactly (x36)
}

int main() {
  dump<0>();
  dump<1>();
  return 0;
}
