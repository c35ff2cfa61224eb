// Host-side dump of the linear maps realized by the kernels' add networks
// (sfc_points.hpp), so that a CPU test can compare them with the oracle's
// matrices.  Prints, for every ALG (0: 6x6/88, 1: 6x6/100, 2: 7x7/132, 3: 7x7/144,
// 4: 4x4/46, 5: 4x4/49, 6: 6x6 with 5x5 filter/184, 7: the same/196, 8: 4x4 with 7x7
// filter/184, 9: the same/196):
//   B <alg> <p> <NI*NI ints>   input transform row p  (impulse responses)
//   G <alg> <p> <R*R ints>     filter transform row p
//   A <alg> <p> <M*M ints>     output transform row p (times 36; times 16 for 4x4)
//   S <alg> <p> <M*M ints>     the same row through the streaming form of the fused kernels
//                              (products fed in processing order, stream_vertical + stream_row)
#include <cmath>
#include <cstdio>
#include <vector>

#include "../../paper_2407_02913_amd/csrc/sfc_points.hpp"

using namespace sfc;

template <int ALG>
void dump() {
  using Tr = AlgTraits<ALG>;
  constexpr int P = Tr::P, NI = Tr::NI, NC = Tr::NC, M = Tr::M, R = Tr::R;
  std::vector<std::vector<int>> B(P, std::vector<int>(NI * NI)), G(P, std::vector<int>(R * R)),
      A(P, std::vector<int>(M * M));
  for (int i = 0; i < NI; ++i)
    for (int j = 0; j < NI; ++j) {
      int x[NI][NI] = {};
      x[i][j] = 1;
      int half[NI][NC], comp[NC][NC];
      for (int r = 0; r < NI; ++r) fwd_input<NI, NC>(x[r], half[r]);
      for (int b = 0; b < NC; ++b) {
        int col[NI], cc[NC];
        for (int r = 0; r < NI; ++r) col[r] = half[r][b];
        fwd_input<NI, NC>(col, cc);
        for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
      }
      for_each_point<ALG>(comp, [&](int p, int v) { B[p][i * NI + j] = v; });
    }
  for (int i = 0; i < R; ++i)
    for (int j = 0; j < R; ++j) {
      int f[R][R] = {};
      f[i][j] = 1;
      int half[R][NC], comp[NC][NC];
      for (int r = 0; r < R; ++r) fwd_filter<R, NC>(f[r], half[r]);
      for (int b = 0; b < NC; ++b) {
        int col[R], cc[NC];
        for (int r = 0; r < R; ++r) col[r] = half[r][b];
        fwd_filter<R, NC>(col, cc);
        for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
      }
      for_each_point<ALG>(comp, [&](int p, int v) { G[p][i * R + j] = v; });
    }
  for (int q = 0; q < P; ++q) {
    float out[M][M];
    output_transform<ALG, float>([&](int p) { return p == q ? 3.0f : 0.0f; }, out);
    for (int o = 0; o < M * M; ++o) A[q][o] = (int)std::lround(out[o / M][o % M] / 3.0f);
  }
  constexpr Order<ALG> order{};
  for (int q = 0; q < P; ++q) {
    int j = 0;
    auto next = [&]() -> float { return order.pt[j++] == q ? 3.0f : 0.0f; };
    float z[NC][M];
    stream_vertical<ALG, float>(next, z);
    std::printf("S %d %d", ALG, q);
    for (int o1 = 0; o1 < M; ++o1) {
      float out[M];
      stream_row<ALG, float>(z, o1, out);
      for (int o2 = 0; o2 < M; ++o2) std::printf(" %d", (int)std::lround(out[o2] / 3.0f));
    }
    std::printf("\n");
    if (q == 0 && j != P) std::printf("S %d -1 %d\n", ALG, j);  // must consume exactly P products
  }
  for (int j = P; j < Order<ALG>::PP; ++j)
    if (order.pt[j] != -1) std::printf("S %d -2 %d\n", ALG, j);
  for (int p = 0; p < P; ++p) {
    std::printf("B %d %d", ALG, p);
    for (int v : B[p]) std::printf(" %d", v);
    std::printf("\nG %d %d", ALG, p);
    for (int v : G[p]) std::printf(" %d", v);
    std::printf("\nA %d %d", ALG, p);
    for (int v : A[p]) std::printf(" %d", v);
    std::printf("\n");
  }
}

int main() {
  dump<0>();
  dump<1>();
  dump<2>();
  dump<3>();
  dump<4>();
  dump<5>();
  dump<6>();
  dump<7>();
  dump<8>();
  dump<9>();
  return 0;
}
