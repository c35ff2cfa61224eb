// Counts the arithmetic operations of the add networks in sfc_points.hpp with a
// counting number type, per input (tile, channel) item and per output (tile, filter)
// pair, for every algorithm.  Prints "alg input_adds output_ops".
// bench.py's vector-ALU roofline uses these counts (plus 3 operations per point for the
// rounding to int8, 2 per point for the int32 -> float conversion and scaling, and one
// multiplication per output for the activation scale).
#include <cstdio>

#include "../../paper_2407_02913_amd/csrc/sfc_points.hpp"

static long g_ops = 0;
struct Op {
  double v;
  Op() : v(0) {}
  Op(double x) : v(x) {}
  Op(int x) : v(x) {}
};
static Op operator+(Op a, Op b) { ++g_ops; return Op(a.v + b.v); }
static Op operator-(Op a, Op b) { ++g_ops; return Op(a.v - b.v); }
static Op operator*(Op a, Op b) { ++g_ops; return Op(a.v * b.v); }
static Op operator-(Op a) { return Op(-a.v); }  // folds into the consuming add/sub
static Op& operator+=(Op& a, Op b) { ++g_ops; a.v += b.v; return a; }
namespace sfc {
template <>
struct Third<Op> {
  static Op apply(Op v) { ++g_ops; return Op(v.v / 3.0); }
};
template <>
struct Half<Op> {
  static Op apply(Op v) { ++g_ops; return Op(v.v / 2.0); }
};
}  // namespace sfc

using namespace sfc;

template <int ALG>
void count() {
  using Tr = AlgTraits<ALG>;
  constexpr int NI = Tr::NI, NC = Tr::NC, M = Tr::M;
  // input: rows, columns, points
  g_ops = 0;
  Op x[NI][NI], half[NI][NC], comp[NC][NC];
  for (int i = 0; i < NI; ++i) fwd_input<NI, NC>(x[i], half[i]);
  for (int b = 0; b < NC; ++b) {
    Op col[NI], cc[NC];
    for (int i = 0; i < NI; ++i) col[i] = half[i][b];
    fwd_input<NI, NC>(col, cc);
    for (int a = 0; a < NC; ++a) comp[a][b] = cc[a];
  }
  long pts = 0;
  for_each_point<ALG>(comp, [&](int, Op) { ++pts; });
  const long in_ops = g_ops;
  // output: streaming vertical pass, then one horizontal pass per output row
  g_ops = 0;
  Op z[NC][M];
  stream_vertical<ALG, Op>([&]() { return Op(1.0); }, z);
  for (int o1 = 0; o1 < M; ++o1) {
    Op out[M];
    stream_row<ALG, Op>(z, o1, out);
  }
  std::printf("%d %ld %ld %ld\n", ALG, pts, in_ops, g_ops);
}

int main() {
  count<0>();
  count<1>();
  count<2>();
  count<3>();
  count<4>();
  count<5>();
  return 0;
}
