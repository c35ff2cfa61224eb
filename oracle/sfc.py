"""Plain numpy oracle for quantized 3x3 (and 5x5, 7x7) convolution by Symbolic Fourier Convolution.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct CPU
statement of the method (arXiv 2407.02913).  It is imported by ``tests/``, by
``__graft_entry__.smoke()`` and by the ``cpu_baseline`` leg of ``bench.py`` and
by nothing else; it never imports the HIP library, and the HIP library never
calls it.  All integer stages are computed exactly (int64, or float64 matmuls
whose every partial sum is an integer below 2**53, which is asserted); all
floating-point stages are float64.

What is the definition and what is the algorithm
------------------------------------------------
* ``direct_conv``            -- the *definition* of the result (cross-correlation,
                               stride 1, zero padding (R-1)/2 for an RxR filter).  In
                               exact-integer mode SFC reaches exactly this result.
* ``sfc6_1d`` ...            -- the 1-D matrices of SFC-6(6,3) as printed in
                               Appendix A (one erratum, see ``BT_PRINTED_ROW7``).
* ``sfc6_1d(6, 5)``          -- SFC-6(6x6,5x5): B^T and G as printed in Appendix A, A
                               the one matrix that fits them (the print of A is
                               unusable); re-derived by ``integrate_1d_5tap``.
* ``sfc6_1d(4, 7)``          -- SFC-6(4x4,7x7) of Table 1: no matrices are printed; they are
                               derived by ``integrate_1d_ten`` (the same five steps, which
                               for 6 outputs and 5 taps reproduce Appendix A's print).
                               Its multiplication count (184 / 196) is PARITY UNPINNED
                               against Table 1, whose 21.99 % is no whole number of
                               multiplications; the results are pinned by the bilinear
                               identity, brute force and ``direct_conv``.
* ``nested_2d``              -- the 2-D form of Eq. (1): Kronecker products,
                               10*10 = 100 multiplications per 6x6 tile.
* ``hermitian_2d``           -- the 88-multiplication form.  Appendix A only
                               states the count; the construction used here is
                               written out in the docstring.
* ``conv_exact``             -- Eq. (1) with exact integers.
* ``conv_requant``           -- Eq. (1) with the frequency-wise / channel-wise
                               transform-domain quantizer of Sec. 5.

Pins (see tests/test_oracle_*.py): printed matrices (tests/golden), the
bilinear identity sum_p A[p,o] B[p,i] G[p,r] = 6 [i = o + r], numpy's FFT for the
symbolic DFT-6, complex multiplication for the 3-multiplication product rule,
brute-force correlation on tiny inputs, torch's conv2d for ``direct_conv``, the
multiplication counts 100/88 and the ratios 3.68x / 2.25x, and bit-exact
equality of ``conv_exact`` with ``direct_conv``.  ``conv_requant`` is an
approximation with no printed values: it is pinned by reduction to
``conv_exact`` (unit scales, power-of-two scales), by hand-computed values of
the quantizer, and by its error against ``direct_conv`` shrinking by about 2x
per extra bit.
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------------------
# Sec. 4.1, "1) DFT-6": symbolic DFT with s = exp(j*pi/3), s^2 = s - 1.
# ---------------------------------------------------------------------------

#: F_6 of Eq. (DFT6): rows are [X0, X1.a0, X1.a1, X2.a0, X2.a1, X3] where a
#: complex point is the first-order polynomial a0 + a1*s.
F6 = np.array(
    [
        [1, 1, 1, 1, 1, 1],
        [1, 1, 0, -1, -1, 0],
        [0, -1, -1, 0, 1, 1],
        [1, 0, -1, 1, 0, -1],
        [0, -1, 1, 0, -1, 1],
        [1, -1, 1, -1, 1, -1],
    ],
    dtype=np.int64,
)

#: iF_6 (numerators; the common factor is 1/6), as printed after Eq. (DFT6).
#: Row c gives the weight of symbol component c in each of the six samples.
#: Read this way, IF6.T @ F6 == 6 * (cyclic advance by one sample): the printed
#: matrix carries the one-sample alignment that the integrated A matrix needs.
IF6 = np.array(
    [
        [1, 1, 1, 1, 1, 1],
        [1, -1, -2, -1, 1, 2],
        [-1, -2, -1, 1, 2, 1],
        [-1, -1, 2, -1, -1, 2],
        [-2, 1, 1, -2, 1, 1],
        [-1, 1, -1, 1, -1, 1],
    ],
    dtype=np.int64,
)

S_ROOT = np.exp(1j * np.pi / 3.0)  # the symbol s, only ever used by checks


def s6_to_complex(sym: np.ndarray) -> np.ndarray:
    """S_6 of Eq. (DFT6): symbolic components -> the six complex DFT values.

    ``sym`` has the six F_6 components on axis 0.  Returns X_0..X_5 with
    X_5 = conj(X_1) and X_4 = conj(X_2) (written in the paper as a0 - a1*s^2,
    since conj(s) = -s^2 = 1 - s).
    """
    sym = np.asarray(sym, dtype=np.float64)
    x0, a10, a11, a20, a21, x3 = sym
    x1 = a10 + a11 * S_ROOT
    x2 = a20 + a21 * S_ROOT
    x5 = a10 + a11 * (-(S_ROOT**2))
    x4 = a20 + a21 * (-(S_ROOT**2))
    return np.stack([x0 + 0j, x1, x2, x3 + 0j, x4, x5])


def poly_mul_s6(a: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Eq. (DFT6M): (a0 + a1 s)(w0 + w1 s) = o0 + o1 s with three multiplications."""
    a0, a1 = a
    w0, w1 = w
    m0 = a0 * w0
    m1 = a1 * w1
    m2 = (a0 + a1) * (w0 + w1)
    return np.stack([m0 - m1, m2 - m0])


def sft6_butterfly(z):
    """F_6 z through the DFT-2 x DFT-3 decomposition of Sec. 4.1.

    Returns (the six components in F_6's row order, number of additions).  A
    subtraction, or an addition of a negated operand, counts as one addition,
    as the paper counts them.
    """
    z = [np.asarray(v, dtype=np.int64) for v in z]
    e = [z[i] + z[i + 3] for i in range(3)]
    d = [z[i] - z[i + 3] for i in range(3)]
    adds = 6
    x0 = e[0] + e[1] + e[2]
    a20, a21 = e[0] - e[2], e[2] - e[1]
    x3 = d[0] - d[1] + d[2]
    a10, a11 = d[0] + d[1], -d[1] - d[2]
    adds += 2 + 2 + 2 + 2
    return np.stack([x0, a10, a11, a20, a21, x3]), adds


# ---------------------------------------------------------------------------
# Appendix A: SFC-6(6x6, 3x3), polynomial multiplication integrated.
# Row roles (0-based): 0 -> k=0 (real); 1,2,3 -> k=1 as (a0, a1, a0+a1);
# 4,5,6 -> k=2 likewise; 7 -> k=3 (real); 8, 9 -> the two correction terms of
# Sec. 4.2 (x0 - x6 paired with f0 -> output 0, x7 - x1 paired with f2 -> output 5).
# ---------------------------------------------------------------------------

#: Row 7 of B^T exactly as printed.  It breaks the bilinear identity; the k=3
#: row of F_6 (alternating signs, as also printed for SFC-6(7x7,3x3)) is used.
BT_PRINTED_ROW7 = np.array([0, 1, -1, 1, 1, -1, 1, 0], dtype=np.int64)

BT_1D = np.array(
    [
        [0, 1, 1, 1, 1, 1, 1, 0],
        [0, 1, 1, 0, -1, -1, 0, 0],
        [0, 0, -1, -1, 0, 1, 1, 0],
        [0, 1, 0, -1, -1, 0, 1, 0],
        [0, 1, 0, -1, 1, 0, -1, 0],
        [0, 0, -1, 1, 0, -1, 1, 0],
        [0, 1, -1, 0, 1, -1, 0, 0],
        [0, 1, -1, 1, -1, 1, -1, 0],  # erratum: printed as BT_PRINTED_ROW7
        [1, 0, 0, 0, 0, 0, -1, 0],
        [0, -1, 0, 0, 0, 0, 0, 1],
    ],
    dtype=np.int64,
)

G_1D = np.array(
    [
        [1, 1, 1],
        [0, 1, 1],
        [-1, -1, 0],
        [-1, 0, 1],
        [-1, 0, 1],
        [1, -1, 0],
        [0, -1, 1],
        [1, -1, 1],
        [1, 0, 0],
        [0, 0, 1],
    ],
    dtype=np.int64,
)

#: Numerators of A; the printed matrix carries the factor 1/6.
A_1D = np.array(
    [
        [1, 1, 1, 1, 1, 1],
        [2, 1, -1, -2, -1, 1],
        [-1, 1, 2, 1, -1, -2],
        [-1, -2, -1, 1, 2, 1],
        [1, -2, 1, 1, -2, 1],
        [1, 1, -2, 1, 1, -2],
        [-2, 1, 1, -2, 1, 1],
        [-1, 1, -1, 1, -1, 1],
        [6, 0, 0, 0, 0, 0],
        [0, 0, 0, 0, 0, 6],
    ],
    dtype=np.int64,
)
A_1D_DEN = 6

# ---------------------------------------------------------------------------
# Appendix A: SFC-6(7x7, 3x3) (also Sec. 4.2, whose printed A has two garbled
# entries; the appendix print satisfies the bilinear identity and is used).
# Rows 0..7 as above, acting on x1..x6 of nine samples; four correction rows:
#   8: (x0 - x6) f0 -> output 0        9: (x7 - x1) f2 -> output 5
#  10: (x7 - x1) f1 -> output 6       11: (x8 - x2) f2 -> output 6
# Output 6 is the cyclic output 0 (same column of A) plus its two corrections:
# the tile is stretched from 6 to 7 outputs with two more multiplications.
# ---------------------------------------------------------------------------
BT7_1D = np.array(
    [
        [0, 1, 1, 1, 1, 1, 1, 0, 0],
        [0, 1, 1, 0, -1, -1, 0, 0, 0],
        [0, 0, -1, -1, 0, 1, 1, 0, 0],
        [0, 1, 0, -1, -1, 0, 1, 0, 0],
        [0, 1, 0, -1, 1, 0, -1, 0, 0],
        [0, 0, -1, 1, 0, -1, 1, 0, 0],
        [0, 1, -1, 0, 1, -1, 0, 0, 0],
        [0, 1, -1, 1, -1, 1, -1, 0, 0],
        [1, 0, 0, 0, 0, 0, -1, 0, 0],
        [0, -1, 0, 0, 0, 0, 0, 1, 0],
        [0, -1, 0, 0, 0, 0, 0, 1, 0],
        [0, 0, -1, 0, 0, 0, 0, 0, 1],
    ],
    dtype=np.int64,
)

G7_1D = np.array(
    [
        [1, 1, 1],
        [0, 1, 1],
        [-1, -1, 0],
        [-1, 0, 1],
        [-1, 0, 1],
        [1, -1, 0],
        [0, -1, 1],
        [1, -1, 1],
        [1, 0, 0],
        [0, 0, 1],
        [0, 1, 0],
        [0, 0, 1],
    ],
    dtype=np.int64,
)

A7_1D = np.array(
    [
        [1, 1, 1, 1, 1, 1, 1],
        [2, 1, -1, -2, -1, 1, 2],
        [-1, 1, 2, 1, -1, -2, -1],
        [-1, -2, -1, 1, 2, 1, -1],
        [1, -2, 1, 1, -2, 1, 1],
        [1, 1, -2, 1, 1, -2, 1],
        [-2, 1, 1, -2, 1, 1, -2],
        [-1, 1, -1, 1, -1, 1, -1],
        [6, 0, 0, 0, 0, 0, 0],
        [0, 0, 0, 0, 0, 6, 0],
        [0, 0, 0, 0, 0, 0, 6],
        [0, 0, 0, 0, 0, 0, 6],
    ],
    dtype=np.int64,
)

# ---------------------------------------------------------------------------
# Appendix A: SFC-6(6x6, 5x5).  B^T (14x10) and G (14x5) are used as printed: rows 0..7 are
# the rows of SFC-6(6x6,3x3) acting on the inner samples x2..x7, with the filter's symbolic
# DFT aligned as G_k = sum_r f_r s^{k (r - 4)}; six correction rows, each "wanted sample
# minus the sample the cyclic convolution supplies" times one tap:
#    8: (x0 - x6) f0 -> output 0      9: (x1 - x7) f0 -> output 1     10: (x1 - x7) f1 -> output 0
#   11: (x8 - x2) f3 -> output 5     12: (x8 - x2) f4 -> output 4     13: (x9 - x3) f4 -> output 5
# A is printed with seven columns for six outputs and cannot be right as it stands.  B^T and
# G determine A uniquely (the 14 bilinear forms B^T[p,i] G[p,r] are linearly independent), and
# that unique A is used: in rows 0..7 it equals the first six printed columns; the
# correction rows send each product to the output named above.
# ---------------------------------------------------------------------------
BT65_1D = np.array(
    [
        [0, 0, 1, 1, 1, 1, 1, 1, 0, 0],
        [0, 0, 1, 1, 0, -1, -1, 0, 0, 0],
        [0, 0, 0, -1, -1, 0, 1, 1, 0, 0],
        [0, 0, 1, 0, -1, -1, 0, 1, 0, 0],
        [0, 0, 1, 0, -1, 1, 0, -1, 0, 0],
        [0, 0, 0, -1, 1, 0, -1, 1, 0, 0],
        [0, 0, 1, -1, 0, 1, -1, 0, 0, 0],
        [0, 0, 1, -1, 1, -1, 1, -1, 0, 0],
        [1, 0, 0, 0, 0, 0, -1, 0, 0, 0],
        [0, 1, 0, 0, 0, 0, 0, -1, 0, 0],
        [0, 1, 0, 0, 0, 0, 0, -1, 0, 0],
        [0, 0, -1, 0, 0, 0, 0, 0, 1, 0],
        [0, 0, -1, 0, 0, 0, 0, 0, 1, 0],
        [0, 0, 0, -1, 0, 0, 0, 0, 0, 1],
    ],
    dtype=np.int64,
)

G65_1D = np.array(
    [
        [1, 1, 1, 1, 1],
        [-1, -1, 0, 1, 1],
        [1, 0, -1, -1, 0],
        [0, -1, -1, 0, 1],
        [0, 1, -1, 0, 1],
        [-1, 0, 1, -1, 0],
        [-1, 1, 0, -1, 1],
        [1, -1, 1, -1, 1],
        [1, 0, 0, 0, 0],
        [1, 0, 0, 0, 0],
        [0, 1, 0, 0, 0],
        [0, 0, 0, 1, 0],
        [0, 0, 0, 0, 1],
        [0, 0, 0, 0, 1],
    ],
    dtype=np.int64,
)

A65_1D = np.array(  # numerators, A = A65_1D / 6
    [
        [1, 1, 1, 1, 1, 1],
        [1, -1, -2, -1, 1, 2],
        [1, 2, 1, -1, -2, -1],
        [-2, -1, 1, 2, 1, -1],
        [-2, 1, 1, -2, 1, 1],
        [1, -2, 1, 1, -2, 1],
        [1, 1, -2, 1, 1, -2],
        [1, -1, 1, -1, 1, -1],
        [6, 0, 0, 0, 0, 0],
        [0, 6, 0, 0, 0, 0],
        [6, 0, 0, 0, 0, 0],
        [0, 0, 0, 0, 0, 6],
        [0, 0, 0, 0, 6, 0],
        [0, 0, 0, 0, 0, 6],
    ],
    dtype=np.int64,
)

# SFC-4(4x4,3x3), Appendix A (first set of matrices): s = j, four-point symbolic DFT of the
# inner samples x1..x4 plus one correction row per wrapped output.  Row order as printed:
# X0, X2 (both real), then the complex point X1 = a0 + a1 j as (a0 + a1, a1, a0), then the
# corrections (x0 - x4) f0 -> output 0 and (x5 - x1) f2 -> output 3.
BT4_1D = np.array(
    [
        [0, 1, 1, 1, 1, 0],
        [0, -1, 1, -1, 1, 0],
        [0, 1, -1, -1, 1, 0],
        [0, 0, -1, 0, 1, 0],
        [0, 1, 0, -1, 0, 0],
        [1, 0, 0, 0, -1, 0],
        [0, -1, 0, 0, 0, 1],
    ],
    dtype=np.int64,
)
G4_1D = np.array(
    [[1, 1, 1], [1, -1, 1], [1, -1, -1], [1, 0, -1], [0, -1, 0], [1, 0, 0], [0, 0, 1]],
    dtype=np.int64,
)
A4_1D = np.array(  # numerators, A = A4_1D / 4
    [
        [1, 1, 1, 1],
        [1, -1, 1, -1],
        [0, 2, 0, -2],
        [2, -2, -2, 2],
        [-2, -2, 2, 2],
        [4, 0, 0, 0],
        [0, 0, 0, 4],
    ],
    dtype=np.int64,
)
A4_1D_DEN = 4
SFC4_COMPLEX_GROUP = (4, 3, 2)  # (a0 row, a1 row, a0+a1 row) of the single complex point

TILE_OUT = 6  # M of the primary variant SFC-6(6x6,3x3)
TILE_IN = 8  # M + R - 1
KERNEL = 3  # R
COMPLEX_GROUPS = ((1, 2, 3), (4, 5, 6))  # (a0 row, a1 row, a0+a1 row), both variants


def sfc6_1d(m: int = 6, r: int = 3):
    """The three 1-D matrices of SFC-6(m,r): (B^T, G, A numerators, 6).

    r = 3, m = 6: B^T 10x8, G 10x3, A 10x6.  r = 3, m = 7: B^T 12x9, G 12x3, A 12x7.
    r = 5, m = 6: B^T 14x10, G 14x5, A 14x6.
    r = 7, m = 4: B^T 14x10, G 14x7, A 14x4 (derived, not printed: ``integrate_1d_ten``).
    """
    if r == 7:
        if m != 4:
            raise ValueError(m)
        return integrate_1d_ten(4, 7)
    if r == 5:
        if m != 6:
            raise ValueError(m)
        return BT65_1D.copy(), G65_1D.copy(), A65_1D.copy(), A_1D_DEN
    if r != 3:
        raise ValueError(r)
    if m == 6:
        return BT_1D.copy(), G_1D.copy(), A_1D.copy(), A_1D_DEN
    if m == 7:
        return BT7_1D.copy(), G7_1D.copy(), A7_1D.copy(), A_1D_DEN
    raise ValueError(m)


def integrate_1d(m: int = 6):
    """Re-derive B^T, G, A of SFC-6(m,3), m = 6 or 7, from Sec. 4.1-4.2 instead of reading them.

    Steps, in the paper's order:
      1. forward SFT-6 (F_6) of the six inner samples x1..x6        (Eq. DFT6)
      2. the same symbolic DFT of the filter, aligned so that the cyclic
         result lands on the tile's outputs: G_k = sum_r f_r s^{k(r-2)}
      3. the 3-multiplication product rule folded into both matrices as an
         extra a0+a1 row per complex point                           (Eq. DFT6M)
      4. inverse transform iF_6, with the product rule's post-additions
         (o0 = m0 - m1, o1 = m2 - m0) folded into A's rows
      5. two correction terms that turn the wrapped outputs 0 and 5 of the
         cyclic convolution into linear-convolution outputs          (Sec. 4.2)
    Returns (B^T, G, A numerators, 6) in the same row order as Appendix A.
    """
    rows = 10 if m == 6 else 12
    bt = np.zeros((rows, m + 2), dtype=np.int64)
    g = np.zeros((rows, 3), dtype=np.int64)
    a = np.zeros((rows, m), dtype=np.int64)

    # powers of s as (c0, c1) with s^n = c0 + c1 s, using s^2 = s - 1
    def s_pow(n):
        c = np.array([1, 0], dtype=np.int64)
        n %= 6
        for _ in range(n):
            c = np.array([-c[1], c[0] + c[1]])  # (c0 + c1 s) s = -c1 + (c0 + c1) s
        return c

    # 1. rows of F_6 act on the inner samples (columns 1..6)
    comp_rows = {0: 0, 1: 1, 2: 2, 4: 3, 5: 4, 7: 5}  # B^T row -> F_6 row
    for brow, frow in comp_rows.items():
        bt[brow, 1:7] = F6[frow]
    # 2. filter DFT: G_k = sum_r f_r s^{k (r - 2)}
    for k, (r0, r1) in ((1, (1, 2)), (2, (4, 5))):
        for r in range(3):
            c = s_pow(k * (r - 2))
            g[r0, r] = c[0]
            g[r1, r] = c[1]
    g[0] = 1  # k = 0
    for r in range(3):  # k = 3: s^{3(r-2)} = (-1)^{r-2}
        g[7, r] = 1 if (r - 2) % 2 == 0 else -1
    # 3. Karatsuba-style sum rows
    for r0, r1, rs in COMPLEX_GROUPS:
        bt[rs] = bt[r0] + bt[r1]
        g[rs] = g[r0] + g[r1]
    # 4. inverse: y = sum_c IF6[c] * component_c, o0 = m0 - m1, o1 = m2 - m0
    a[0, :6] = IF6[0]
    a[7, :6] = IF6[5]
    for (r0, r1, rs), (c0, c1) in zip(COMPLEX_GROUPS, ((1, 2), (3, 4))):
        a[r0, :6] = IF6[c0] - IF6[c1]
        a[r1, :6] = -IF6[c0]
        a[rs, :6] = IF6[c1]
    # 5. corrections: output 0 wraps x6 where x0 is wanted (times f0); output 5
    # wraps x1 where x7 is wanted (times f2).  One multiplication each, and the
    # products are not divided by 6.
    bt[8, 0], bt[8, 6] = 1, -1
    g[8, 0] = 1
    a[8, 0] = 6
    bt[9, 7], bt[9, 1] = 1, -1
    g[9, 2] = 1
    a[9, 5] = 6
    if m == 7:
        # a seventh output: the cyclic result wraps output 6 onto output 0
        # (x6 f0 + x1 f1 + x2 f2), where x7 f1 and x8 f2 are wanted
        a[:8, 6] = a[:8, 0]
        bt[10, 7], bt[10, 1] = 1, -1
        g[10, 1] = 1
        a[10, 6] = 6
        bt[11, 8], bt[11, 2] = 1, -1
        g[11, 2] = 1
        a[11, 6] = 6
    return bt, g, a, 6


def integrate_1d_5tap():
    """Re-derive B^T, G, A of SFC-6(6x6,5x5) from Sec. 4.1-4.2 (same five steps as
    ``integrate_1d``): the cyclic part works on the six inner samples x2..x7 of ten, the
    filter's symbolic DFT is G_k = sum_r f_r s^{k (r - 4)}, and every (output o, tap r) whose
    sample x_{o+r} lies outside x2..x7 gets one correction row (x_{o+r} minus the inner
    sample six positions away, times f_r, added to output o); rows ordered by (r, o).
    Returns (B^T 14x10, G 14x5, A numerators 14x6, 6).
    """
    bt = np.zeros((14, 10), dtype=np.int64)
    g = np.zeros((14, 5), dtype=np.int64)
    a = np.zeros((14, 6), dtype=np.int64)

    def s_pow(n):
        c = np.array([1, 0], dtype=np.int64)
        for _ in range(n % 6):
            c = np.array([-c[1], c[0] + c[1]])
        return c

    for brow, frow in {0: 0, 1: 1, 2: 2, 4: 3, 5: 4, 7: 5}.items():
        bt[brow, 2:8] = F6[frow]
    for k, (r0, r1) in ((1, (1, 2)), (2, (4, 5))):
        for r in range(5):
            c = s_pow(k * (r - 4))
            g[r0, r], g[r1, r] = c[0], c[1]
    g[0] = 1
    for r in range(5):
        g[7, r] = 1 if (r - 4) % 2 == 0 else -1
    for r0, r1, rs in COMPLEX_GROUPS:
        bt[rs] = bt[r0] + bt[r1]
        g[rs] = g[r0] + g[r1]
    # the inverse: with this alignment the cyclic result of iF_6 comes out rotated by one
    # position (component products -> cyclic output (o + 1) mod 6 lands on output o)
    rot = [(o + 1) % 6 for o in range(6)]
    a[0] = IF6[0][rot]
    a[7] = IF6[5][rot]
    for (r0, r1, rs), (c0, c1) in zip(COMPLEX_GROUPS, ((1, 2), (3, 4))):
        a[r0] = IF6[c0][rot] - IF6[c1][rot]
        a[r1] = -IF6[c0][rot]
        a[rs] = IF6[c1][rot]
    row = 8
    for r in range(5):
        for o in range(6):
            i = o + r
            if 2 <= i <= 7:
                continue
            supplied = 2 + (i - 2) % 6
            bt[row, i], bt[row, supplied] = 1, -1
            g[row, r] = 1
            a[row, o] = 6
            row += 1
    assert row == 14
    return bt, g, a, 6


def integrate_1d_ten(m: int, r: int):
    """B^T, G, A of an SFC-6 algorithm on ten samples, m + r - 1 = 10, from Sec. 4.1-4.2:
    SFC-6(6,5) (Appendix A) and SFC-6(4,7) (Table 1, no matrices printed).

    The five steps of ``integrate_1d``, with the window and the alignment of the printed
    SFC-6(6,5) matrices:
      1. forward SFT-6 (F_6) of the six inner samples x2..x7                       (Eq. DFT6)
      2. the filter's symbolic DFT aligned on its last tap, G_k = sum_t f_t s^{k(t-(r-1))}
      3. one a0+a1 row per complex point                                           (Eq. DFT6M)
      4. iF_6 with the product rule's post-additions folded in; with that alignment the
         cyclic result for output o is the one iF_6 as printed delivers at position
         (o + r - 4) mod 6
      5. one correction row for every (tap t, output o) whose sample x_{o+t} lies outside
         x2..x7: (x_{o+t} minus the inner sample a multiple of six positions away) times
         f_t, added to output o; rows ordered by (t, o)                             (Sec. 4.2)
    For m = 4, r = 7 there are six such pairs -- (0,0) (0,1) (1,0) (5,3) (6,2) (6,3) -- so
    B^T is the printed B^T of SFC-6(6,5) and the algorithm has 8 + 6 = 14 rows.
    Returns (B^T, G, A numerators, 6).
    """
    if m + r - 1 != 10:
        raise ValueError((m, r))
    outside = [(t, o) for t in range(r) for o in range(m) if not 2 <= o + t <= 7]
    rows = 8 + len(outside)
    bt = np.zeros((rows, 10), dtype=np.int64)
    g = np.zeros((rows, r), dtype=np.int64)
    a = np.zeros((rows, m), dtype=np.int64)

    def s_pow(n):
        c = np.array([1, 0], dtype=np.int64)
        for _ in range(n % 6):
            c = np.array([-c[1], c[0] + c[1]])
        return c

    for brow, frow in {0: 0, 1: 1, 2: 2, 4: 3, 5: 4, 7: 5}.items():
        bt[brow, 2:8] = F6[frow]
    for k, (r0, r1) in ((1, (1, 2)), (2, (4, 5))):
        for t in range(r):
            c = s_pow(k * (t - (r - 1)))
            g[r0, t], g[r1, t] = c[0], c[1]
    g[0] = 1
    for t in range(r):
        g[7, t] = 1 if (t - (r - 1)) % 2 == 0 else -1
    for r0, r1, rs in COMPLEX_GROUPS:
        bt[rs] = bt[r0] + bt[r1]
        g[rs] = g[r0] + g[r1]
    rot = [(o + r - 4) % 6 for o in range(m)]
    a[0] = IF6[0][rot]
    a[7] = IF6[5][rot]
    for (r0, r1, rs), (c0, c1) in zip(COMPLEX_GROUPS, ((1, 2), (3, 4))):
        a[r0] = IF6[c0][rot] - IF6[c1][rot]
        a[r1] = -IF6[c0][rot]
        a[rs] = IF6[c1][rot]
    for row, (t, o) in enumerate(outside, start=8):
        i = o + t
        bt[row, i], bt[row, 2 + (i - 2) % 6] = 1, -1
        g[row, t] = 1
        a[row, o] = 6
    return bt, g, a, 6


# ---------------------------------------------------------------------------
# 2-D forms (Eq. 1: y = A^T [ (G f G^T) . (B^T x B) ] A )
# ---------------------------------------------------------------------------


def nested_2d(m: int = 6, r: int = 3):
    """Nested (Kronecker) 2-D form: 100 points per 6x6 tile, 144 per 7x7 tile (3x3 filter),
    196 per 6x6 tile with a 5x5 filter.

    Returns (B2 [P,(m+r-1)^2], G2 [P,r^2], A2 numerators [P,m^2], 36); point
    p = rows*p1 + p2 with p1 along the vertical (row) axis of the tile.
    """
    bt, g, a, den = sfc6_1d(m, r)
    return np.kron(bt, bt), np.kron(g, g), np.kron(a, a), den * den


def hermitian_2d(m: int = 6, r: int = 3):
    """88-point (6x6) / 132-point (7x7) / 184-point (6x6 outputs, 5x5 filter) 2-D form ("when Hermitian symmetry is fully considered", Appendix A).

    The paper states the count only.  Construction used here:

    * Every nested point in which at most one axis is a complex frequency is
      kept unchanged, in nested order (64 of the 100 points).
    * For each pair of complex frequencies (k1, k2) in {1,2}^2 the nested form
      spends 3*3 = 9 multiplications on the product of two elements of
      Z[s]/(s^2-s+1) (x) Z[t]/(t^2-t+1), a = a00 + a10 s + a01 t + a11 s t.
      Because t^2 - t + 1 = (t - s)(t - (1 - s)), that ring maps into
      Z[s] x Z[s] by t -> s and t -> 1 - s.  These images are the true 2-D DFT
      values Z[k1, k2] and Z[k1, -k2]; the remaining two conjugates are
      redundant for real data, which is the Hermitian symmetry being used:
          U = (a00 - a11)       + (a10 + a01 + a11) s        (t -> s)
          V = (a00 + a01 + a11) + (a10 - a01) s              (t -> 1 - s)
      Each image is multiplied by the 3-multiplication rule of Eq. (DFT6M),
      i.e. points U0, U1, U0+U1, V0, V1, V0+V1: 6 multiplications.
    * Inverse of the ring map (exact over the integers because the result is
      the integer nested product):
          o01 = (2 (Uo1 - Vo1) - (Vo0 - Uo0)) / 3
          o11 = (2 (Vo0 - Uo0) - (Uo1 - Vo1)) / 3
          o00 = Uo0 + o11,   o10 = Vo1 + o01
      and the tile output is sum_ij (c_i (x) c_j) o_ij with c_0 = -A[a1 row],
      c_1 = A[sum row] (the iF_6 rows recovered from the folded A).
    Count: 64 + 4*6 = 88 for the 6x6 tile; 108 + 24 = 132 for the 7x7 tile; 160 + 24 = 184
    for SFC-6(6x6,5x5) (the same construction: only the number of correction rows differs).  Order: the
    kept points in nested order, then the blocks (k1,k2) = (1,1), (1,2), (2,1),
    (2,2), six points each in the order U0, U1, U0+U1, V0, V1, V0+V1.

    Returns (B2 [P,(m+r-1)^2], G2 [P,r^2], A2 numerators [P,m^2], 36).
    """
    bt, g, a, den = sfc6_1d(m, r)
    nrows = bt.shape[0]
    complex_rows = {r for grp in COMPLEX_GROUPS for r in grp}
    b_rows, g_rows, a_rows = [], [], []
    for p1 in range(nrows):
        for p2 in range(nrows):
            if p1 in complex_rows and p2 in complex_rows:
                continue
            b_rows.append(np.kron(bt[p1], bt[p2]))
            g_rows.append(np.kron(g[p1], g[p2]))
            a_rows.append(np.kron(a[p1], a[p2]))

    def six_points(m, grp1, grp2):
        """U0, U1, U0+U1, V0, V1, V0+V1 for a 1-D matrix m (B^T or G)."""
        c = [[np.kron(m[grp1[i]], m[grp2[j]]) for j in range(2)] for i in range(2)]
        u0 = c[0][0] - c[1][1]
        u1 = c[1][0] + c[0][1] + c[1][1]
        v0 = c[0][0] + c[0][1] + c[1][1]
        v1 = c[1][0] - c[0][1]
        return [u0, u1, u0 + u1, v0, v1, v0 + v1]

    # 3 * o_ij as integer combinations of the six products (mU0,mU1,mU2,mV0,mV1,mV2)
    uo0 = np.array([1, -1, 0, 0, 0, 0])
    uo1 = np.array([-1, 0, 1, 0, 0, 0])
    vo0 = np.array([0, 0, 0, 1, -1, 0])
    vo1 = np.array([0, 0, 0, -1, 0, 1])
    o01_x3 = 2 * (uo1 - vo1) - (vo0 - uo0)
    o11_x3 = 2 * (vo0 - uo0) - (uo1 - vo1)
    o00_x3 = 3 * uo0 + o11_x3
    o10_x3 = 3 * vo1 + o01_x3
    o_x3 = {(0, 0): o00_x3, (1, 0): o10_x3, (0, 1): o01_x3, (1, 1): o11_x3}

    for grp1 in COMPLEX_GROUPS:
        for grp2 in COMPLEX_GROUPS:
            b_rows += six_points(bt, grp1, grp2)
            g_rows += six_points(g, grp1, grp2)
            c1 = (-a[grp1[1]], a[grp1[2]])
            c2 = (-a[grp2[1]], a[grp2[2]])
            block = np.zeros((6, m * m), dtype=np.int64)
            for (i, j), comb in o_x3.items():
                block += np.outer(comb, np.kron(c1[i], c2[j]))
            assert np.all(block % 3 == 0), "thirds must cancel"
            a_rows += list(block // 3)
    return (
        np.array(b_rows, dtype=np.int64),
        np.array(g_rows, dtype=np.int64),
        np.array(a_rows, dtype=np.int64),
        den * den,
    )


def sfc4_1d():
    """The three 1-D matrices of SFC-4(4,3) as printed in Appendix A: (B^T 7x6, G 7x3, A numerators 7x4, 4)."""
    return BT4_1D.copy(), G4_1D.copy(), A4_1D.copy(), A4_1D_DEN


def nested4_2d(m: int = 4):
    """Nested 2-D form of SFC-4(4x4,3x3): 49 points, p = 7*p1 + p2 (Appendix A)."""
    bt, g, a, den = sfc4_1d()
    return np.kron(bt, bt), np.kron(g, g), np.kron(a, a), den * den


def hermitian4_2d(m: int = 4):
    """46-point 2-D form of SFC-4(4x4,3x3) ("when Hermitian symmetry is fully considered").

    The paper states the count only.  Same construction as for SFC-6, with s = j: every
    nested point in which at most one axis is the complex point is kept (40 of 49, nested
    order).  The complex x complex block is the product of two elements of
    Z[s]/(s^2+1) (x) Z[t]/(t^2+1), a = a00 + a10 s + a01 t + a11 s t; since
    t^2 + 1 = (t - s)(t + s) that ring maps into Z[s] x Z[s] by t -> s and t -> -s, the 2-D
    DFT values Z[1,1] and Z[1,-1]:
        U = (a00 - a11) + (a10 + a01) s        (t -> s)
        V = (a00 + a11) + (a10 - a01) s        (t -> -s)
    each multiplied with the 3-multiplication rule of Eq. (DFT4M) (o0 = m0 - m1,
    o1 = m2 - m0 - m1): points U0, U1, U0+U1, V0, V1, V0+V1, 6 multiplications instead of 9.
    Inverse of the ring map: o00 = (Uo0 + Vo0)/2, o11 = (Vo0 - Uo0)/2, o10 = (Uo1 + Vo1)/2,
    o01 = (Uo1 - Vo1)/2; the tile output is sum_ij (c_i (x) c_j) o_ij with c_1 = A[sum row]
    and c_0 = A[a0 row] + c_1 (the inverse-DFT rows recovered from the folded A); the halves
    cancel exactly.  Count: 40 + 6 = 46.
    Returns (B2 [46,36], G2 [46,9], A2 numerators [46,16], 16).
    """
    bt, g, a, den = sfc4_1d()
    r0, r1, rs = SFC4_COMPLEX_GROUP
    complex_rows = {r0, r1, rs}
    nrows = bt.shape[0]
    b_rows, g_rows, a_rows = [], [], []
    for p1 in range(nrows):
        for p2 in range(nrows):
            if p1 in complex_rows and p2 in complex_rows:
                continue
            b_rows.append(np.kron(bt[p1], bt[p2]))
            g_rows.append(np.kron(g[p1], g[p2]))
            a_rows.append(np.kron(a[p1], a[p2]))

    def six_points(mat):
        c = [[np.kron(mat[(r0, r1)[i]], mat[(r0, r1)[j]]) for j in range(2)] for i in range(2)]
        u0 = c[0][0] - c[1][1]
        u1 = c[1][0] + c[0][1]
        v0 = c[0][0] + c[1][1]
        v1 = c[1][0] - c[0][1]
        return [u0, u1, u0 + u1, v0, v1, v0 + v1]

    # 2 * o_ij as integer combinations of the six products (mU0,mU1,mU2,mV0,mV1,mV2)
    uo0 = np.array([1, -1, 0, 0, 0, 0])
    uo1 = np.array([-1, -1, 1, 0, 0, 0])
    vo0 = np.array([0, 0, 0, 1, -1, 0])
    vo1 = np.array([0, 0, 0, -1, -1, 1])
    o_x2 = {(0, 0): uo0 + vo0, (1, 1): vo0 - uo0, (1, 0): uo1 + vo1, (0, 1): uo1 - vo1}
    b_rows += six_points(bt)
    g_rows += six_points(g)
    c = (a[r0] + a[rs], a[rs])  # inverse-DFT coefficient rows of the real and imaginary part
    block = np.zeros((6, m * m), dtype=np.int64)
    for (i, j), comb in o_x2.items():
        block += np.outer(comb, np.kron(c[i], c[j]))
    assert np.all(block % 2 == 0), "halves must cancel"
    a_rows += list(block // 2)
    return (
        np.array(b_rows, dtype=np.int64),
        np.array(g_rows, dtype=np.int64),
        np.array(a_rows, dtype=np.int64),
        den * den,
    )


_ALGORITHMS = {  # name -> (2-D construction, outputs per tile edge M, filter size R)
    "6x6_p88": (hermitian_2d, 6, 3),
    "6x6_p100": (nested_2d, 6, 3),
    "7x7_p132": (hermitian_2d, 7, 3),
    "7x7_p144": (nested_2d, 7, 3),
    "4x4_p46": (hermitian4_2d, 4, 3),
    "4x4_p49": (nested4_2d, 4, 3),
    "6x6_5x5_p184": (hermitian_2d, 6, 5),
    "6x6_5x5_p196": (nested_2d, 6, 5),
    "4x4_7x7_p184": (hermitian_2d, 4, 7),
    "4x4_7x7_p196": (nested_2d, 4, 7),
}


def algorithm(name: str):
    """(B2, G2, A2 numerators, denominator) for "6x6_p88", "6x6_p100", "7x7_p132", "7x7_p144",
    "4x4_p46", "4x4_p49" (3x3 filters), "6x6_5x5_p184", "6x6_5x5_p196" (5x5 filters) and
    "4x4_7x7_p184", "4x4_7x7_p196" (7x7 filters)."""
    build, m, r = _ALGORITHMS[name]
    return build(m) if r == 3 else build(m, r)


def tile_out(name: str) -> int:
    """Outputs per tile edge (M of SFC-N(MxM,RxR))."""
    return _ALGORITHMS[name][1]


def kernel_size(name: str) -> int:
    """Filter edge (R of SFC-N(MxM,RxR))."""
    return _ALGORITHMS[name][2]


def multiplications_per_tile(name: str) -> int:
    """Real multiplications per output tile and (Cin, Cout) pair: one per point."""
    return algorithm(name)[0].shape[0]


def direct_multiplications_per_tile(m: int = TILE_OUT, r: int = KERNEL) -> int:
    return m * m * r * r


# ---------------------------------------------------------------------------
# The definition: direct RxR cross-correlation (R = 3 or 5), stride 1, zero padding (R-1)/2.
# ---------------------------------------------------------------------------


def _exact_f64(*max_abs_and_len):
    """Assert that a float64 contraction of integers is exact (below 2**53)."""
    bound = 1.0
    for v in max_abs_and_len:
        bound *= float(v)
    assert bound < 2.0**53, "integer contraction would not be exact in float64"


def direct_conv(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """acc[n,k,h,w] = sum_{c,r,s} x[n,c,h+r-pad,w+s-pad] * w[k,c,r,s], zeros outside, for an
    R x R filter (R odd) with pad = (R-1)/2.

    int8 inputs, exact int64 result.  (No kernel flip: the paper's matrices
    compute y_o = sum_r x_{o+r} f_r.)
    """
    x = np.asarray(x)
    w = np.asarray(w)
    n, c, h, wd = x.shape
    k, rr = w.shape[0], w.shape[2]
    assert w.shape == (k, c, rr, rr) and rr % 2 == 1
    pad = (rr - 1) // 2
    _exact_f64(np.abs(x).max(initial=1), np.abs(w).max(initial=1), rr * rr * c)
    xp = np.zeros((n, c, h + 2 * pad, wd + 2 * pad), dtype=np.float64)
    xp[:, :, pad : pad + h, pad : pad + wd] = x
    wf = w.astype(np.float64)
    acc = np.zeros((k, n, h, wd), dtype=np.float64)
    for r in range(rr):
        for s in range(rr):
            acc += np.tensordot(wf[:, :, r, s], xp[:, :, r : r + h, s : s + wd], axes=([1], [1]))
    return np.rint(acc).astype(np.int64).transpose(1, 0, 2, 3)


def dequantize(acc: np.ndarray, x_scale, w_scale) -> np.ndarray:
    """y = acc * (s_x * s_w[k]) in float64; ``w_scale`` is a scalar or has Cout entries."""
    ws = np.broadcast_to(np.asarray(w_scale, dtype=np.float64).reshape(-1), (acc.shape[1],))
    return acc.astype(np.float64) * (float(x_scale) * ws)[None, :, None, None]


# ---------------------------------------------------------------------------
# Tiling (paper silent on padding; reading: zero pad (R-1)/2, ragged tiles read zeros
# beyond the image and their surplus outputs are dropped -- exact by linearity)
# ---------------------------------------------------------------------------


def tile_grid(h: int, w: int, m: int = TILE_OUT):
    return -(-h // m), -(-w // m)


def gather_tiles(x: np.ndarray, m: int = TILE_OUT, r: int = KERNEL) -> np.ndarray:
    """[N,C,H,W] -> tiles [T, C, m+r-1, m+r-1], T = N*th*tw, t = (n*th + ti)*tw + tj.

    Tile (ti,tj) covers input rows m*ti-pad .. m*ti+m-1+pad and the same columns of tj,
    pad = (r-1)/2 (r = 3: rows m*ti-1 .. m*ti+m).
    """
    n, c, h, w = x.shape
    th, tw = tile_grid(h, w, m)
    pad, ni = (r - 1) // 2, m + r - 1
    xp = np.zeros((n, c, m * th + 2 * pad, m * tw + 2 * pad), dtype=np.int64)
    xp[:, :, pad : pad + h, pad : pad + w] = x
    tiles = np.empty((n, th, tw, c, ni, ni), dtype=np.int64)
    for ti in range(th):
        for tj in range(tw):
            tiles[:, ti, tj] = xp[:, :, m * ti : m * ti + ni, m * tj : m * tj + ni]
    return tiles.reshape(n * th * tw, c, ni, ni)


def scatter_tiles(o: np.ndarray, n: int, h: int, w: int) -> np.ndarray:
    """Tile outputs [T, K, m, m] -> [N, K, H, W], dropping the ragged surplus."""
    m = o.shape[-1]
    th, tw = tile_grid(h, w, m)
    k = o.shape[1]
    o = o.reshape(n, th, tw, k, m, m)
    full = np.empty((n, k, m * th, m * tw), dtype=o.dtype)
    for ti in range(th):
        for tj in range(tw):
            full[:, :, m * ti : m * ti + m, m * tj : m * tj + m] = o[:, ti, tj]
    return np.ascontiguousarray(full[:, :, :h, :w])


def _isqrt(n: int) -> int:
    r = int(round(n**0.5))
    assert r * r == n
    return r


# ---------------------------------------------------------------------------
# The three stages of Eq. (1)
# ---------------------------------------------------------------------------


def input_transform(x: np.ndarray, b2: np.ndarray, r: int = KERNEL) -> np.ndarray:
    """V[p,t,c] = sum_ij B2[p,(i,j)] * tile[t,c,i,j]  (B^T x B, additions only); r = filter edge."""
    n_in = _isqrt(b2.shape[1])
    tiles = gather_tiles(x, n_in - (r - 1), r)
    t, c = tiles.shape[:2]
    v = b2 @ tiles.reshape(t * c, n_in * n_in).T  # int64, exact
    return v.reshape(b2.shape[0], t, c)


def filter_transform(w: np.ndarray, g2: np.ndarray) -> np.ndarray:
    """U[p,k,c] = sum_rs G2[p,(r,s)] * w[k,c,r,s]  (G f G^T, additions only)."""
    k, c = w.shape[:2]
    u = g2 @ np.asarray(w, dtype=np.int64).reshape(k * c, g2.shape[1]).T
    return u.reshape(g2.shape[0], k, c)


def pointwise_product(v: np.ndarray, u: np.ndarray) -> np.ndarray:
    """M[p,t,k] = sum_c V[p,t,c] * U[p,k,c]: the element-wise product of Eq. (1)
    summed over input channels, i.e. one [T x Cin] . [Cin x Cout] product per point."""
    _exact_f64(np.abs(v).max(initial=1), np.abs(u).max(initial=1), v.shape[2])
    m = np.matmul(v.astype(np.float64), u.astype(np.float64).transpose(0, 2, 1))
    return np.rint(m).astype(np.int64)


def output_transform_exact(m: np.ndarray, a2: np.ndarray, den: int, n: int, h: int, w: int):
    """acc = (A2^T M) / den, which must divide exactly; returns int64 [N,K,H,W]."""
    p, t, k = m.shape
    mo = _isqrt(a2.shape[1])
    o = (a2.T @ m.reshape(p, t * k)).reshape(mo * mo, t, k)
    assert np.all(o % den == 0), "exact SFC output must be divisible by the denominator"
    o = (o // den).transpose(1, 2, 0).reshape(t, k, mo, mo)
    return scatter_tiles(o, n, h, w)


def conv_exact(x, w, alg="6x6_p88", return_taps=False):
    """Eq. (1) over the integers, no transform-domain rounding: equals ``direct_conv``."""
    b2, g2, a2, den = algorithm(alg)
    n, _, h, wd = x.shape
    v = input_transform(x, b2, kernel_size(alg))
    u = filter_transform(w, g2)
    m = pointwise_product(v, u)
    acc = output_transform_exact(m, a2, den, n, h, wd)
    if return_taps:
        return acc, {"V": v, "U": u, "M": m}
    return acc


# ---------------------------------------------------------------------------
# Sec. 5: frequency-wise (activations) and channel+frequency-wise (filters)
# quantization in the transform domain.
# ---------------------------------------------------------------------------

QMAX = 127  # symmetric int8


def reciprocal_f32(scale) -> np.ndarray:
    """1/scale as one correctly rounded float32 division (what the quantizer multiplies by)."""
    return (np.float32(1.0) / np.asarray(scale, dtype=np.float32)).astype(np.float32)


def quantize(values: np.ndarray, inv_scale: np.ndarray, qmax: int = QMAX) -> np.ndarray:
    """round-half-even(values * inv_scale), clamped to [-qmax, qmax].

    The product of a transform-domain integer (below 2**14) with a float32
    reciprocal scale has at most 38 significant bits, so the float64 product
    is exact and ``rint`` rounds the true product once, ties to even.
    """
    prod = np.asarray(values, dtype=np.float64) * np.asarray(inv_scale, dtype=np.float64)
    return np.clip(np.rint(prod), -qmax, qmax).astype(np.int64)


def calibrate_act_scales(x_calib: np.ndarray, alg="6x6_p88", qmax: int = QMAX) -> np.ndarray:
    """s_Tx[p] = max |V[p,.,.]| / qmax over a calibration tensor (float32; 0 -> 1).

    The paper learns its scales with AdaQuant on ImageNet images; abs-max
    calibration stands in for that.  One scale per multiplication point.
    """
    v = input_transform(x_calib, algorithm(alg)[0], kernel_size(alg))
    mx = np.abs(v).max(axis=(1, 2)).astype(np.float32)
    s = mx / np.float32(qmax)
    return np.where(mx == 0, np.float32(1.0), s).astype(np.float32)


def calibrate_filter_scales(w: np.ndarray, alg="6x6_p88", qmax: int = QMAX) -> np.ndarray:
    """s_Tf[p,k] = max_c |U[p,k,c]| / qmax (float32; 0 -> 1): channel + frequency wise."""
    u = filter_transform(w, algorithm(alg)[1])
    mx = np.abs(u).max(axis=2).astype(np.float32)
    s = mx / np.float32(qmax)
    return np.where(mx == 0, np.float32(1.0), s).astype(np.float32)


def group_scales(sx_pt: np.ndarray, sw_pt: np.ndarray, act: str = "point", filt: str = "channel_point"):
    """Scale granularities of the ablation study (Sec. 6, "Ablation Study on Quantization
    Granularity"), from the finest abs-max scales ``sx_pt`` [P] and ``sw_pt`` [P, Cout].

    ``act``: "tensor" (one activation scale) or "point" (one per frequency, Sec. 5's [T x T]).
    ``filt``: "channel" (one per output channel), "point" (one per frequency) or
    "channel_point" (Sec. 5's [OC x T x T]).  A group's abs-max scale is the largest scale
    in the group, since all of them are maxima divided by the same qmax.  Returns float32
    arrays of the full shapes [P] and [P, Cout], ready for ``conv_requant``.
    """
    sx = np.asarray(sx_pt, dtype=np.float32)
    sw = np.asarray(sw_pt, dtype=np.float32)
    if act == "tensor":
        sx = np.full_like(sx, sx.max())
    elif act != "point":
        raise ValueError(act)
    if filt == "channel":
        sw = np.broadcast_to(sw.max(axis=0, keepdims=True), sw.shape).copy()
    elif filt == "point":
        sw = np.broadcast_to(sw.max(axis=1, keepdims=True), sw.shape).copy()
    elif filt != "channel_point":
        raise ValueError(filt)
    return sx.copy(), sw


def output_transform_dequant(m, a2, den, sx_pt, sw_pt, x_scale, w_scale, n, h, w):
    """y[o] = (s_x s_w[k] / den) * sum_p A2[p,o] * (M[p] * s_Tx[p] * s_Tf[p,k]), float64."""
    p, t, k = m.shape
    scale = np.asarray(sx_pt, dtype=np.float64)[:, None] * np.asarray(sw_pt, dtype=np.float64)
    md = m.astype(np.float64) * scale[:, None, :]
    mo = _isqrt(a2.shape[1])
    o = (a2.T.astype(np.float64) @ md.reshape(p, t * k)).reshape(mo * mo, t, k)
    o = o.transpose(1, 2, 0).reshape(t, k, mo, mo)
    y = scatter_tiles(o, n, h, w)
    ws = np.broadcast_to(np.asarray(w_scale, dtype=np.float64).reshape(-1), (k,))
    return y * (float(x_scale) * ws / den)[None, :, None, None]


def conv_requant(x, w, sx_pt, sw_pt, x_scale, w_scale, alg="6x6_p88", qmax=QMAX, return_taps=False):
    """The quantized fast convolution of Sec. 5 (unnumbered equation):

        y = sum_Cin ( s_Tx round(B^T x B / s_Tx) . s_Tf round(G f G^T / s_Tf) )

    followed by the output transform and the spatial-domain scales.
    ``sx_pt`` [P] and ``sw_pt`` [P, Cout] are float32 scales.
    """
    b2, g2, a2, den = algorithm(alg)
    n, _, h, wd = x.shape
    v = input_transform(x, b2, kernel_size(alg))
    u = filter_transform(w, g2)
    vq = quantize(v, reciprocal_f32(sx_pt)[:, None, None], qmax)
    uq = quantize(u, reciprocal_f32(sw_pt)[:, :, None], qmax)
    m = pointwise_product(vq, uq)
    y = output_transform_dequant(m, a2, den, sx_pt, sw_pt, x_scale, w_scale, n, h, wd)
    if return_taps:
        return y, {"V": vq, "U": uq, "M": m}
    return y


def requantize_activation(y: np.ndarray, y_scale: float) -> np.ndarray:
    """Next layer's int8 input: clamp(round-half-even(max(y, 0) / s_act), 0, 127)."""
    inv = float(reciprocal_f32(y_scale))
    return np.clip(np.rint(np.maximum(y, 0.0) * inv), 0, QMAX).astype(np.int8)
