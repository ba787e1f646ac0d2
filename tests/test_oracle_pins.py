"""Pins for the CPU oracle: each check fixes it to something other than itself.

Definition under test: y[i] = sum_j W[i,j] x[j], S[i] = sum_j |W[i,j] x[j]| in FP64 from
FP16 inputs (paper Sections 1, 2.1, 2.2).  A dropped term, a wrong sign, a transposed
operand, a wrong FP16 decode or a row/column mix-up fails at least one of these.
"""
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import oracle as orc
from workloads import generators as gen


def _exact_fraction(h: np.float16) -> Fraction:
    """Exact rational value of an FP16 number, decoded from its bits by the IEEE 754 rule."""
    b = int(np.array(h, dtype=np.float16).view(np.uint16))
    s, e, f = b >> 15, (b >> 10) & 31, b & 1023
    assert e != 31
    v = Fraction(f, 1 << 24) if e == 0 else Fraction(1024 + f, 1024) * (Fraction(2) ** (e - 15))
    return -v if s else v


def test_half_conversion_all_patterns():
    """Every one of the 65536 FP16 patterns converts like numpy's float16 -> float64."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([orc.half_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


@pytest.mark.parametrize("shape", [(1, 1), (1, 7), (7, 1), (5, 8), (8, 8), (3, 6)])
def test_brute_force_exact_rationals(shape):
    """Against exact rational arithmetic: the FP64 result is the exact value within an ulp or so."""
    m, n = shape
    for seed in range(4):
        W, x = gen.small_random(m, n, 0.6, seed, scale=1.0)
        y, S = orc.spmv_oracle(W, x)
        for i in range(m):
            exact = sum((_exact_fraction(W[i, j]) * _exact_fraction(x[j]) for j in range(n)), Fraction(0))
            exact_abs = sum((abs(_exact_fraction(W[i, j]) * _exact_fraction(x[j])) for j in range(n)), Fraction(0))
            tol = float(exact_abs) * n * 2.0 ** -52 + 5e-324
            assert abs(Fraction(y[i]) - exact) <= Fraction(tol)
            assert abs(Fraction(S[i]) - exact_abs) <= Fraction(tol)


def test_c_matches_python_loops_bitwise():
    """The C loop and the same definition written as Python loops agree bit for bit."""
    for seed, (m, n) in enumerate([(9, 33), (16, 16), (4, 100)]):
        W, x = gen.small_random(m, n, 0.5, 100 + seed)
        y, S = orc.spmv_oracle(W, x)
        yp, Sp = orc.spmv_oracle_py(W, x)
        assert np.array_equal(y, yp) and np.array_equal(S, Sp)


def test_all_zero_matrix():
    W = np.zeros((13, 29), dtype=np.float16)
    x = gen.make_vector(29, seed=3)
    y, S = orc.spmv_oracle(W, x)
    assert np.all(y == 0.0) and np.all(S == 0.0)


def test_unit_vector_returns_column():
    W, _ = gen.small_random(40, 37, 0.5, 7)
    for j in (0, 5, 36):
        x = np.zeros(37, dtype=np.float16)
        x[j] = 1.0
        y, S = orc.spmv_oracle(W, x)
        assert np.array_equal(y, W[:, j].astype(np.float64))
        assert np.array_equal(S, np.abs(W[:, j].astype(np.float64)))


def test_row_and_column_permutation():
    W, x = gen.small_random(31, 45, 0.4, 11)
    y, S = orc.spmv_oracle(W, x)
    rng = np.random.default_rng(5)
    pr = rng.permutation(31)
    yp, Sp = orc.spmv_oracle(W[pr], x)
    assert np.array_equal(yp, y[pr]) and np.array_equal(Sp, S[pr])          # rows: exact
    pc = rng.permutation(45)
    yq, Sq = orc.spmv_oracle(W[:, pc], x[pc])
    assert np.all(np.abs(yq - y) <= 45 * 2.0 ** -52 * S + 1e-300)            # columns: re-association only
    assert np.all(np.abs(Sq - S) <= 45 * 2.0 ** -52 * S + 1e-300)


def test_power_of_two_scaling_is_exact():
    W, x = gen.small_random(20, 50, 0.5, 13)
    y, S = orc.spmv_oracle(W, x)
    x4 = (x.astype(np.float32) * 4.0).astype(np.float16)
    assert np.array_equal(x4.astype(np.float64), x.astype(np.float64) * 4.0)
    y4, S4 = orc.spmv_oracle(W, x4)
    assert np.array_equal(y4, 4.0 * y) and np.array_equal(S4, 4.0 * S)


def test_closed_forms():
    n = 64
    x = gen.make_vector(n, seed=17)
    y, _ = orc.spmv_oracle(np.eye(n, dtype=np.float16), x)
    assert np.array_equal(y, x.astype(np.float64))                          # identity
    d = gen.make_vector(n, seed=18)
    y, S = orc.spmv_oracle(np.diag(d).astype(np.float16), x)
    assert np.array_equal(y, d.astype(np.float64) * x.astype(np.float64))   # diagonal
    ones = np.ones((3, 2000), dtype=np.float16)
    y, S = orc.spmv_oracle(ones, np.ones(2000, dtype=np.float16))
    assert np.all(y == 2000.0) and np.all(S == 2000.0)                      # all-ones row
    # sign pattern: S counts magnitudes, y cancels
    W = np.array([[1.0, -1.0, 2.0, -2.0]], dtype=np.float16)
    y, S = orc.spmv_oracle(W, np.ones(4, dtype=np.float16))
    assert y[0] == 0.0 and S[0] == 6.0
    # non-square, distinguishes W x from W^T x
    W = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float16)
    y, _ = orc.spmv_oracle(W, np.array([1, 10, 100], dtype=np.float16))
    assert np.array_equal(y, [321.0, 654.0])


def test_subnormal_inputs_are_not_flushed():
    W = np.full((2, 8), 2.0 ** -24, dtype=np.float16)                       # smallest FP16 subnormal
    x = np.ones(8, dtype=np.float16)
    y, S = orc.spmv_oracle(W, x)
    assert np.all(y == 8 * 2.0 ** -24) and np.all(S == y)


def test_against_numpy_and_scipy_on_generated_workloads():
    """Independent library code (BLAS gemv, scipy CSR), different summation order."""
    for cid in (0, 4):
        cfg = gen.scaled(gen.config(cid), 8 if cid else 1)
        W, x = gen.make_case(cfg, 0, seed=0)
        n = W.shape[1]
        y, S = orc.spmv_oracle(W, x)
        W64, x64 = W.astype(np.float64), x.astype(np.float64)
        tol = n * 2.0 ** -52 * S + 1e-300
        assert np.all(np.abs(W64 @ x64 - y) <= tol)
        assert np.all(np.abs(sp.csr_matrix(W64) @ x64 - y) <= tol)
        assert np.all(np.abs(np.abs(W64) @ np.abs(x64) - S) <= tol)


def test_leading_rows_do_not_leak():
    """Row i depends on row i of W only."""
    W, x = gen.small_random(12, 30, 0.5, 23)
    y, _ = orc.spmv_oracle(W, x)
    W2 = W.copy()
    W2[5] = 0
    y2, _ = orc.spmv_oracle(W2, x)
    assert y2[5] == 0.0
    assert np.array_equal(np.delete(y2, 5), np.delete(y, 5))


def test_pattern_triples_definition():
    W = np.array([[0.0, 1.5, -0.0], [2.0 ** -24, 0.0, -3.0]], dtype=np.float16)
    r, c, b = orc.pattern_triples(W)
    assert r.tolist() == [0, 1, 1] and c.tolist() == [1, 0, 2]
    assert b.tolist() == [0x3E00, 0x0001, 0xC200]


def test_pattern_triples_f32_definition():
    """FP32 twin, on bit patterns written out by hand: +0 and -0 are not stored; the smallest subnormal, 1.5, a
    negative value and a NaN pattern are, with exactly the bits they came with."""
    bits = np.array([[0x00000000, 0x3FC00000, 0x80000000, 0x00000001],
                     [0x80000001, 0x00000000, 0xC0400000, 0x7FC00001]], dtype=np.uint32)
    r, c, b = orc.pattern_triples_f32(bits.view(np.float32))
    assert r.tolist() == [0, 0, 1, 1, 1] and c.tolist() == [1, 3, 0, 2, 3]
    assert b.dtype == np.uint32 and b.tolist() == [0x3FC00000, 0x00000001, 0x80000001, 0xC0400000, 0x7FC00001]
    # and the values behind three of them, to tie the bit patterns to numbers
    assert np.array([0x3FC00000, 0xC0400000, 0x00000001], dtype=np.uint32).view(np.float32).tolist() == [1.5, -3.0, 2.0 ** -149]


def test_band_helper():
    ok, ratio = orc.within_band(np.array([1.0, 2.0]), np.array([1.0, 2.001]), np.array([1.0, 1.0]))
    assert ok and 0.49 < ratio < 0.51
    ok, _ = orc.within_band(np.array([1.0]), np.array([1.01]), np.array([1.0]))
    assert not ok
