"""FP32 values (the paper's other precision): the oracle's FP32 entry point against what the mathematics fixes, and
the encoder's round trip; no GPU."""
from fractions import Fraction

import numpy as np
import pytest

import paper_2507_12205_amd as E
from paper_2507_12205_amd import binding as B
from oracle import oracle as orc
from workloads import generators as gen


def make_f32(W16, seed):
    """An FP32 matrix with the pattern of W16 whose values need all 24 significand bits."""
    rng = np.random.default_rng(seed)
    W = W16.astype(np.float32) * (1.0 + rng.uniform(-1e-3, 1e-3, W16.shape)).astype(np.float32)
    assert np.array_equal(W != 0, W16 != 0)
    return W


# ---- oracle pins ------------------------------------------------------------------------------------------------

def test_oracle_f32_equals_exact_rational_arithmetic():
    rng = np.random.default_rng(0)
    for m, n in ((1, 1), (3, 5), (8, 8), (1, 40), (7, 1)):
        W = (rng.standard_normal((m, n)) * rng.choice([0, 1], (m, n))).astype(np.float32)
        x = rng.standard_normal(n).astype(np.float32)
        y, S = orc.spmv_oracle_f32(W, x)
        for i in range(m):
            exact = sum(Fraction(float(W[i, j])) * Fraction(float(x[j])) for j in range(n))
            mag = sum(abs(Fraction(float(W[i, j])) * Fraction(float(x[j]))) for j in range(n))
            assert abs(Fraction(float(y[i])) - exact) <= Fraction(float(np.spacing(max(float(mag), 1e-300)))) * n
            assert abs(Fraction(float(S[i])) - mag) <= Fraction(float(np.spacing(max(float(mag), 1e-300)))) * n


def test_oracle_f32_closed_forms_and_invariants():
    rng = np.random.default_rng(1)
    n = 300
    W = (rng.standard_normal((50, n)) * (rng.random((50, n)) < 0.3)).astype(np.float32)
    x = rng.standard_normal(n).astype(np.float32)
    y, S = orc.spmv_oracle_f32(W, x)
    assert np.array_equal(orc.spmv_oracle_f32(np.zeros_like(W), x)[0], np.zeros(50))
    for j in (0, 7, n - 1):                                           # x = e_j returns column j exactly
        e = np.zeros(n, dtype=np.float32)
        e[j] = 1.0
        assert np.array_equal(orc.spmv_oracle_f32(W, e)[0], W[:, j].astype(np.float64))
    perm = rng.permutation(50)
    assert np.array_equal(orc.spmv_oracle_f32(W[perm], x)[0], y[perm])
    assert np.array_equal(orc.spmv_oracle_f32(W, (x * 4).astype(np.float32))[0], y * 4)
    ref = W.astype(np.float64) @ x.astype(np.float64)                 # a library routine, another summation order
    assert np.all(np.abs(y - ref) <= n * 2.0 ** -52 * S)
    assert np.all(S >= np.abs(y))
    A = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)            # tells W x from W^T x
    assert orc.spmv_oracle_f32(A, np.array([1, 10, 100], dtype=np.float32))[0].tolist() == [321.0, 654.0]
    t = np.float32(1 + 2.0 ** -23)                                    # an FP32-only value: the product needs FP64
    assert orc.spmv_oracle_f32(np.array([[t]], dtype=np.float32), np.array([t], dtype=np.float32))[0][0] == float(t) * float(t)


# ---- encoder round trip ----------------------------------------------------------------------------------------

def roundtrip_ok(A, W):
    r, c, v = A.ecspmv_decode_f32()
    rr, cc, vv = orc.pattern_triples_f32(W)
    o = np.lexsort((c, r))
    return np.array_equal(r[o], rr) and np.array_equal(c[o], cc) and np.array_equal(v[o], vv)


@pytest.mark.parametrize("cid,div,bits", [(0, 1, 8), (1, 4, 8), (3, 4, 8), (4, 8, 8), (1, 4, 4), (3, 4, 4)])
def test_roundtrip_bit_exact(cid, div, bits):
    cfg = gen.scaled(gen.config(cid), div) if div > 1 else gen.config(cid)
    W = make_f32(gen.make_matrix(cfg, 0), seed=cid)
    A = E.ecspmv_build_dense_f32(W, E.make_opts(delta_bits=bits))
    assert roundtrip_ok(A, W)
    st = A.ecspmv_stats()
    nnz = int(np.count_nonzero(W))
    assert st.value_bits == 32 and st.nnz == nnz and sum(st.nnz_by_g) == nnz
    assert st.csr32_bytes == 8 * nnz + 4 * (W.shape[0] + 1) and st.csr16_bytes == 6 * nnz + 4 * (W.shape[0] + 1)
    stored = nnz + st.pad_elements
    assert st.value_bytes == 4 * stored                       # 4-byte values; one delta per block column or residual entry
    entries_with_a_delta = st.nnz_by_g[0] + st.pad_elements + sum(st.nnz_by_g[t] >> t for t in range(1, 5))
    assert st.delta_bytes * (8 // bits) == entries_with_a_delta


def test_same_blocks_as_the_fp16_matrix_of_the_same_pattern():
    W16 = gen.make_matrix(gen.scaled(gen.config(1), 8), 0)
    W32 = make_f32(W16, 5)
    a = E.ecspmv_build_dense(W16, E.make_opts(max_granularity=4)).ecspmv_block_sets()
    b = E.ecspmv_build_dense_f32(W32, E.make_opts(max_granularity=4)).ecspmv_block_sets()
    assert all(np.array_equal(p, q) for p, q in zip(a, b)) and len(a[0]) > 0


def test_edge_cases_and_refusals():
    W = np.zeros((4, 70), dtype=np.float32)
    W.view(np.uint32)[:] = 0x80000000                                 # all -0: nothing stored
    assert E.ecspmv_build_dense_f32(W).ecspmv_stats().nnz == 0
    W = np.zeros((3, 600), dtype=np.float32)
    W[0, [0, 599]] = [np.float32(1e-45), np.float32(3e38)]            # a subnormal and a huge value; a gap of 599 columns
    W[2, 300] = -2.5
    for bits in (4, 8):
        A = E.ecspmv_build_dense_f32(W, E.make_opts(delta_bits=bits))
        assert roundtrip_ok(A, W)
    big = np.ones((40, 500), dtype=np.float32)[:, :333]               # ld = 500 > n = 333
    assert roundtrip_ok(E.ecspmv_build_dense_f32(big), np.ascontiguousarray(big))
    A16 = E.ecspmv_build_dense(np.ones((2, 2), dtype=np.float16))
    A32 = E.ecspmv_build_dense_f32(np.ones((2, 2), dtype=np.float32))
    with pytest.raises(E.EcspmvError):
        A16.ecspmv_decode_f32()
    with pytest.raises(E.EcspmvError):
        A32.ecspmv_decode()
    W16 = gen.small_random(50, 400, 0.2, 3)[0]
    W32 = make_f32(W16, 9)
    rp = np.concatenate([[0], np.cumsum(np.count_nonzero(W32, axis=1))])
    rows, cols = np.nonzero(W32)
    Ac = E.ecspmv_build_csr_f32(rp, cols, W32[rows, cols], 50, 400)
    assert roundtrip_ok(Ac, W32)
