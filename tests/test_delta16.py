"""Index compression switched off inside the same format and kernel (delta_bits = 16: every index is the 16-bit
column itself), the first step of the ablation of the paper's Section 8.3.  Host side: round trip, the Python reading of
the image, byte accounting.  No GPU."""
import numpy as np
import pytest

import paper_2507_12205_amd as E
from paper_2507_12205_amd import binding as B
from oracle import oracle as orc
from workloads import generators as gen

import pyformat


def roundtrip_ok(A, W):
    rr, cc, vv = orc.pattern_triples(W)
    r, c, v = A.ecspmv_decode()
    o = np.lexsort((c, r))
    return np.array_equal(r[o], rr) and np.array_equal(c[o], cc) and np.array_equal(v[o], vv)


@pytest.mark.parametrize("cid,div", [(0, 1), (1, 8), (2, 8), (3, 8), (4, 8)])
def test_roundtrip_bit_exact_on_the_configs(cid, div):
    cfg = gen.scaled(gen.config(cid), div) if div > 1 else gen.config(cid)
    for sid in range(len(cfg.shapes)):
        W = gen.make_matrix(cfg, sid)
        A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=16))
        assert A.ecspmv_stats().delta_bits == 16
        assert roundtrip_ok(A, W)


def test_python_reading_of_the_image_agrees_and_indices_are_the_columns():
    cfg = gen.scaled(gen.config(1), 16)
    W = gen.make_matrix(cfg, 0)
    A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=16, flags=B.FLAG_KEEP_SMALL_SETS))
    img = A.ecspmv_export_image()
    rr, cc, vv = orc.pattern_triples(W)
    r, c, v = pyformat.triples(img)
    assert np.array_equal(r, rr) and np.array_equal(c, cc) and np.array_equal(v, vv)
    kinds = set()
    for u in pyformat.walk(img):
        kinds.add(u["kind"])
        assert np.array_equal(u["deltas"], u["cols"])                    # what is stored IS the column
        assert np.all(np.diff(u["cols"]) >= 0)
    assert kinds == {"block", "lane"}


def test_no_fillers_and_wide_gaps():
    """A gap of 60000 columns costs nothing: there is no delta range to exceed, so no zero fillers are stored, and a
    block may span it."""
    W = np.zeros((2, 65535), dtype=np.float16)
    cols = list(range(0, 64, 2)) + list(range(60000, 60064, 2))
    W[:, cols] = 1.5
    W[0, 65534] = -2.0
    A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=16, num_panels=1))
    st = A.ecspmv_stats()
    assert st.gap_pad_elements == 0
    assert st.nnz_by_g[1] == 128 and st.nnz_by_g[0] == 1
    assert roundtrip_ok(A, W)
    B8 = E.ecspmv_build_dense(W, E.make_opts(delta_bits=8, num_panels=1))
    assert B8.ecspmv_stats().nnz_by_g[1] == 0 and B8.ecspmv_stats().gap_pad_elements > 200     # 8-bit deltas: fillers


def test_byte_accounting_against_csr16():
    """Residual-only image with 16-bit columns: 4 bytes per stored entry plus padding and tables, which is CSR with
    16-bit indices in this library's layout."""
    cfg = gen.scaled(gen.config(4), 8)
    W = gen.make_matrix(cfg, 0)
    A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=16, max_granularity=1))
    st = A.ecspmv_stats()
    elems = st.nnz + st.pad_elements
    assert st.delta_bytes == 2 * elems and st.value_bytes == 2 * elems
    assert st.pad_elements < 16 * st.m                                   # tail alignment only
    assert 4 * st.nnz <= st.delta_bytes + st.value_bytes < 4 * (st.nnz + 16 * st.m)
    assert st.csr16_bytes == 4 * st.nnz + 4 * (st.m + 1)


def test_options_that_do_not_combine():
    W = np.ones((4, 64), dtype=np.float32)
    with pytest.raises(E.EcspmvError) as e:
        E.ecspmv_build_dense_f32(W, E.make_opts(delta_bits=16))
    assert e.value.status == B.ERR_UNSUPPORTED
    with pytest.raises(E.EcspmvError):
        E.ecspmv_build_dense(W.astype(np.float16), E.make_opts(delta_bits=12))
