"""Host side of the library (no GPU): EC-CSR encoding, decoding, block extraction invariants, byte accounting,
the C ABI's symbols and error paths.  What "the stored entries of W" are comes from the oracle module."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2507_12205_amd as E
from paper_2507_12205_amd import binding as B
from oracle import oracle as orc
from workloads import generators as gen

import pyformat

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def roundtrip_ok(A, W):
    r, c, v = A.ecspmv_decode()
    rr, cc, vv = orc.pattern_triples(W)
    o = np.lexsort((c, r))
    return np.array_equal(r[o], rr) and np.array_equal(c[o], cc) and np.array_equal(v[o], vv)


# ---- ABI surface -------------------------------------------------------------------------------------------

def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ecspmv.h")).read()
    declared = set(re.findall(r"\b(ecspmv_[a-z0-9_]+)\s*\(", hdr))
    declared -= {"ecspmv_build_opts"}
    lib = B.lib()
    assert len(declared) >= 18
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared in include/ecspmv.h but not exported"
    assert set(B.EXPORTS) == declared


def test_error_paths_without_gpu():
    lib = B.lib()
    W, _ = gen.small_random(8, 64, 0.5, 1)
    out = ctypes.c_void_p(0)
    u = W.view(np.uint16)
    assert lib.ecspmv_build_dense(None, 8, 64, 64, None, ctypes.byref(out)) == B.ERR_INVALID
    assert lib.ecspmv_build_dense(u.ctypes.data, 0, 64, 64, None, ctypes.byref(out)) == B.ERR_INVALID
    assert lib.ecspmv_build_dense(u.ctypes.data, 8, 64, 32, None, ctypes.byref(out)) == B.ERR_INVALID      # ld < n
    assert lib.ecspmv_build_dense(u.ctypes.data, 1, 70000, 70000, None, ctypes.byref(out)) == B.ERR_UNSUPPORTED
    for bad in (dict(delta_bits=6), dict(max_granularity=3), dict(threads_per_wg=100)):
        o = E.make_opts(**bad)
        st = lib.ecspmv_build_dense(u.ctypes.data, 8, 64, 64, ctypes.byref(o), ctypes.byref(out))
        assert st in (B.ERR_UNSUPPORTED, B.ERR_INVALID) and not out.value
    A = E.ecspmv_build_dense(W)
    n = ctypes.c_int64(1)
    buf = np.zeros(4, dtype=np.int32)
    v = np.zeros(4, dtype=np.uint16)
    assert lib.ecspmv_decode(A._h, ctypes.byref(n), buf.ctypes.data, buf.ctypes.data, v.ctypes.data) == B.ERR_TOO_SMALL
    assert lib.ecspmv_run(A._h, ctypes.c_void_p(16), ctypes.c_void_p(32), None) == B.ERR_NOT_UPLOADED
    assert lib.ecspmv_run(None, None, None, None) == B.ERR_INVALID
    assert lib.ecspmv_run_multi(A._h, ctypes.c_void_p(16), ctypes.c_void_p(32), 4, None) == B.ERR_NOT_UPLOADED
    assert lib.ecspmv_run_multi(A._h, ctypes.c_void_p(16), ctypes.c_void_p(32), 3, None) == B.ERR_INVALID
    assert lib.ecspmv_run_multi(None, ctypes.c_void_p(16), ctypes.c_void_p(32), 2, None) == B.ERR_INVALID
    hs = (ctypes.c_void_p * 2)(A._h.value, A._h.value)
    ptrs = (ctypes.c_void_p * 2)(16, 32)
    assert lib.ecspmv_run_batch(hs, ptrs, ptrs, 2, None) == B.ERR_NOT_UPLOADED
    assert lib.ecspmv_run_batch(hs, ptrs, ptrs, 0, None) == B.ERR_INVALID
    assert lib.ecspmv_run_batch(None, ptrs, ptrs, 2, None) == B.ERR_INVALID
    odd = (ctypes.c_void_p * 2)(17, 32)
    assert lib.ecspmv_run_batch(hs, odd, ptrs, 2, None) == B.ERR_INVALID
    lib.ecspmv_destroy(None)                                                                                 # no-op
    assert lib.ecspmv_strerror(B.ERR_TOO_SMALL).decode() == "buffer too small"
    texts = {lib.ecspmv_strerror(c).decode() for c in (B.ERR_INVALID, B.ERR_UNSUPPORTED, B.ERR_NOMEM, B.ERR_HIP,
                                                      B.ERR_NOT_UPLOADED, B.ERR_TOO_SMALL, B.ERR_INTERNAL)}
    assert len(texts) == 7 and "unknown status" not in texts and lib.ecspmv_strerror(-99).decode() == "unknown status"


def test_csr_input_matches_dense_input_and_is_validated():
    W, _ = gen.small_random(50, 400, 0.3, 3)
    r, c, v = orc.pattern_triples(W)
    rowptr = np.zeros(51, dtype=np.int64)
    np.add.at(rowptr, r + 1, 1)
    rowptr = np.cumsum(rowptr)
    A = E.ecspmv_build_csr(rowptr, c, v, 50, 400)
    D = E.ecspmv_build_dense(W)
    assert roundtrip_ok(A, W)
    assert np.array_equal(A.ecspmv_export_image()[256:], D.ecspmv_export_image()[256:])
    bad = c.copy()
    bad[1], bad[0] = c[0], c[1]                                                 # unsorted columns
    with pytest.raises(E.EcspmvError):
        E.ecspmv_build_csr(rowptr, bad, v, 50, 400)
    bad = c.copy()
    bad[0] = 400                                                                # out of range
    with pytest.raises(E.EcspmvError):
        E.ecspmv_build_csr(rowptr, bad, v, 50, 400)


# ---- round trip ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("cid,div", [(0, 1), (1, 4), (2, 8), (3, 4), (4, 8)])
def test_roundtrip_bit_exact_on_the_configs(cid, div):
    cfg = gen.scaled(gen.config(cid), div) if div > 1 else gen.config(cid)
    for sid in range(len(cfg.shapes)):
        if cid == 3 and sid in (1, 2, 3, 5):
            continue
        W = gen.make_matrix(cfg, sid)
        A = E.ecspmv_build_dense(W)
        assert roundtrip_ok(A, W), (cid, sid)
        st = A.ecspmv_stats()
        assert st.nnz == int(np.count_nonzero(W.view(np.uint16) & 0x7FFF))
        assert sum(st.nnz_by_g) == st.nnz


@pytest.mark.parametrize("opts", [dict(max_granularity=1), dict(max_granularity=2), dict(max_granularity=16),
                                  dict(num_panels=1), dict(num_panels=7, threads_per_wg=256),
                                  dict(flags=B.FLAG_GLOBAL_MATCHING), dict(flags=B.FLAG_NO_REORDER)])
def test_roundtrip_under_options(opts):
    cfg = gen.scaled(gen.config(3), 8)
    W = gen.make_matrix(cfg, 0)
    A = E.ecspmv_build_dense(W, E.make_opts(**opts))
    assert roundtrip_ok(A, W)


def test_roundtrip_edge_shapes():
    rng = np.random.default_rng(0)
    cases = [np.zeros((5, 9), dtype=np.float16), np.ones((1, 1), dtype=np.float16),
             gen.small_random(1, 3000, 0.5, 1)[0], gen.small_random(300, 1, 0.5, 2)[0],
             gen.small_random(64, 6000, 0.001, 3)[0], gen.small_random(33, 1000, 1.5, 4)[0]]
    W = np.zeros((4, 70), dtype=np.float16)
    W.view(np.uint16)[:] = 0x8000                                               # all -0: nothing stored
    cases.append(W)
    W = np.zeros((3, 600), dtype=np.float16)
    W[0, [0, 599]] = 1.0                                                        # one gap of 599 columns
    W[2, 300] = -2.0
    cases.append(W)
    for W in cases:
        A = E.ecspmv_build_dense(W)
        assert roundtrip_ok(A, W), W.shape


def test_strided_input():
    big = gen.small_random(40, 500, 0.4, 9)[0]
    W = big[:, :333]                                                            # ld = 500 > n = 333
    A = E.ecspmv_build_dense(W)
    assert roundtrip_ok(A, np.ascontiguousarray(W))


# ---- the image, read by an independent Python decoder ----------------------------------------------------------

def test_python_reading_of_the_image_agrees():
    cfg = gen.scaled(gen.config(1), 8)
    W = gen.make_matrix(cfg, 0)
    A = E.ecspmv_build_dense(W)
    r, c, v = pyformat.triples(A.ecspmv_export_image())
    rr, cc, vv = orc.pattern_triples(W)
    assert np.array_equal(r, rr) and np.array_equal(c, cc) and np.array_equal(v, vv)


def test_delta_index_rules():
    """Section 6.2: deltas fit 8 bits, the first delta of a base-carrying unit is 0 and its base is the absolute
    first column (as in the worked example: base 2, deltas 0 2 -> columns 2 4), columns strictly increase."""
    cfg = gen.scaled(gen.config(3), 8)
    W = gen.make_matrix(cfg, 0)
    bits = W.view(np.uint16)
    A = E.ecspmv_build_dense(W)
    nblock = nlane = 0
    for u in pyformat.walk(A.ecspmv_export_image()):
        assert u["deltas"].min() >= 0 and u["deltas"].max() <= 255
        if u["kind"] == "block":
            nblock += 1
            assert u["deltas"][0] == 0 and u["cols"][0] == u["base"]
            assert np.all(np.diff(u["cols"]) > 0)
            assert len(set(u["rows"].tolist())) == u["g"]                         # g distinct rows
            for k, row in enumerate(u["rows"]):                                   # fully dense, right values
                assert np.array_equal(bits[row, u["cols"]], u["values"][:, k])
                assert np.all((u["values"][:, k] & 0x7FFF) != 0)
        else:
            nlane += 1
            if u["first_of_row"]:
                assert u["deltas"][0] == 0
            stored = (u["values"] & 0x7FFF) != 0
            assert np.array_equal(bits[u["row"], u["cols"][stored]], u["values"][stored])
            assert np.all(np.diff(u["cols"]) >= 0)
    assert nblock > 0 and nlane > 0


def test_worked_example_of_the_delta_scheme():
    """The paper's Fig. 4 example in this layout: a 2-grained block over columns 2, 4, 5, 6 (continued to a full
    64-column unit) has base 2 and deltas 0, 2, 1, 1, ..."""
    cols = np.array([2, 4, 5, 6] + list(range(10, 130, 2)))
    assert len(cols) == 64
    W = np.zeros((2, 200), dtype=np.float16)
    W[:, cols] = np.arange(1, 129, dtype=np.float16).reshape(2, 64)
    A = E.ecspmv_build_dense(W, E.make_opts(num_panels=1))
    units = list(pyformat.walk(A.ecspmv_export_image()))
    assert len(units) == 1 and units[0]["kind"] == "block" and units[0]["g"] == 2
    u = units[0]
    assert u["base"] == 2 and u["deltas"][:4].tolist() == [0, 2, 1, 1]
    assert u["cols"].tolist() == cols.tolist()
    assert np.array_equal(u["values"].T, W[:, cols].view(np.uint16))            # values[j*G + k]: column j, row k


def test_gap_filling_and_tail_padding_of_residual_rows():
    """Section 6.2 / 6.3.1: across a gap wider than 255 columns explicit zeros are stored every 255 columns; a
    residual row is padded with zeros to a whole number of 16-element lane units."""
    W = np.zeros((1, 2000), dtype=np.float16)
    W[0, [10, 11, 700, 1999]] = [1, 2, 3, 4]
    A = E.ecspmv_build_dense(W)
    st = A.ecspmv_stats()
    # 11 -> 700: gap 689 = 255 + 255 + 179 (2 fillers); 700 -> 1999: gap 1299 = 5 * 255 + 24 (5 fillers)
    assert st.gap_pad_elements == 7
    assert st.pad_elements == 7 + (16 - (4 + 7) % 16)
    lanes = [u for u in pyformat.walk(A.ecspmv_export_image())]
    assert len(lanes) == 1
    d, v = lanes[0]["deltas"], lanes[0]["values"]
    assert d[:11].tolist() == [0, 1, 255, 255, 179, 255, 255, 255, 255, 255, 24]
    assert lanes[0]["cols"][:11].tolist() == [10, 11, 266, 521, 700, 955, 1210, 1465, 1720, 1975, 1999]
    assert np.all(v[[2, 3, 5, 6, 7, 8, 9]] == 0) and np.all(d[11:] == 0) and np.all(v[11:] == 0)
    assert roundtrip_ok(A, W)


# ---- block extraction (Algorithms 1 and 2): invariants and cases with a known answer ----------------------------

def block_cover(A, shape):
    g, rows, cols = A.ecspmv_block_sets()
    cover = np.zeros(shape, dtype=np.int32)
    gran = np.zeros(shape, dtype=np.int32)
    p = 0
    for u in range(len(g)):
        rs = rows[p:p + g[u]]
        p += g[u]
        cover[np.ix_(rs, cols[u])] += 1
        gran[np.ix_(rs, cols[u])] = g[u]
    return g, cover, gran


def test_blocks_partition_and_are_dense():
    cfg = gen.scaled(gen.config(1), 8)
    W = gen.make_matrix(cfg, 0)
    stored = (W.view(np.uint16) & 0x7FFF) != 0
    A = E.ecspmv_build_dense(W)
    g, cover, _ = block_cover(A, W.shape)
    assert set(np.unique(g)) <= {2, 4, 8}
    assert cover.max() == 1                                  # no entry is in two blocks
    assert not np.any((cover == 1) & ~stored)                # blocks hold stored entries only (fully dense)
    st = A.ecspmv_stats()
    assert int(cover.sum()) == st.nnz - st.nnz_by_g[0]       # the rest is the residual
    assert st.nnz_by_g[1] > 0.3 * st.nnz                     # two random rows here share many columns


def test_identical_rows_reach_the_coarsest_granularity():
    rng = np.random.default_rng(5)
    pat = np.sort(rng.choice(3000, size=640, replace=False))
    W = np.zeros((16, 3000), dtype=np.float16)
    W[:, pat] = (rng.standard_normal((16, 640)) * 0.02 + 1).astype(np.float16)
    for maxg in (2, 4, 8, 16):
        A = E.ecspmv_build_dense(W, E.make_opts(max_granularity=maxg, num_panels=1))
        st = A.ecspmv_stats()
        t = {2: 1, 4: 2, 8: 3, 16: 4}[maxg]
        assert st.nnz_by_g[t] == 16 * 640, (maxg, list(st.nnz_by_g))     # 640 = 10 whole units: all of it
        assert abs(st.x_access_cost - 16 * 640 / maxg) < 1e-6
        assert roundtrip_ok(A, W)


def test_multi_round_extraction_splits_a_row_between_two_partners():
    """Section 4.3's example in spirit: row 2 shares one half of its columns with row 0 and the other half with
    row 1; rounds 1 and 2 put both halves into 2-grained blocks."""
    W = np.zeros((3, 1024), dtype=np.float16)
    a = np.arange(0, 256, 2)            # 128 columns shared by rows 0 and 2
    b = np.arange(512, 768, 2)          # 128 columns shared by rows 1 and 2
    W[0, a] = 1
    W[1, b] = 2
    W[2, a] = 3
    W[2, b] = 4
    A = E.ecspmv_build_dense(W, E.make_opts(num_panels=1))
    g, rows, cols = A.ecspmv_block_sets()
    assert g.tolist() == [2, 2, 2, 2]
    pairs = sorted(tuple(sorted(rows[2 * i:2 * i + 2].tolist())) for i in range(4))
    assert pairs == [(0, 2), (0, 2), (1, 2), (1, 2)]
    assert A.ecspmv_stats().nnz_by_g[0] == 0


def test_columns_beyond_whole_units_stay_in_the_residual():
    W = np.zeros((2, 500), dtype=np.float16)
    W[:, :100] = 1.0                    # 100 shared columns: one unit of 64, 36 left over per row
    A = E.ecspmv_build_dense(W, E.make_opts(num_panels=1))
    st = A.ecspmv_stats()
    assert st.nnz_by_g[1] == 128 and st.nnz_by_g[0] == 72


def test_a_wide_gap_breaks_a_unit():
    """Columns farther apart than the delta range are not put into one unit (Section 6.2)."""
    W = np.zeros((2, 4000), dtype=np.float16)
    cols = np.concatenate([np.arange(0, 40), np.arange(1000, 1040)])       # two runs of 40, gap of 961
    W[:, cols] = 1.0
    A = E.ecspmv_build_dense(W, E.make_opts(num_panels=1))
    st = A.ecspmv_stats()
    assert st.nnz_by_g[1] == 0 and st.nnz_by_g[0] == 160                    # neither run fills a unit


# ---- storage accounting (Section 8.2) ---------------------------------------------------------------------------

def test_byte_accounting():
    cfg = gen.scaled(gen.config(4), 4)
    W = gen.make_matrix(cfg, 0)
    nnz = int(np.count_nonzero(W))
    m = W.shape[0]
    A = E.ecspmv_build_dense(W, E.make_opts(max_granularity=1))            # delta compression only
    st = A.ecspmv_stats()
    assert st.csr32_bytes == 6 * nnz + 4 * (m + 1) and st.csr16_bytes == 4 * nnz + 4 * (m + 1)
    assert st.image_bytes == st.value_bytes + st.delta_bytes + st.meta_bytes + st.slack_bytes
    assert st.image_bytes == A.ecspmv_device_bytes() and st.image_bytes % 256 == 0
    stored_elems = nnz + st.pad_elements
    assert st.value_bytes == 2 * stored_elems and st.delta_bytes == stored_elems
    assert st.pad_elements <= 15 * m + st.gap_pad_elements
    assert 0.49 < st.image_bytes / st.csr32_bytes < 0.57                  # FP16 value + 8-bit delta: about half of CSR-32
    B2 = E.ecspmv_build_dense(W)                                          # with blocks: fewer index bytes
    s2 = B2.ecspmv_stats()
    assert s2.delta_bytes < st.delta_bytes and s2.x_access_cost < st.x_access_cost
    # one gap is recorded per residual entry except the first of each row
    assert sum(s2.delta_hist) == s2.nnz_by_g[0] - _rows_with_residual(B2)


def _rows_with_residual(A):
    rows = set()
    for u in pyformat.walk(A.ecspmv_export_image()):
        if u["kind"] == "lane":
            rows.add(u["row"])
    return len(rows)


def test_panels_are_contiguous_and_cover_all_rows():
    W = gen.small_random(1000, 300, 0.2, 8)[0]
    A = E.ecspmv_build_dense(W, E.make_opts(num_panels=37))
    img = A.ecspmv_export_image()
    ih = pyformat.image_header(img)
    assert ih["num_panels"] == 37 and ih["m"] == 1000 and ih["n"] == 300
    nxt = 0
    for p in range(37):
        hdr = img[256 + p * ih["panel_stride"]:][:128].view(np.uint32)
        assert hdr[0] == nxt and hdr[1] >= 1
        nxt += int(hdr[1])
    assert nxt == 1000


def test_few_long_rows_get_more_panels_so_that_the_partial_sums_fit_lds():
    """64 dense rows of 60000 columns: with the usual 16 rows per panel a panel would hold 60000 lane units (240 KB of
    partial sums); the automatic choice makes more panels instead of refusing the matrix."""
    W = np.full((64, 60000), 0.5, dtype=np.float16)
    A = E.ecspmv_build_dense(W, E.make_opts(max_granularity=1))
    st = A.ecspmv_stats()
    assert st.num_panels > 4 and st.lds_bytes <= 160 * 1024
    assert st.nnz == 64 * 60000
    with pytest.raises(E.EcspmvError) as e:                        # an explicit panel count is taken as given
        E.ecspmv_build_dense(W, E.make_opts(max_granularity=1, num_panels=2))
    assert e.value.status == B.ERR_UNSUPPORTED
