"""Pins for the extraction oracle (hand-derived block sets) and parity of the library's encoder with it.

A "group" below is 16 consecutive columns, so that 4 groups make one 64-column unit: the paper's small examples
(Section 4.3: a row that shares four columns with one row and four others with another) carry over with one paper
column = one group."""
import numpy as np
import pytest

import paper_2507_12205_amd as E
from paper_2507_12205_amd import binding as B
from oracle import extraction_oracle as xo
from workloads import generators as gen


def groups(*ids):
    return {16 * g + k for g in ids for k in range(16)}


def as_sets(block_sets):
    return {g: sorted((tuple(r), tuple(c)) for r, c in units) for g, units in block_sets.items()}


# ---- pins: expected results derived by hand from Algorithms 1 and 2 ----------------------------------------

def test_pin_row_split_between_two_partners():
    """Rows 0 and 1 are disjoint; row 2 holds both their column sets.  Round 1: row 2 is popped first (most
    columns), both partners share 64 columns, the tie goes to row 0 -> block (2, 0) over row 0's columns.
    Round 2: rows 1 and 2 now hold 64 columns each; the tie in the pop order goes to row 1, which takes row 2 ->
    block (1, 2).  Nothing remains, no level-2 block (the two blocks share row 2 but no column)."""
    rows = [groups(3, 4, 5, 6), groups(0, 2, 7, 8), groups(0, 2, 3, 4, 5, 6, 7, 8)]
    bs, resid = xo.hierarchical_block_extraction(rows)
    assert as_sets(bs) == {2: sorted([((2, 0), tuple(sorted(groups(3, 4, 5, 6)))),
                                      ((1, 2), tuple(sorted(groups(0, 2, 7, 8))))])}
    assert resid == [[], [], []]


def test_pin_identical_rows_climb_every_level():
    """Four identical rows of 128 columns: level 0 pairs (0,1) and (2,3); level 1 pairs the two blocks; the
    result is two 4-grained units with member order (0,1,2,3) and nothing else."""
    cols = groups(*range(8))
    bs, resid = xo.hierarchical_block_extraction([set(cols) for _ in range(4)], max_granularity=8)
    s = sorted(cols)
    assert as_sets(bs) == {4: [((0, 1, 2, 3), tuple(s[:64])), ((0, 1, 2, 3), tuple(s[64:]))]}
    assert resid == [[], [], [], []]
    bs2, _ = xo.hierarchical_block_extraction([set(cols) for _ in range(4)], max_granularity=2)
    assert as_sets(bs2) == {2: [((0, 1), tuple(s[:64])), ((0, 1), tuple(s[64:])),
                                ((2, 3), tuple(s[:64])), ((2, 3), tuple(s[64:]))]}


def test_pin_leftover_below_a_unit_stays_residual():
    rows = [set(range(100)), set(range(100))]
    bs, resid = xo.hierarchical_block_extraction(rows)
    assert as_sets(bs) == {2: [((0, 1), tuple(range(64)))]}
    assert resid == [list(range(64, 100))] * 2


def test_pin_gap_wider_than_delta_range_breaks_a_unit():
    cols = set(range(40)) | set(range(1000, 1040))          # two runs of 40 columns, 961 apart
    bs, resid = xo.hierarchical_block_extraction([set(cols), set(cols)])
    assert bs == {} and resid == [sorted(cols)] * 2
    cols = set(range(40)) | set(range(294, 334))            # gap of exactly 255: still one unit
    bs, resid = xo.hierarchical_block_extraction([set(cols), set(cols)])
    s = sorted(cols)
    assert as_sets(bs) == {2: [((0, 1), tuple(s[:64]))]} and resid == [s[64:]] * 2


def test_pin_partner_choice_and_pop_order():
    """Row 3 has the most columns and is popped first; it shares 128 columns with row 1 and 64 with rows 0 and 2,
    so it takes row 1.  Rows 0 and 2 (64 identical columns) are left for each other."""
    rows = [groups(0, 1, 2, 3), groups(4, 5, 6, 7, 8, 9, 10, 11), groups(0, 1, 2, 3),
            groups(0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12)]
    bs, resid = xo.hierarchical_block_extraction(rows, max_granularity=2)
    s1 = sorted(groups(4, 5, 6, 7, 8, 9, 10, 11))
    assert as_sets(bs) == {2: sorted([((3, 1), tuple(s1[:64])), ((3, 1), tuple(s1[64:])),
                                      ((0, 2), tuple(sorted(groups(0, 1, 2, 3))))])}
    assert resid[3] == sorted(groups(0, 1, 2, 3, 12)) and resid[0] == resid[1] == resid[2] == []


def test_pin_form_units_rule():
    taken, rest = xo.form_units(list(range(0, 130, 2)) + [1000], 64, 255)
    assert taken == list(range(0, 128, 2)) and rest == [128, 1000]
    taken, rest = xo.form_units([0, 300] + list(range(301, 364)), 64, 255)      # the gap drops column 0 only
    assert taken == [300] + list(range(301, 364)) and rest == [0]


def test_partition_invariant_on_random_rows():
    rng = np.random.default_rng(1)
    p = rng.uniform(0.1, 0.9, 3000)
    rows = [set(np.nonzero(rng.random(3000) < p)[0].tolist()) for _ in range(12)]
    bs, resid = xo.hierarchical_block_extraction(rows, max_granularity=8)
    seen = [set(r) for r in resid]
    for g, units in bs.items():
        for members, cols in units:
            assert len(members) == g == len(set(members)) and len(cols) == 64
            assert all(b - a <= 255 and b > a for a, b in zip(cols, cols[1:]))
            for m in members:
                assert not (seen[m] & set(cols))                 # no entry twice
                seen[m] |= set(cols)
    assert seen == rows                                          # every entry exactly once
    assert bs.get(2) and bs.get(4)


def test_pin_leftovers_of_a_lifted_block_fall_back_two_levels():
    """A fall-back that reaches down two levels and, on its way, completes a unit with columns that were waiting
    there.  Hand derivation, with a unit of 4 columns and a delta range that admits only neighbouring columns:

      rows 0, 1: columns 0..11      rows 2, 3: columns 0..7      rows 4..7: columns 2..5

    Level 0 (pop order: most columns first): (0,1) share 0..11 -> three units; (2,3) share 0..7 -> two units;
    (4,5) and (6,7) share 2..5 -> one unit each.  Nothing is left, round 2 finds nothing.
    Level 1, rows A=(0,1){0..11}, B=(2,3){0..7}, C=(4,5){2..5}, D=(6,7){2..5}: A is popped, B is its best partner
    (8 shared against 4) -> block AB over 0..7, A keeps 8..11; C takes D -> block CD over 2..5.
    Level 2, rows AB{0..7}, CD{2..5}: they share 2..5 -> the 8-grained block over 2..5.  AB keeps 0,1,6,7: neither
    0,1 nor 6,7 is a unit and 1 -> 6 exceeds the delta range, so all four fall back to A and to B.
    Decoding level 1: A now holds 0,1,6,7 beside its own 8..11.  0,1 stand alone (gap to 6), 6,7,8,9 are four
    neighbours -> one 2-grained unit of rows (0,1); 10,11 and 0,1 fall back to rows 0 and 1.  B holds 0,1,6,7: no
    unit, they fall back to rows 2 and 3."""
    rows = [set(range(12)), set(range(12)), set(range(8)), set(range(8))] + [set(range(2, 6)) for _ in range(4)]
    bs, resid = xo.hierarchical_block_extraction(rows, max_granularity=8, unit=4, max_delta=1)
    assert as_sets(bs) == {8: [((0, 1, 2, 3, 4, 5, 6, 7), (2, 3, 4, 5))], 2: [((0, 1), (6, 7, 8, 9))]}
    assert resid == [[0, 1, 10, 11], [0, 1, 10, 11], [0, 1, 6, 7], [0, 1, 6, 7], [], [], [], []]
    # with the cap on g at 4 the level-2 block does not exist and AB keeps both its units
    bs4, resid4 = xo.hierarchical_block_extraction(rows, max_granularity=4, unit=4, max_delta=1)
    assert as_sets(bs4) == {4: [((0, 1, 2, 3), (0, 1, 2, 3)), ((0, 1, 2, 3), (4, 5, 6, 7)), ((4, 5, 6, 7), (2, 3, 4, 5))],
                            2: [((0, 1), (8, 9, 10, 11))]}
    assert resid4 == [[] for _ in range(8)]


def test_library_agrees_with_the_hand_derived_fall_back():
    """The same matrix through the library: one hand column = 16 real columns, so four hand columns make the
    library's unit of 64, and with 4-bit deltas (range 15) only neighbouring hand columns may follow one another."""
    wide = lambda cs: sorted(16 * c + k for c in cs for k in range(16))
    hand = [set(range(12)), set(range(12)), set(range(8)), set(range(8))] + [set(range(2, 6)) for _ in range(4)]
    W = np.zeros((8, 16 * 12), dtype=np.float16)
    for i, cs in enumerate(hand):
        W[i, wide(cs)] = 1.0
    A = E.ecspmv_build_dense(W, E.make_opts(max_granularity=8, delta_bits=4,
                                            flags=B.FLAG_GLOBAL_MATCHING | B.FLAG_KEEP_SMALL_SETS))
    assert library_block_sets(A) == {8: [((0, 1, 2, 3, 4, 5, 6, 7), tuple(wide([2, 3, 4, 5])))],
                                     2: [((0, 1), tuple(wide([6, 7, 8, 9])))]}
    res = library_residual(A, 8)
    assert [res[i] for i in range(8)] == [wide(c) for c in ([0, 1, 10, 11], [0, 1, 10, 11], [0, 1, 6, 7], [0, 1, 6, 7],
                                                            [], [], [], [])]


# ---- parity: the library's encoder against the oracle -------------------------------------------------------

def library_block_sets(A):
    g, rows, cols = A.ecspmv_block_sets()
    out, p = {}, 0
    for u in range(len(g)):
        out.setdefault(int(g[u]), []).append((tuple(int(v) for v in rows[p:p + g[u]]), tuple(int(v) for v in cols[u])))
        p += g[u]
    return {k: sorted(v) for k, v in out.items()}


def oracle_for_matrix(W, bounds, max_g, panels=None):
    """The oracle run panel by panel: `bounds` cuts contiguous panels, `panels` lists each panel's rows in its order."""
    pat = (W.view(np.uint16) & 0x7FFF) != 0
    if panels is None:
        panels = [list(range(r0, r1)) for r0, r1 in zip(bounds[:-1], bounds[1:])]
    blocks, resid = {}, {}
    for prow in panels:
        rows = [set(np.nonzero(pat[i])[0].tolist()) for i in prow]
        bs, rs = xo.hierarchical_block_extraction(rows, max_granularity=max_g)
        for g, units in bs.items():
            blocks.setdefault(g, []).extend((tuple(prow[m] for m in mem), cols) for mem, cols in units)
        for i, c in enumerate(rs):
            resid[prow[i]] = c
    return {k: sorted(v) for k, v in blocks.items()}, resid


def library_residual(A, m):
    import pyformat
    resid = {i: [] for i in range(m)}
    for u in pyformat.walk(A.ecspmv_export_image()):
        if u["kind"] == "lane":
            keep = (u["values"] & 0x7FFF) != 0
            resid[u["row"]].extend(int(c) for c in u["cols"][keep])
    return resid


@pytest.mark.parametrize("maxg", [2, 4, 8, 16])
def test_encoder_matches_oracle_matching_over_all_rows(maxg):
    """One panel = the whole matrix: row matching over all rows, as the algorithm is printed."""
    cfg = gen.scaled(gen.config(3), 4)
    W = gen.make_matrix(cfg, 0)[:96]
    A = E.ecspmv_build_dense(W, E.make_opts(max_granularity=maxg, flags=B.FLAG_GLOBAL_MATCHING | B.FLAG_KEEP_SMALL_SETS))
    want, want_res = oracle_for_matrix(W, [0, W.shape[0]], maxg)
    assert library_block_sets(A) == want
    assert library_residual(A, W.shape[0]) == want_res
    assert sum(len(v) for v in want.values()) > 50


@pytest.mark.parametrize("cid,div,panels", [(1, 16, 0), (3, 8, 0), (4, 8, 40), (0, 1, 0)])
def test_encoder_matches_oracle_per_panel(cid, div, panels):
    cfg = gen.scaled(gen.config(cid), div) if div > 1 else gen.config(cid)
    W = gen.make_matrix(cfg, 0)
    m = W.shape[0]
    A = E.ecspmv_build_dense(W, E.make_opts(num_panels=panels, flags=B.FLAG_KEEP_SMALL_SETS))
    P = A.ecspmv_stats().num_panels
    assert P == (panels or min(256, max(1, m // 16)))
    import pyformat
    bounds = pyformat.panel_bounds(A.ecspmv_export_image())          # the library's own panels, read from the image
    want, want_res = oracle_for_matrix(W, bounds, 8)
    assert library_block_sets(A) == want
    assert library_residual(A, m) == want_res


# ---- rows brought together before the panels are cut (ECSPMV_FLAG_CLUSTER_ROWS) ------------------------------

def planted(m=512, n=2048, rho=0.1, h=16, w=256, seed=0):
    rng = np.random.default_rng(seed)
    W = ((rng.random((m, n)) < rho) * rng.standard_normal((m, n)) * 0.02).astype(np.float16)
    rows = np.sort(rng.choice(m, h, replace=False))
    cols = np.sort(rng.choice(n, w, replace=False))
    W[np.ix_(rows, cols)] = (0.05 + 0.02 * rng.standard_normal((h, w))).astype(np.float16)
    return W, rows, cols


def test_a_block_on_scattered_rows_is_found_once_rows_are_clustered():
    """One dense 16 x 256 block on rows scattered over a 512-row matrix of density 0.1.  Panels of contiguous rows hold at
    most a row or two of it and find nothing beyond pairs; with the rows brought together first, the block's rows land
    in the same panels and most of it comes out at granularity 8, under otherwise default options."""
    W, rows, cols = planted()
    plain = E.ecspmv_build_dense(W, E.make_opts(flags=B.FLAG_KEEP_SMALL_SETS))
    assert plain.ecspmv_stats().num_panels == 32
    assert plain.ecspmv_stats().nnz_by_g[3] == 0 and plain.ecspmv_stats().nnz_by_g[2] == 0
    A = E.ecspmv_build_dense(W, E.make_opts(flags=B.FLAG_CLUSTER_ROWS | B.FLAG_KEEP_SMALL_SETS))
    st = A.ecspmv_stats()
    assert st.num_panels == 32
    bs = library_block_sets(A)
    S, C = set(rows.tolist()), set(cols.tolist())

    def planted_cells(g):
        return {(r, c) for rs, cs in bs.get(g, []) if set(rs) <= S for r in rs for c in cs if c in C}

    # the block's rows sit in two panels of eight; more than half of it comes out 8-grained (units are 64 columns of a
    # pair's shared columns, so what two pairs took does not always line up one level higher), three quarters of it in blocks
    assert len(planted_cells(8)) >= 0.5 * 16 * 256
    assert {r for rs, _ in bs.get(8, []) if set(rs) <= S for r in rs} == S
    assert len(planted_cells(8) | planted_cells(4) | planted_cells(2)) >= 0.75 * 16 * 256
    # the image still decodes to W, and every row is owned by exactly one panel
    import pyformat
    from oracle import oracle as orc
    r, c, v = A.ecspmv_decode()
    rr, cc, vv = orc.pattern_triples(W)
    o = np.lexsort((c, r))
    assert np.array_equal(r[o], rr) and np.array_equal(c[o], cc) and np.array_equal(v[o], vv)
    owned = pyformat.panel_rows(A.ecspmv_export_image())
    assert any(p != sorted(p) or p != list(range(p[0], p[0] + len(p))) for p in owned)      # panels are not contiguous


@pytest.mark.parametrize("cid,div", [(1, 16), (3, 8)])
def test_encoder_matches_oracle_per_panel_with_clustered_rows(cid, div):
    """Whatever rows a panel is given, extraction inside it is Algorithm 1 on those rows in that order."""
    import pyformat
    cfg = gen.scaled(gen.config(cid), div)
    W = gen.make_matrix(cfg, 0)
    A = E.ecspmv_build_dense(W, E.make_opts(flags=B.FLAG_CLUSTER_ROWS | B.FLAG_KEEP_SMALL_SETS))
    panels = pyformat.panel_rows(A.ecspmv_export_image())
    want, want_res = oracle_for_matrix(W, None, 8, panels=panels)
    assert library_block_sets(A) == want
    assert library_residual(A, W.shape[0]) == want_res
