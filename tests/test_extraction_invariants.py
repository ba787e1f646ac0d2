"""Checks of the library's block extraction that do not go through the extraction oracle: rules every block set must
obey, read off the library's output (Sections 4.1, 6.2, 6.3.1), and what greedy row matching guarantees, against a
brute-force search over all matchings of a few rows (Section 4.3 poses matching as a maximum-weight matching and
solves it greedily).  No GPU."""
import itertools

import numpy as np
import pytest

import paper_2507_12205_amd as E
from paper_2507_12205_amd import binding as B
from workloads import generators as gen

import pyformat


def units_of(A):
    g, rows, cols = A.ecspmv_block_sets()
    out, p = [], 0
    for u in range(len(g)):
        out.append((int(g[u]), [int(v) for v in rows[p:p + g[u]]], [int(v) for v in cols[u]]))
        p += g[u]
    return out


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("cid,div,flags", [(1, 16, 0), (3, 8, 0), (0, 1, 0), (3, 16, B.FLAG_GLOBAL_MATCHING)])
def test_rules_on_the_block_sets(cid, div, flags, bits):
    cfg = gen.scaled(gen.config(cid), div) if div > 1 else gen.config(cid)
    W = gen.make_matrix(cfg, 0)
    if flags & B.FLAG_GLOBAL_MATCHING:
        W = W[:128]
    m, n = W.shape
    pat = (W.view(np.uint16) & 0x7FFF) != 0
    A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=bits, max_granularity=16, flags=flags | B.FLAG_KEEP_SMALL_SETS))
    bounds = pyformat.panel_bounds(A.ecspmv_export_image())
    panel_of = np.searchsorted(bounds, np.arange(m), side="right") - 1
    covered = np.zeros((m, n), dtype=np.int32)
    units = units_of(A)
    for g, rows, cols in units:
        assert g in (2, 4, 8, 16) and len(rows) == g and len(set(rows)) == g            # g distinct rows
        assert len({int(panel_of[r]) for r in rows}) == 1                               # owned by one panel
        d = np.diff(cols)
        assert len(cols) == 64 and np.all(d >= 1) and np.all(d <= (255 if bits == 8 else 15))   # delta range
        assert pat[np.ix_(rows, cols)].all()                                            # fully dense
        covered[np.ix_(rows, cols)] += 1
    assert covered.max() <= 1                                                           # units do not overlap
    # what the blocks do not hold is exactly what the residual rows hold
    resid = np.zeros((m, n), dtype=np.int32)
    for u in pyformat.walk(A.ecspmv_export_image()):
        if u["kind"] == "lane":
            keep = (u["values"] & 0x7FFF) != 0
            np.add.at(resid, (u["row"], u["cols"][keep]), 1)
    assert np.array_equal(covered + resid, pat.astype(np.int32))
    if bits == 8:
        assert units, "these inputs have pairs of rows with 64 shared columns in reach"


def widen(cs):
    return sorted(16 * c + k for c in cs for k in range(16))


def best_matching_weight(sim, unit):
    """Largest total weight over all sets of disjoint pairs whose weight reaches `unit` (brute force)."""
    R = len(sim)

    def rec(free):
        if len(free) < 2:
            return 0
        a, rest = free[0], free[1:]
        best = rec(rest)                                    # a stays single
        for k, b in enumerate(rest):
            if sim[a][b] >= unit:
                best = max(best, sim[a][b] + rec(rest[:k] + rest[k + 1:]))
        return best

    return rec(list(range(R)))


@pytest.mark.parametrize("seed", range(12))
def test_one_round_of_matching_against_brute_force(seed):
    """One round at level 0 on 6-8 rows of 14 hand columns (one hand column = 16 real ones, a unit = 4 hand columns).
    Whatever order rows are popped in and however ties go, greedy matching (Algorithm 2) gives: disjoint pairs; every
    pair shares at least a unit; the first row popped, the one with the most columns, gets a partner it shares the
    most with; no two rows left single could have formed a pair; and the total weight is at least half the best."""
    rng = np.random.default_rng(seed)
    R, C, unit = int(rng.integers(6, 9)), 14, 4
    hand = [set(np.nonzero(rng.random(C) < rng.uniform(0.4, 0.9))[0].tolist()) for _ in range(R)]
    W = np.zeros((R, 16 * C), dtype=np.float16)
    for i, cs in enumerate(hand):
        W[i, widen(cs)] = 1.0
    A = E.ecspmv_build_dense(W, E.make_opts(max_granularity=2, max_rounds=1,
                                            flags=B.FLAG_GLOBAL_MATCHING | B.FLAG_KEEP_SMALL_SETS))
    pairs = {}
    for g, rows, cols in units_of(A):
        assert g == 2
        pairs.setdefault(tuple(sorted(rows)), set()).update(c // 16 for c in cols)
    sim = [[len(hand[a] & hand[b]) if a != b else 0 for b in range(R)] for a in range(R)]
    used = [r for p in pairs for r in p]
    assert len(used) == len(set(used))                                              # disjoint pairs
    for (a, b), cs in pairs.items():
        assert sim[a][b] >= unit and cs <= (hand[a] & hand[b])
        assert len(cs) == sim[a][b] // unit * unit                                  # whole units, as many as fit
    single = [r for r in range(R) if r not in used and len(hand[r]) >= unit]
    for a, b in itertools.combinations(single, 2):
        assert sim[a][b] < unit                                                     # nothing was left on the table
    most = max(len(h) for h in hand)
    tops = [r for r in range(R) if len(hand[r]) == most]
    if len(tops) == 1 and max(sim[tops[0]]) >= unit:                                # the first row popped is unambiguous
        (partner,) = [b if a == tops[0] else a for (a, b) in pairs if tops[0] in (a, b)]
        assert sim[tops[0]][partner] == max(sim[tops[0]])
    got = sum(sim[a][b] for a, b in pairs)
    assert 2 * got >= best_matching_weight(sim, unit)                               # greedy is a 1/2-approximation
