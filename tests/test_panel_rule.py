"""The library's work distribution (its own rule, not the paper's: Section 5 only asks for even work per processing
unit): contiguous row panels with about equal numbers of stored entries.  Hand values, read back from the panel headers
of the image.  No GPU."""
import numpy as np
import pytest

import paper_2507_12205_amd as E

import pyformat


def bounds_for(row_nnz, panels, n=64):
    W = np.zeros((len(row_nnz), n), dtype=np.float16)
    for i, k in enumerate(row_nnz):
        W[i, :k] = 1.0
    A = E.ecspmv_build_dense(W, E.make_opts(num_panels=panels, max_granularity=1))
    assert A.ecspmv_stats().num_panels == min(panels, len(row_nnz))
    return pyformat.panel_bounds(A.ecspmv_export_image())


def test_even_rows_split_evenly():
    assert bounds_for([1] * 8, 4) == [0, 2, 4, 6, 8]


def test_a_panel_ends_where_the_running_count_reaches_its_share():
    # 20 entries, 2 panels: the first panel's share (10) is reached after row 0; the empty rows that follow cost
    # nothing and stay with it until the count would pass the share
    assert bounds_for([10, 0, 0, 0, 10, 0, 0, 0], 2) == [0, 4, 8]


def test_the_row_that_crosses_the_share_goes_where_it_lands_closer():
    # 3 + 3 + 10 + 4 = 20, share 10: after rows 0, 1 the count is 6 (4 short); with row 2 it is 16 (6 over) -> row 2
    # starts the second panel
    assert bounds_for([3, 3, 10, 4], 2) == [0, 2, 4]
    # 4 + 4 + 5 + 7 = 20: after rows 0, 1 the count is 8 (2 short); with row 2 it is 13 (3 over) -> row 2 starts panel 1
    assert bounds_for([4, 4, 5, 7], 2) == [0, 2, 4]
    # 4 + 5 + 4 + 7 = 20: after row 0 the count is 4; with row 1 it is 9 (1 short); with row 2 it is 13 (3 over)
    assert bounds_for([4, 5, 4, 7], 2) == [0, 2, 4]
    # 9 + 2 + 9 = 20: after row 0 the count is 9 (1 short); with row 1 it is 11 (1 over): a tie stays short
    assert bounds_for([9, 2, 9], 2) == [0, 1, 3]


def test_every_panel_owns_a_row_and_an_empty_matrix_is_split_by_rows():
    assert bounds_for([0] * 6, 4) == [0, 2, 4, 5, 6]
    assert bounds_for([5, 5, 5], 8) == [0, 1, 2, 3]                     # never more panels than rows
    assert bounds_for([30, 0, 0, 0], 4) == [0, 1, 2, 3, 4]              # one heavy row cannot starve the later panels


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_panels_are_balanced_within_one_row(seed):
    rng = np.random.default_rng(seed)
    nnz = rng.integers(0, 60, size=200).tolist()
    P = 16
    b = bounds_for(nnz, P)
    assert len(b) == P + 1 and all(x < y for x, y in zip(b, b[1:]))
    pre = np.concatenate([[0], np.cumsum(nnz)])
    for p in range(1, P):                                               # every cut lies within one row of its target
        target = pre[-1] * p / P
        assert pre[b[p]] - max(nnz) <= target <= pre[b[p]] + max(nnz)
