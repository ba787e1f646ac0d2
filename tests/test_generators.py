"""The synthetic workload generators: seeded, of the stated density and structure."""
import numpy as np

from workloads import generators as gen


def test_reproducible_and_distinct_copies():
    cfg = gen.scaled(gen.config(1), 8)
    a = gen.make_matrix(cfg, 0, seed=0, copy=0)
    b = gen.make_matrix(cfg, 0, seed=0, copy=0)
    c = gen.make_matrix(cfg, 0, seed=0, copy=1)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    assert not np.array_equal(a.view(np.uint16), c.view(np.uint16))


def test_density_matches_config():
    for cid, div in ((0, 1), (1, 8), (3, 8), (4, 8)):
        cfg = gen.scaled(gen.config(cid), div)
        for sid, (_, m, n) in enumerate(cfg.shapes[:2]):
            mask = gen.make_mask(cfg, m, n, 0, sid, 0)
            assert abs(mask.mean() - cfg.density) < 0.02, (cid, sid, mask.mean())


def test_column_correlation_present_only_where_stated():
    cfg = gen.scaled(gen.config(3), 8)
    _, m, n = cfg.shapes[0]
    col = gen.make_mask(cfg, m, n).mean(axis=0)
    assert col.std() > 0.15                       # Beta(0.5, 0.5): widely spread column densities
    cfg4 = gen.scaled(gen.config(4), 8)
    _, m, n = cfg4.shapes[0]
    col = gen.make_mask(cfg4, m, n).mean(axis=0)
    assert col.std() < 0.03                       # i.i.d. Bernoulli(0.2)


def test_planted_blocks_are_dense():
    cfg = gen.config(0)
    _, m, n = cfg.shapes[0]
    mask = gen.make_mask(cfg, m, n)
    blocks = gen._planted_blocks(gen._rng(0, cfg.cid, 0, 0, 1), cfg, m, n)
    assert len(blocks) == 8
    for rows, cols in blocks:
        assert len(rows) == 16 and len(cols) == 32
        assert mask[np.ix_(rows, cols)].all()


def test_values_and_vector_scale():
    cfg = gen.scaled(gen.config(1), 8)
    W, x = gen.make_case(cfg)
    nz = W[W != 0].astype(np.float64)
    assert W.dtype == np.float16 and x.dtype == np.float16
    assert abs(nz.std() - 0.02) < 0.002 and abs(x.astype(np.float64).std() - 1.0) < 0.1
