"""GPU parity of the path with index compression switched off (delta_bits = 16: absolute 16-bit columns through the
same kernel, the first step of the ablation of the paper's Section 8.3) against the FP64 CPU oracle, element by element,
inside the acceptance band |y_i - y_ref_i| <= 2e-3 * S_i + 1e-6 with S_i = sum_j |W_ij x_j|."""
import numpy as np
import pytest

from oracle import oracle as orc
from workloads import generators as gen

pytestmark = pytest.mark.gpu

REL, ABS = 2e-3, 1e-6


@pytest.fixture(scope="module")
def E():
    import torch
    assert torch.cuda.is_available()
    import paper_2507_12205_amd as pkg
    from paper_2507_12205_amd import device
    pkg.binding.lib()            # fails loudly if the HIP library is not built
    pkg.device = device
    return pkg


def run(E, W, x, **opts):
    import torch
    A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=16, **opts))
    assert A.ecspmv_stats().delta_bits == 16
    E.device.upload(A)
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    yd = torch.full((W.shape[0],), float("nan"), dtype=torch.float16, device="cuda")
    E.device.run(A, xd, yd)
    torch.cuda.synchronize()
    return A, yd.cpu().numpy()


def check(E, W, x, label, **opts):
    print(f"[case] delta16 {label} shape={W.shape}", flush=True)
    A, y = run(E, W, x, **opts)
    y_ref, S = orc.spmv_oracle(W, x)
    assert not np.isnan(y.astype(np.float64)).any(), "a row of y was not written"
    err = np.abs(y.astype(np.float64) - y_ref)
    lim = REL * S + ABS
    bad = np.nonzero(err > lim)[0]
    assert bad.size == 0, f"{label}: {bad.size} rows out of band, first {bad[:5]}, err {err[bad[:5]]}, lim {lim[bad[:5]]}"
    return A, y


@pytest.mark.parametrize("cid,div", [(0, 1), (1, 4), (2, 4), (3, 4), (4, 4)])
def test_configs_reduced(E, cid, div):
    cfg = gen.scaled(gen.config(cid), div) if div > 1 else gen.config(cid)
    for sid in range(len(cfg.shapes)):
        if cid == 3 and sid in (1, 2, 3, 5):
            continue
        W, x = gen.make_case(cfg, sid)
        check(E, W, x, f"cfg{cid}/{cfg.shapes[sid][0]}/div{div}")


@pytest.mark.parametrize("maxg", [1, 2, 8, 16])
def test_granularity_caps(E, maxg):
    W, x = gen.make_case(gen.scaled(gen.config(1), 4), 0)
    A, _ = check(E, W, x, f"maxg{maxg}", max_granularity=maxg)
    st = A.ecspmv_stats()
    for t in range(1, 5):
        if (1 << t) > maxg:
            assert st.nnz_by_g[t] == 0
    if maxg > 1:
        assert st.nnz_by_g[1] > 0


def test_identical_rows_make_coarse_blocks(E):
    rng = np.random.default_rng(21)
    base = rng.random(2048) < 0.5
    W = np.zeros((64, 2048), dtype=np.float16)
    W[:, base] = (rng.standard_normal((64, int(base.sum()))) * 0.02).astype(np.float16)
    x = gen.make_vector(2048, seed=22)
    for maxg in (4, 8, 16):
        A, _ = check(E, W, x, f"identical/maxg{maxg}", max_granularity=maxg, num_panels=2)
        assert A.ecspmv_stats().nnz_by_g[{4: 2, 8: 3, 16: 4}[maxg]] > 0


def test_unit_vectors_return_columns_bit_for_bit(E):
    """x = e_j: y must be column j of W exactly (w * 1 is exact, every other term is 0): checks the column of every
    stored index, including the widest column a 16-bit index can hold."""
    rng = np.random.default_rng(5)
    n = 65535
    W = np.zeros((48, n), dtype=np.float16)
    cols = np.unique(np.concatenate([rng.integers(0, n, 400), [0, 1, 255, 256, 4095, 4096, 65534]]))
    W[:, cols] = (rng.standard_normal((48, len(cols))) * 0.02).astype(np.float16)
    W[rng.random(W.shape) < 0.3] = 0
    import torch
    A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=16, max_granularity=8))
    E.device.upload(A)
    for j in [0, 1, 255, 256, 4096, 65534] + cols[::37].tolist():
        x = np.zeros(n, dtype=np.float16)
        x[j] = 1.0
        xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
        yd = torch.full((48,), float("nan"), dtype=torch.float16, device="cuda")
        E.device.run(A, xd, yd)
        torch.cuda.synchronize()
        got = yd.cpu().numpy().view(np.uint16)
        want = W[:, j].view(np.uint16).copy()
        want[(want & 0x7FFF) == 0] = 0                       # an empty row sum is +0
        assert np.array_equal(got, want), f"column {j}"


def test_edge_shapes(E):
    rng = np.random.default_rng(3)
    for m, n, rho in [(1, 1, 1.0), (3, 17, 0.5), (70, 1000, 0.05), (257, 129, 0.9), (16, 5000, 0.002)]:
        W = ((rng.random((m, n)) < rho) * rng.standard_normal((m, n)) * 0.02).astype(np.float16)
        x = rng.standard_normal(n).astype(np.float16)
        check(E, W, x, f"edge {m}x{n}")


def test_batch_of_three_in_one_launch(E):
    import torch
    cfg = gen.scaled(gen.config(3), 4)
    As, xs, ys, refs = [], [], [], []
    for sid in (0, 4, 6):
        W, x = gen.make_case(cfg, sid)
        A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=16))
        E.device.upload(A)
        As.append(A)
        xs.append(torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16))
        ys.append(torch.full((W.shape[0],), float("nan"), dtype=torch.float16, device="cuda"))
        refs.append(orc.spmv_oracle(W, x))
    E.Batch(As, [t.data_ptr() for t in xs], [t.data_ptr() for t in ys]).ecspmv_run_batch(int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    for y, (y_ref, S) in zip(ys, refs):
        ok, ratio = orc.within_band(y.cpu().numpy(), y_ref, S, REL, ABS)
        assert ok, ratio


def test_several_right_hand_sides_are_refused(E):
    import torch
    W, _ = gen.make_case(gen.scaled(gen.config(1), 8), 0)
    A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=16))
    E.device.upload(A)
    X = torch.zeros((W.shape[1], 2), dtype=torch.float16, device="cuda")
    Y = torch.zeros((W.shape[0], 2), dtype=torch.float16, device="cuda")
    with pytest.raises(E.EcspmvError) as e:
        E.device.run_multi(A, X, Y)
    assert e.value.status == E.binding.ERR_UNSUPPORTED
