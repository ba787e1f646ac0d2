"""GPU parity of the FP32 path (FP32 values, x and y: the paper's other precision) against the FP64 CPU oracle,
element by element.  Band: |y_i - y_ref_i| <= 2e-3 * S_i + 1e-6, S_i = sum_j |W_ij x_j| (the same band as FP16: FP32
products now round, 2^-24 each, and so does every addition; nnz_row * 2^-23 * S_i stays below it for the rows here;
the stored result is FP32, 2^-24 |y_i|)."""
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
    pkg.binding.lib()
    pkg.device = device
    return pkg


def make_f32(W16, seed):
    rng = np.random.default_rng(seed)
    return W16.astype(np.float32) * (1.0 + rng.uniform(-1e-3, 1e-3, W16.shape)).astype(np.float32)


def check(E, W, x, label, **opts):
    import torch
    print(f"[case] f32 {label} shape={W.shape}", flush=True)
    A = E.ecspmv_build_dense_f32(W, E.make_opts(**opts))
    assert A.ecspmv_stats().value_bits == 32
    E.device.upload(A)
    xd = torch.from_numpy(x).cuda()
    yd = torch.full((W.shape[0],), float("nan"), dtype=torch.float32, device="cuda")
    E.device.run(A, xd, yd)
    torch.cuda.synchronize()
    y = yd.cpu().numpy()
    assert not np.isnan(y).any(), "a row of y was not written"
    y_ref, S = orc.spmv_oracle_f32(W, x)
    err = np.abs(y.astype(np.float64) - y_ref)
    lim = REL * S + ABS
    bad = np.nonzero(err > lim)[0]
    assert bad.size == 0, f"{label}: {bad.size} rows out of band, first {bad[:5]}, err {err[bad[:5]]}, lim {lim[bad[:5]]}"
    # FP32 keeps far more than the band asks for: a much tighter check catches a path that rounds through FP16
    assert np.all(err <= 2.0 ** -17 * S + 1e-9), "more error than FP32 accumulation explains"
    return A, y


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("cid,div", [(0, 1), (1, 4), (2, 4), (3, 4), (4, 4)])
def test_configs_reduced(E, cid, div, bits):
    cfg = gen.scaled(gen.config(cid), div) if div > 1 else gen.config(cid)
    for sid in range(len(cfg.shapes)):
        if cid == 3 and sid in (1, 2, 3, 5):
            continue
        W16, x16 = gen.make_case(cfg, sid)
        x = (x16.astype(np.float32) * np.float32(1.0001)).astype(np.float32)
        check(E, make_f32(W16, sid), x, f"cfg{cid}/{cfg.shapes[sid][0]}/div{div}/bits{bits}", delta_bits=bits)


@pytest.mark.parametrize("maxg", [1, 2, 4, 8, 16])
def test_granularity_caps(E, maxg):
    rng = np.random.default_rng(11)
    base = rng.random(2048) < 0.4
    W = np.zeros((64, 2048), dtype=np.float32)                        # identical rows: blocks up to the cap
    W[:, base] = (rng.standard_normal((64, int(base.sum()))) * 0.02).astype(np.float32)
    W[::3, ::7] = 0.5
    x = rng.standard_normal(2048).astype(np.float32)
    A, _ = check(E, W, x, f"identical/maxg{maxg}", max_granularity=maxg, num_panels=2)
    st = A.ecspmv_stats()
    if maxg > 1:
        assert st.nnz_by_g[{2: 1, 4: 2, 8: 3, 16: 4}[maxg]] > 0


def test_edge_shapes(E):
    rng = np.random.default_rng(3)
    f = lambda p: (make_f32(p[0], 1), p[1].astype(np.float32))
    cases = {
        "single_row": f(gen.small_random(1, 777, 0.5, 1)),
        "single_col": f(gen.small_random(333, 1, 0.7, 2)),
        "one_by_one": (np.array([[0.5]], dtype=np.float32), np.array([2.0], dtype=np.float32)),
        "ragged_n": f(gen.small_random(70, 1003, 0.3, 3)),
        "dense": f(gen.small_random(64, 512, 1.1, 4)),
        "gaps_over_255": f(gen.small_random(128, 5000, 0.002, 5)),
        "all_zero": (np.zeros((50, 80), dtype=np.float32), rng.standard_normal(80).astype(np.float32)),
        "wide_x": f(gen.small_random(16, 30000, 0.05, 6)),
    }
    for label, (W, x) in cases.items():
        check(E, W, x, label)
        check(E, W, x, label + "/4bit", delta_bits=4)


@pytest.mark.parametrize("panels,threads", [(1, 64), (3, 256), (64, 512), (500, 128)])
def test_launch_shapes(E, panels, threads):
    W16, x16 = gen.small_random(517, 1031, 0.35, seed=5)
    check(E, make_f32(W16, 2), x16.astype(np.float32), f"P{panels}/T{threads}", num_panels=panels, threads_per_wg=threads)


def test_unit_vectors_return_columns_bit_exactly(E):
    import torch
    W = make_f32(gen.make_matrix(gen.scaled(gen.config(3), 8), 0), 4)
    A = E.ecspmv_build_dense_f32(W)
    E.device.upload(A)
    m, n = W.shape
    yd = torch.empty(m, dtype=torch.float32, device="cuda")
    for j in (0, 1, n // 2, n - 1):
        x = np.zeros(n, dtype=np.float32)
        x[j] = 1.0
        E.device.run(A, torch.from_numpy(x).cuda(), yd)
        torch.cuda.synchronize()
        col = W[:, j].copy()
        col[col == 0] = 0
        assert np.array_equal(yd.cpu().numpy().view(np.uint32), col.view(np.uint32)), f"column {j}"


def test_batch_with_fp16_and_fp32_matrices(E):
    """ecspmv_run_batch over FP16 and FP32 matrices: launches are split where the value width changes; every y equals
    the lone launch's, bit for bit."""
    import torch
    mats, xs, lone = [], [], []
    for i, vb in enumerate((16, 32, 32, 16)):
        W16, x16 = gen.small_random(200 + 50 * i, 900 + 100 * i, 0.3, seed=40 + i)
        if vb == 32:
            A = E.ecspmv_build_dense_f32(make_f32(W16, i))
            xd = torch.from_numpy(x16.astype(np.float32)).cuda()
            yd = torch.empty(W16.shape[0], dtype=torch.float32, device="cuda")
        else:
            A = E.ecspmv_build_dense(W16)
            xd = torch.from_numpy(x16.view(np.int16)).cuda().view(torch.float16)
            yd = torch.empty(W16.shape[0], dtype=torch.float16, device="cuda")
        E.device.upload(A)
        E.device.run(A, xd, yd)
        torch.cuda.synchronize()
        mats.append(A)
        xs.append(xd)
        lone.append(yd.clone())
    ys = [torch.zeros_like(l) for l in lone]
    E.ecspmv_run_batch(mats, [x.data_ptr() for x in xs], [y.data_ptr() for y in ys],
                       torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for y, l in zip(ys, lone):
        assert torch.equal(y, l)


def check_multi(E, W, nb, label, x_offset=0, **opts):
    """Y = W X with FP32 values: every column inside the band of the FP32 oracle, and bit-equal to the single-vector
    launch on that column."""
    import torch
    print(f"[case] f32 multi {label} nb={nb} shape={W.shape} x_offset={x_offset}", flush=True)
    m, n = W.shape
    A = E.ecspmv_build_dense_f32(W, E.make_opts(**opts))
    E.device.upload(A)
    rng = np.random.default_rng(nb + n)
    X = rng.standard_normal((n, nb)).astype(np.float32)
    flat = torch.zeros(n * nb + 16, dtype=torch.float32, device="cuda")
    Xd = flat[x_offset:x_offset + n * nb].view(n, nb)
    Xd.copy_(torch.from_numpy(X).cuda())
    Yd = torch.full((m, nb), float("nan"), dtype=torch.float32, device="cuda")
    E.device.run_multi(A, Xd, Yd)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()
    assert not np.isnan(Y).any(), "an entry of Y was not written"
    yd = torch.empty(m, dtype=torch.float32, device="cuda")
    for b in range(nb):
        xb = np.ascontiguousarray(X[:, b])
        y_ref, S = orc.spmv_oracle_f32(W, xb)
        err = np.abs(Y[:, b].astype(np.float64) - y_ref)
        assert np.all(err <= REL * S + ABS) and np.all(err <= 2.0 ** -17 * S + 1e-9), (label, b)
        E.device.run(A, torch.from_numpy(xb).cuda(), yd)
        torch.cuda.synchronize()
        assert np.array_equal(yd.cpu().numpy().view(np.uint32), np.ascontiguousarray(Y[:, b]).view(np.uint32)), (label, b)
    return A


@pytest.mark.parametrize("nb", [2, 4, 8])
@pytest.mark.parametrize("bits", [4, 8])
def test_several_right_hand_sides(E, nb, bits):
    for cid, div in ((0, 1), (1, 4), (3, 8)):
        cfg = gen.scaled(gen.config(cid), div) if div > 1 else gen.config(cid)
        check_multi(E, make_f32(gen.make_matrix(cfg, 0), cid), nb, f"cfg{cid}/div{div}/bits{bits}", delta_bits=bits)
    W = np.zeros((24, 900), dtype=np.float32)                        # identical rows: 4-grained sets take part
    W[:, ::2] = np.linspace(0.5, 1.5, 450, dtype=np.float32)
    A = check_multi(E, W, nb, f"4-grained/bits{bits}", delta_bits=bits, flags=E.binding.FLAG_KEEP_SMALL_SETS)
    assert A.ecspmv_stats().nnz_by_g[2] > 0


def test_several_right_hand_sides_split_and_refused(E):
    import torch
    # 4 * n * nb bytes of X exceed LDS: two or four launches with a row stride, aligned and not
    for (m, n, nb) in ((64, 9000, 8), (48, 15000, 4)):
        W = make_f32(gen.small_random(m, n, 0.05, 5 + nb)[0], 9)
        A = check_multi(E, W, nb, f"split {m}x{n}", delta_bits=4, max_granularity=2)
        assert 4 * n * nb + A.ecspmv_stats().meta_stride > 160 * 1024
        check_multi(E, W, nb, f"split {m}x{n}, X four bytes off a 16-byte boundary", x_offset=1, delta_bits=4, max_granularity=2)
    W = np.zeros((16, 3000), dtype=np.float32)
    W[:, ::3] = 1.0                                                  # identical rows: an 8-grained set if asked for
    A = E.ecspmv_build_dense_f32(W, E.make_opts(max_granularity=8))
    assert A.ecspmv_stats().nnz_by_g[3] > 0
    E.device.upload(A)
    X = torch.zeros((3000, 2), dtype=torch.float32, device="cuda")
    Y = torch.zeros((16, 2), dtype=torch.float32, device="cuda")
    with pytest.raises(E.EcspmvError) as e:
        A.ecspmv_run_multi(X.data_ptr(), Y.data_ptr(), 2)
    assert e.value.status == E.binding.ERR_UNSUPPORTED
    torch.cuda.synchronize()
