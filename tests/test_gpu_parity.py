"""GPU parity: the HIP path (through the C ABI) against the FP64 CPU oracle, element by element.

Acceptance band (stated with the metric): |y_i - y_ref_i| <= 2e-3 * S_i + 1e-6 with S_i = sum_j |W_ij x_j|.
It covers FP32 accumulation in a different order (<= nnz_row * 2^-24 * S_i), the FP16 rounding of the stored
result (<= 2^-11 |y_i|) and FP16-subnormal results (the absolute term).
"""
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


def gpu_spmv(E, W, x, opts=None, reps=1):
    import torch
    A = E.ecspmv_build_dense(W, opts)
    E.device.upload(A)
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    yd = torch.full((W.shape[0],), float("nan"), dtype=torch.float16, device="cuda")
    for _ in range(reps):
        E.device.run(A, xd, yd)
    torch.cuda.synchronize()
    return A, yd.cpu().numpy()


def check(E, W, x, opts=None, label=""):
    print(f"[case] {label} shape={W.shape}", flush=True)
    A, y = gpu_spmv(E, W, x, opts)
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
            continue            # same shape and recipe as an earlier one
        W, x = gen.make_case(cfg, sid)
        check(E, W, x, label=f"cfg{cid}/{cfg.shapes[sid][0]}/div{div}")


@pytest.mark.parametrize("maxg", [1, 2, 4, 16])
def test_granularity_caps(E, maxg):
    cfg = gen.scaled(gen.config(3), 4)
    W, x = gen.make_case(cfg, 0)
    A, _ = check(E, W, x, E.make_opts(max_granularity=maxg), label=f"maxg{maxg}")
    st = A.ecspmv_stats()
    for t in range(1, 5):
        if (1 << t) > maxg:
            assert st.nnz_by_g[t] == 0


@pytest.mark.parametrize("panels,threads", [(1, 64), (3, 256), (64, 512), (256, 1024), (500, 128)])
def test_launch_shapes(E, panels, threads):
    W, x = gen.small_random(517, 1031, 0.35, seed=5)
    check(E, W, x, E.make_opts(num_panels=panels, threads_per_wg=threads), label=f"P{panels}/T{threads}")


def test_unit_vectors_return_columns_bit_exactly(E):
    import torch
    cfg = gen.scaled(gen.config(1), 8)
    W, _ = gen.make_case(cfg, 0)
    A = E.ecspmv_build_dense(W)
    E.device.upload(A)
    m, n = W.shape
    yd = torch.empty(m, dtype=torch.float16, device="cuda")
    for j in (0, 1, n // 2, n - 1):
        x = np.zeros(n, dtype=np.float16)
        x[j] = 1.0
        xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
        E.device.run(A, xd, yd)
        torch.cuda.synchronize()
        y = yd.cpu().numpy()
        col = W[:, j].copy()
        col[col == 0] = 0          # -0 -> +0 (zeros are not stored)
        assert np.array_equal(y.view(np.uint16), col.view(np.uint16)), f"column {j}"


def test_all_zero_matrix_gives_plus_zero(E):
    W = np.zeros((300, 200), dtype=np.float16)
    x = gen.make_vector(200, seed=2)
    _, y = gpu_spmv(E, W, x)
    assert np.all(y.view(np.uint16) == 0)


def test_edge_shapes(E):
    rng = np.random.default_rng(3)
    cases = {
        "single_row": gen.small_random(1, 777, 0.5, 1),
        "single_col": gen.small_random(333, 1, 0.7, 2),
        "one_by_one": (np.array([[0.5]], dtype=np.float16), np.array([2.0], dtype=np.float16)),
        "ragged_n": gen.small_random(70, 1003, 0.3, 3),
        "dense": gen.small_random(64, 512, 1.1, 4),
        "very_sparse_gaps_over_255": gen.small_random(128, 5000, 0.002, 5),
        "m_below_cu_count": gen.small_random(7, 2048, 0.4, 6),
    }
    W, x = gen.small_random(200, 600, 0.4, 7)
    W[10:50] = 0                                      # empty rows
    W[:, 100:300] = 0                                 # empty columns
    cases["empty_rows_cols"] = (W, x)
    W = np.zeros((96, 4096), dtype=np.float16)        # rows with exactly one entry, far apart
    W[np.arange(96), rng.integers(0, 4096, 96)] = 1.5
    cases["one_entry_rows"] = (W, gen.make_vector(4096, seed=8))
    for label, (W, x) in cases.items():
        check(E, W, x, label=label)


def test_identical_rows_make_blocks(E):
    """Rows that share every column must end up in g > 1 blocks and still give the right product."""
    rng = np.random.default_rng(11)
    base = rng.random(2048) < 0.4
    W = np.zeros((64, 2048), dtype=np.float16)
    W[:, base] = (rng.standard_normal((64, int(base.sum()))) * 0.02).astype(np.float16)
    x = gen.make_vector(2048, seed=12)
    A, _ = check(E, W, x, E.make_opts(max_granularity=16, num_panels=2), label="identical_rows")
    st = A.ecspmv_stats()
    assert st.nnz_by_g[4] > 0.8 * st.nnz


def test_subnormal_weights_are_not_flushed(E):
    W = np.zeros((40, 1024), dtype=np.float16)
    rng = np.random.default_rng(13)
    mask = rng.random(W.shape) < 0.5
    W.view(np.uint16)[mask] = rng.integers(1, 0x400, int(mask.sum())).astype(np.uint16)   # subnormals only
    x = (np.abs(gen.make_vector(1024, seed=14)) * 32).astype(np.float16)
    A, y = check(E, W, x, label="subnormal_weights")
    assert np.count_nonzero(y) > 30


def test_signed_zero_and_cancellation(E):
    W = np.zeros((8, 256), dtype=np.float16)
    W[:, 0::2] = 1.0
    W[:, 1::2] = -1.0
    x = np.ones(256, dtype=np.float16)
    _, y = check(E, W, x, label="cancellation")
    assert np.all(y == 0)


def test_misaligned_x_and_y(E):
    import torch
    W, x = gen.small_random(130, 999, 0.4, 21)
    A = E.ecspmv_build_dense(W)
    E.device.upload(A)
    xbuf = torch.zeros(999 + 8, dtype=torch.float16, device="cuda")
    ybuf = torch.zeros(130 + 8, dtype=torch.float16, device="cuda")
    xd = xbuf[3:3 + 999]
    xd.copy_(torch.from_numpy(x.view(np.int16)).view(torch.float16))
    yd = ybuf[1:1 + 130]
    A.ecspmv_run(xd.data_ptr(), yd.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    y_ref, S = orc.spmv_oracle(W, x)
    ok, ratio = orc.within_band(yd.cpu().numpy(), y_ref, S, REL, ABS)
    assert ok, ratio
    assert float(ybuf[0]) == 0.0 and float(ybuf[131]) == 0.0      # neighbours untouched


def test_repeatable_bits(E):
    cfg = gen.scaled(gen.config(3), 4)
    W, x = gen.make_case(cfg, 0)
    _, y1 = gpu_spmv(E, W, x)
    _, y2 = gpu_spmv(E, W, x, reps=3)
    assert np.array_equal(y1.view(np.uint16), y2.view(np.uint16))


def test_csr_comparison_kernel(E):
    import torch
    cfg = gen.scaled(gen.config(4), 4)
    W, x = gen.make_case(cfg, 0)
    C = E.ecspmv_csr_build_dense(W)
    E.device.csr_upload(C)
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    yd = torch.empty(W.shape[0], dtype=torch.float16, device="cuda")
    E.device.csr_run(C, xd, yd)
    torch.cuda.synchronize()
    y_ref, S = orc.spmv_oracle(W, x)
    ok, ratio = orc.within_band(yd.cpu().numpy(), y_ref, S, REL, ABS)
    assert ok, ratio


def test_stream_read_checksum(E):
    import torch
    buf = torch.randint(0, 2 ** 31 - 1, (1 << 20,), dtype=torch.int32, device="cuda")
    out = torch.zeros(256, dtype=torch.int32, device="cuda")
    E.ecspmv_stream_read(buf.data_ptr(), buf.numel() * 4, out.data_ptr(), 256, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(out.cpu().numpy().view(np.uint32))
    want = np.bitwise_xor.reduce(buf.cpu().numpy().view(np.uint32))
    assert got == want


@pytest.mark.parametrize("nwords,nwg,threads", [(1 << 20, 256, 1024), ((1 << 20) + 4 * 37, 100, 512), (4 * 50, 7, 256)])
def test_sliced_read_checksum_and_empty_launch(E, nwords, nwg, threads):
    """The launch-floor aids: the sliced read covers every 16 bytes exactly once (ragged slices and workgroups with
    nothing to read included); the empty launch stores one word per workgroup."""
    import torch
    buf = torch.randint(0, 2 ** 31 - 1, (nwords,), dtype=torch.int32, device="cuda")
    out = torch.full((nwg,), 5, dtype=torch.int32, device="cuda")
    sh = torch.cuda.current_stream().cuda_stream
    E.ecspmv_stream_read_sliced(buf.data_ptr(), nwords * 4, out.data_ptr(), nwg, threads, sh)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(out.cpu().numpy().view(np.uint32))
    want = np.bitwise_xor.reduce(buf.cpu().numpy().view(np.uint32))
    assert got == want
    E.ecspmv_empty_launch(out.data_ptr(), nwg, threads, 3, sh)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), np.arange(nwg, dtype=np.int32))
    with pytest.raises(E.EcspmvError):
        E.ecspmv_stream_read_sliced(buf.data_ptr(), nwords * 4, out.data_ptr(), nwg, 384, sh)


def test_errors_from_the_abi(E):
    import torch
    W, x = gen.small_random(20, 100, 0.5, 1)
    A = E.ecspmv_build_dense(W)
    xd = torch.zeros(100, dtype=torch.float16, device="cuda")
    yd = torch.zeros(20, dtype=torch.float16, device="cuda")
    with pytest.raises(E.EcspmvError) as ei:
        A.ecspmv_run(xd.data_ptr(), yd.data_ptr(), 0)
    assert ei.value.status == E.binding.ERR_NOT_UPLOADED
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(E.EcspmvError) as ei:
        A.ecspmv_upload(small.data_ptr(), 256, 0)
    assert ei.value.status == E.binding.ERR_TOO_SMALL


def test_batched_launch_equals_single_launches(E):
    """One launch over several independent SpMVs gives the same bits as one launch each."""
    import torch
    cfg = gen.scaled(gen.config(3), 4)
    mats, xs, ys1, ys2 = [], [], [], []
    for sid in (0, 4, 6, 0, 4):
        W, x = gen.make_case(cfg, sid, copy=len(mats))
        A = E.ecspmv_build_dense(W)
        E.device.upload(A)
        mats.append(A)
        xs.append(torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16))
        ys1.append(torch.full((W.shape[0],), float("nan"), dtype=torch.float16, device="cuda"))
        ys2.append(torch.full((W.shape[0],), float("nan"), dtype=torch.float16, device="cuda"))
    sh = torch.cuda.current_stream().cuda_stream
    for A, x, y in zip(mats, xs, ys1):
        A.ecspmv_run(x.data_ptr(), y.data_ptr(), sh)
    b = E.Batch(mats, [x.data_ptr() for x in xs], [y.data_ptr() for y in ys2])
    b.ecspmv_run_batch(sh)
    torch.cuda.synchronize()
    for y1, y2 in zip(ys1, ys2):
        a, c = y1.cpu().numpy(), y2.cpu().numpy()
        assert not np.isnan(a.astype(np.float32)).any()
        assert np.array_equal(a.view(np.uint16), c.view(np.uint16))


def test_batch_larger_than_one_launch(E):
    import torch
    W, x = gen.small_random(64, 700, 0.4, 31)
    A = E.ecspmv_build_dense(W)
    E.device.upload(A)
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
    ys = [torch.full((64,), float("nan"), dtype=torch.float16, device="cuda") for _ in range(37)]
    E.ecspmv_run_batch([A] * 37, [xd.data_ptr()] * 37, [y.data_ptr() for y in ys], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    y_ref, S = orc.spmv_oracle(W, x)
    for y in ys:
        ok, ratio = orc.within_band(y.cpu().numpy(), y_ref, S, REL, ABS)
        assert ok, ratio


@pytest.mark.parametrize("n", [40000, 65535])
def test_widest_supported_x(E, n):
    """x of up to 65535 entries (128 KB) still fits LDS next to the tables; needs the large-LDS launch attribute."""
    rng = np.random.default_rng(n)
    m = 48
    W = np.zeros((m, n), dtype=np.float16)
    mask = rng.random((m, n)) < 0.05
    W[mask] = (rng.standard_normal(int(mask.sum())) * 0.02).astype(np.float16)
    W[:, n - 1] = 0.5                                  # the last column is used by every row
    x = gen.make_vector(n, seed=n)
    A, y = check(E, W, x, label=f"wide_x_{n}")
    assert A.ecspmv_stats().lds_bytes > 2 * n


def test_too_wide_is_refused_on_the_host(E):
    W = np.zeros((2, 65536), dtype=np.float16)
    with pytest.raises(E.EcspmvError) as ei:
        E.ecspmv_build_dense(W)
    assert ei.value.status == E.binding.ERR_UNSUPPORTED


def test_launches_can_be_captured_in_a_graph(E):
    """ecspmv_run, ecspmv_run_batch and ecspmv_run_multi allocate nothing and set no memory: a captured graph of them
    gives the eager bits on every replay, with eager work and synchronisations between the replays."""
    import torch
    cfg = gen.scaled(gen.config(3), 4)
    mats = []
    for sid in (0, 4, 6):
        W, x = gen.make_case(cfg, sid)
        A = E.ecspmv_build_dense(W, E.make_opts(max_granularity=4))
        E.device.upload(A)
        xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
        X4 = torch.stack([xd, -xd, xd * 0.5, xd * 2.0], dim=1).contiguous()
        mats.append(dict(A=A, x=xd, X=X4, y=torch.empty(W.shape[0], dtype=torch.float16, device="cuda"),
                         yb=torch.empty(W.shape[0], dtype=torch.float16, device="cuda"),
                         Y=torch.empty((W.shape[0], 4), dtype=torch.float16, device="cuda")))

    def work(sh):
        for e in mats:
            e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
            e["A"].ecspmv_run_multi(e["X"].data_ptr(), e["Y"].data_ptr(), 4, sh)
        E.ecspmv_run_batch([e["A"] for e in mats], [e["x"].data_ptr() for e in mats],
                           [e["yb"].data_ptr() for e in mats], sh)

    work(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = [(e["y"].clone(), e["yb"].clone(), e["Y"].clone()) for e in mats]
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        work(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        for e in mats:
            e["y"].fill_(float("nan")), e["yb"].fill_(float("nan")), e["Y"].fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for e, (y, yb, Y) in zip(mats, want):
            assert torch.equal(e["y"].view(torch.int16), y.view(torch.int16)), rep
            assert torch.equal(e["yb"].view(torch.int16), yb.view(torch.int16)), rep
            assert torch.equal(e["Y"].view(torch.int16), Y.view(torch.int16)), rep
        work(torch.cuda.current_stream().cuda_stream)          # eager work between replays
        torch.cuda.synchronize()


def test_few_long_dense_rows(E):
    """64 dense rows of 60000 columns: the automatic panel count goes up so that the partial sums fit LDS."""
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((64, 60000)) * 0.02).astype(np.float16)
    x = gen.make_vector(60000, seed=6)
    A, _ = check(E, W, x, E.make_opts(max_granularity=1), label="64 x 60000 dense")
    assert A.ecspmv_stats().num_panels > 4
    check(E, W, x, E.make_opts(max_granularity=1, delta_bits=4), label="64 x 60000 dense 4-bit")


@pytest.mark.parametrize("bits", [8, 4, 16])
def test_rows_clustered_before_the_panels_are_cut(E, bits):
    """ECSPMV_FLAG_CLUSTER_ROWS: a panel owns rows from all over the matrix and y is stored through the panel's row
    index table.  Every row of y must still be written, to its own place: oracle band on a config, a planted block on
    scattered rows, and x = e_j returning column j bit for bit."""
    import torch
    flags = E.binding.FLAG_CLUSTER_ROWS | E.binding.FLAG_KEEP_SMALL_SETS
    W, x = gen.make_case(gen.scaled(gen.config(1), 4), 0)
    A, _ = check(E, W, x, E.make_opts(delta_bits=bits, flags=flags), label=f"clustered cfg1/div4 bits{bits}")
    rng = np.random.default_rng(8)
    m, n = 512, 2048
    W = ((rng.random((m, n)) < 0.1) * rng.standard_normal((m, n)) * 0.02).astype(np.float16)
    rows, cols = rng.choice(m, 16, replace=False), np.sort(rng.choice(n, 256, replace=False))
    W[np.ix_(rows, cols)] = (0.05 + 0.02 * rng.standard_normal((16, 256))).astype(np.float16)
    x = rng.standard_normal(n).astype(np.float16)
    A, _ = check(E, W, x, E.make_opts(delta_bits=bits, flags=flags), label=f"clustered planted bits{bits}")
    if bits != 4:
        assert A.ecspmv_stats().nnz_by_g[3] > 0                      # the planted block came out 8-grained
    for j in (int(cols[0]), int(cols[100]), 7, n - 1):
        e = np.zeros(n, dtype=np.float16)
        e[j] = 1.0
        xd = torch.from_numpy(e.view(np.int16)).cuda().view(torch.float16)
        yd = torch.full((m,), float("nan"), dtype=torch.float16, device="cuda")
        E.device.run(A, xd, yd)
        torch.cuda.synchronize()
        want = W[:, j].view(np.uint16).copy()
        want[(want & 0x7FFF) == 0] = 0
        assert np.array_equal(yd.cpu().numpy().view(np.uint16), want), f"column {j}"
