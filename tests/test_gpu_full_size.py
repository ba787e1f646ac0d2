"""GPU parity at the full sizes of the five workload configs, in the launch configurations bench.py times
(256 row panels, workgroup size chosen at launch; EC-CSR-4, the bench's default format, and EC-CSR-8; one launch each
and, for config 3, the whole layer in one launch).  Every row is compared with the FP64 oracle and the EC-CSR image
must decode to exactly W's stored entries."""
import numpy as np
import pytest

from oracle import oracle as orc
from workloads import generators as gen

pytestmark = pytest.mark.gpu

REL, ABS = 2e-3, 1e-6


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("cid", [0, 1, 2, 3, 4])
def test_full_size_config(cid, bits):
    import torch
    import paper_2507_12205_amd as E
    from paper_2507_12205_amd import device as D
    cfg = gen.config(cid)
    for sid, (name, m, n) in enumerate(cfg.shapes):
        if cid == 3 and sid in (1, 2, 3, 5):
            continue                                   # same shape and recipe as q / gate
        print(f"[case] cfg{cid} {name} {m}x{n} EC-CSR-{bits}", flush=True)
        W, x = gen.make_case(cfg, sid)
        A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=bits))
        st = A.ecspmv_stats()
        assert st.num_panels == min(256, m // 16)
        r, c, v = A.ecspmv_decode()
        rr, cc, vv = orc.pattern_triples(W)
        o = np.lexsort((c, r))
        assert np.array_equal(r[o], rr) and np.array_equal(c[o], cc) and np.array_equal(v[o], vv), "round trip"
        D.upload(A)
        xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)
        yd = torch.full((m,), float("nan"), dtype=torch.float16, device="cuda")
        D.run(A, xd, yd)
        torch.cuda.synchronize()
        y = yd.cpu().numpy().astype(np.float64)
        y_ref, S = orc.spmv_oracle(W, x)
        assert not np.isnan(y).any()
        err = np.abs(y - y_ref)
        lim = REL * S + ABS
        assert np.all(err <= lim), f"{name}: worst err/lim {np.max(err / lim):.3f}"
        print(f"        worst err/lim {np.max(err / lim):.4f}  EC-CSR/CSR-32 {st.image_bytes / st.csr32_bytes:.3f}", flush=True)
        del A, xd, yd


def test_full_size_layer_in_one_launch():
    """Config 3 as bench.py --launch all submits it: the seven matrices of a layer, EC-CSR-4, one launch."""
    import torch
    import paper_2507_12205_amd as E
    from paper_2507_12205_amd import device as D
    cfg = gen.config(3)
    mats, xs, ys, refs = [], [], [], []
    for sid, (name, m, n) in enumerate(cfg.shapes):
        print(f"[case] layer {name} {m}x{n}", flush=True)
        W, x = gen.make_case(cfg, sid)
        A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=4))
        D.upload(A)
        mats.append(A)
        xs.append(torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16))
        ys.append(torch.full((m,), float("nan"), dtype=torch.float16, device="cuda"))
        refs.append(orc.spmv_oracle(W, x))
    E.ecspmv_run_batch(mats, [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for (name, m, n), y, (y_ref, S) in zip(cfg.shapes, ys, refs):
        yh = y.cpu().numpy().astype(np.float64)
        assert not np.isnan(yh).any(), name
        err = np.abs(yh - y_ref)
        assert np.all(err <= REL * S + ABS), f"{name}: worst err/lim {np.max(err / (REL * S + ABS)):.3f}"


@pytest.mark.parametrize("bits", [4, 8])
def test_full_size_fp32_values(bits):
    """Config 3 with FP32 values, x and y, as bench.py times it (`fp32_values`): the three shapes one launch each, then
    all seven matrices of the layer in one launch.  Band of the benchmark spec and the tighter 2^-17 * S check that a path
    rounding through FP16 would fail."""
    import torch
    import paper_2507_12205_amd as E
    from paper_2507_12205_amd import device as D
    cfg = gen.config(3)
    mats, xs, ys, refs = [], [], [], []
    for sid, (name, m, n) in enumerate(cfg.shapes):
        print(f"[case] fp32 {name} {m}x{n} EC-CSR-{bits}", flush=True)
        W16, x16 = gen.make_case(cfg, sid)
        W, x = W16.astype(np.float32), x16.astype(np.float32)
        A = E.ecspmv_build_dense_f32(W, E.make_opts(delta_bits=bits))
        D.upload(A)
        xd = torch.from_numpy(x).cuda()
        yd = torch.full((m,), float("nan"), dtype=torch.float32, device="cuda")
        y_ref, S = orc.spmv_oracle_f32(W, x)
        if sid in (0, 4, 6):                                            # one launch each for the three shapes
            D.run(A, xd, yd)
            torch.cuda.synchronize()
            y = yd.cpu().numpy().astype(np.float64)
            assert not np.isnan(y).any()
            err = np.abs(y - y_ref)
            assert np.all(err <= REL * S + ABS) and np.all(err <= 2.0 ** -17 * S + 1e-9), name
            yd.fill_(float("nan"))
        mats.append(A), xs.append(xd), ys.append(yd), refs.append((y_ref, S))
    E.ecspmv_run_batch(mats, [x.data_ptr() for x in xs], [y.data_ptr() for y in ys], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for (name, m, n), y, (y_ref, S) in zip(cfg.shapes, ys, refs):
        yh = y.cpu().numpy().astype(np.float64)
        assert not np.isnan(yh).any(), name
        err = np.abs(yh - y_ref)
        assert np.all(err <= REL * S + ABS) and np.all(err <= 2.0 ** -17 * S + 1e-9), name


@pytest.mark.parametrize("sid", [0, 4, 6])
def test_full_size_several_right_hand_sides(sid):
    """ecspmv_run_multi as bench.py times it (`multi_rhs`: EC-CSR-4 images with 512 panels): nb = 2, 4, 8 on the three
    shapes of config 3 at full size; with nb = 8 the two wide shapes run as two launches of four right-hand sides.  Every
    column of Y against the oracle, and bit-equal to the single-vector launch."""
    import torch
    import paper_2507_12205_amd as E
    from paper_2507_12205_amd import device as D
    cfg = gen.config(3)
    name, m, n = cfg.shapes[sid]
    W = gen.make_matrix(cfg, sid)
    A = E.ecspmv_build_dense(W, E.make_opts(delta_bits=4, num_panels=512, max_granularity=4))
    D.upload(A)
    Xh = np.stack([gen.make_vector(n, seed=0, cid=3, shape_id=sid, copy=40 + b) for b in range(8)], axis=1)
    refs, singles = [], []
    for b in range(8):
        refs.append(orc.spmv_oracle(W, np.ascontiguousarray(Xh[:, b])))
        xd = torch.from_numpy(np.ascontiguousarray(Xh[:, b]).view(np.int16)).cuda().view(torch.float16)
        yd = torch.full((m,), float("nan"), dtype=torch.float16, device="cuda")
        D.run(A, xd, yd)
        torch.cuda.synchronize()
        singles.append(yd.cpu().numpy())
    for nb in (2, 4, 8):
        print(f"[case] multi {name} {m}x{n} nb={nb}", flush=True)
        X = torch.from_numpy(np.ascontiguousarray(Xh[:, :nb]).view(np.int16)).cuda().view(torch.float16)
        Y = torch.full((m, nb), float("nan"), dtype=torch.float16, device="cuda")
        D.run_multi(A, X, Y)
        torch.cuda.synchronize()
        Yh = Y.cpu().numpy()
        for b in range(nb):
            y_ref, S = refs[b]
            col = Yh[:, b].astype(np.float64)
            assert not np.isnan(col).any()
            assert np.all(np.abs(col - y_ref) <= REL * S + ABS), f"nb={nb} column {b}"
            assert np.array_equal(Yh[:, b].view(np.uint16), singles[b].view(np.uint16)), f"nb={nb} column {b}: bits"
