#!/usr/bin/env python3
"""Where the time of a lone SpMV launch goes: clock stamps taken inside the kernel.

Loads libecspmv_trace.so (the library's own sources compiled with -DECS_TRACE, built by build.build_all()), launches
cold SpMVs of one shape back to back on one stream, and prints, for every stamp the kernel takes, when the
wavefronts of a launch pass it (microseconds after the launch's first wavefront started: earliest, median, latest
wavefront), averaged over the traced launches, plus the gap from a launch's last stamp to the next launch's first.

    python -m paper_2507_12205_amd.timeline --config 3 --shape 0 --delta-bits 4 [--json out.json]

The stamped kernel is a few per cent slower than the product kernel (the stamps wait for outstanding loads where the
product kernel would not); the event-timed figure of the same launches is printed beside it.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

STAMPS = [
    (0, "wavefront started"),
    (22, "before the header request"),
    (23, "header requested"),
    (20, "header and first pieces requested"),
    (1, "panel header here"),
    (2, "first chunks requested"),
    (21, "first piece of tables / x here"),
    (3, "tables and x pieces written to LDS"),
    (4, "first barrier passed"),
    (5, "chunk 0 data here"),
    (6, "chunk 0 done"),
    (7, "chunk 1 data here"),
    (8, "chunk 1 done"),
    (9, "chunk 2 data here"),
    (10, "chunk 2 done"),
    (11, "all chunks done"),
    (12, "second barrier passed"),
]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--shape", type=int, default=0, help="index into the config's shapes")
    ap.add_argument("--delta-bits", type=int, default=4)
    ap.add_argument("--max-granularity", type=int, default=0)
    ap.add_argument("--copies", type=int, default=0, help="distinct matrices (0 = enough for > 300 MB of images)")
    ap.add_argument("--launches", type=int, default=32, help="traced launches (after one untraced rotation)")
    ap.add_argument("--json", type=str, default="")
    ap.add_argument("--raw", type=str, default="", help="write the raw stamps of every point as .npz")
    args = ap.parse_args()

    from paper_2507_12205_amd import build as B
    if not os.path.exists(B.TRACE_LIB):
        raise SystemExit(f"{B.TRACE_LIB} is missing: run build.build_all()")
    os.environ["ECSPMV_LIB"] = os.environ.get("ECSPMV_TRACE_LIB", B.TRACE_LIB)      # (or a differently built one)
    import torch
    import paper_2507_12205_amd as E
    from paper_2507_12205_amd import device as D
    from workloads import generators as gen

    L = E.binding.lib()
    L.ecspmv_trace_buffer.argtypes = [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32]
    L.ecspmv_trace_buffer.restype = ctypes.c_int

    cfg = gen.config(args.config)
    name, m, n = cfg.shapes[args.shape]
    est = 2.5 * cfg.density * m * n
    copies = args.copies or max(2, int(np.ceil((300 << 20) / est)))
    opts = E.make_opts(delta_bits=args.delta_bits, max_granularity=args.max_granularity)
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    sh = int(stream.cuda_stream)
    mats = []
    for c in range(copies):
        W = gen.make_matrix(cfg, args.shape, seed=0, copy=c)
        A = E.ecspmv_build_dense(W, opts)
        D.upload(A, stream=stream)
        x = gen.make_vector(n, seed=0, cid=cfg.cid, shape_id=args.shape, copy=c)
        mats.append((A, torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)))
    st = mats[0][0].ecspmv_stats()
    P = int(st.num_panels)
    R = args.launches
    y = torch.empty(m, dtype=torch.float16, device="cuda")
    words = torch.zeros(R * P * 128, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()

    def run(i):
        A, x = mats[i % copies]
        A.ecspmv_run(x.data_ptr(), y.data_ptr(), sh)

    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def traced(sel):
        """R launches back to back, each stamping point `sel`; returns (stamps[R, P, 16, 8], us per launch)."""
        for i in range(copies):                # untraced rotation: code and clocks warm, images cold again after it
            run(i)
        torch.cuda.synchronize()
        words.zero_()
        torch.cuda.synchronize()
        assert L.ecspmv_trace_buffer(words.data_ptr(), R, P, sel) == 0
        ev0.record(stream)
        for r in range(R):
            run(r)
        ev1.record(stream)
        torch.cuda.synchronize()
        assert L.ecspmv_trace_buffer(None, 0, 0, 0) == 0
        return words.cpu().numpy().reshape(R, P, 16, 8).copy(), ev0.elapsed_time(ev1) * 1e3 / R

    # the same library with the stamps switched off, for comparison
    for i in range(copies):
        run(i)
    torch.cuda.synchronize()
    ev0.record(stream)
    for r in range(4 * R):
        run(r)
    ev1.record(stream)
    torch.cuda.synchronize()
    us_plain = ev0.elapsed_time(ev1) * 1e3 / (4 * R)

    rows, raw, us_traced = [], {}, []
    mhz = None
    for k, label in STAMPS:
        if k == 0:
            continue
        T, us = traced(k)
        us_traced.append(us)
        raw[k] = T
        valid = T[..., 0] > 0
        if mhz is None:
            d_real = (T[..., 4] - T[..., 3])[valid].astype(np.float64)
            d_clk = (T[..., 2] - T[..., 0])[valid].astype(np.float64)
            mhz = float(d_clk.sum() / d_real.sum() * 100.0)
        # The stamp counter is not the same on every part of the chip; the constant-rate counter is.  Every wavefront's
        # stamps are therefore placed on the constant-rate axis through its own pair (start stamp, constant-rate start);
        # differences are taken in integers first.
        real0 = np.where(valid, T[..., 3], np.iinfo(np.int64).max).min(axis=(1, 2))              # per launch
        start = (T[..., 3] - real0[:, None, None]).astype(np.float64) * 0.01                     # us
        at = start + (T[..., 1] - T[..., 0]).astype(np.float64) / mhz
        end = start + (T[..., 2] - T[..., 0]).astype(np.float64) / mhz
        ok = valid & (T[..., 1] > 0)
        use = [r for r in range(1, R) if ok[r].any()]
        if not use:
            continue
        if not rows:
            rows.append(dict(stamp=0, label=STAMPS[0][1],
                             first_us=0.0, median_us=round(float(np.mean([np.median(start[r][valid[r]]) for r in use])), 3),
                             last_us=round(float(np.mean([start[r][valid[r]].max() for r in use])), 3),
                             last_wave_of_wg_median_us=round(float(np.mean([np.median(start[r].max(axis=1)) for r in use])), 3)))
        # the slowest wavefront of a workgroup is the one a barrier waits for
        wg_last = [np.median(np.where(ok[r], at[r], -np.inf).max(axis=1)) for r in use]
        rows.append(dict(stamp=k, label=label, first_us=round(float(np.mean([at[r][ok[r]].min() for r in use])), 3),
                         median_us=round(float(np.mean([np.median(at[r][ok[r]]) for r in use])), 3),
                         last_us=round(float(np.mean([at[r][ok[r]].max() for r in use])), 3),
                         last_wave_of_wg_median_us=round(float(np.mean(wg_last)), 3),
                         wavefronts=int(ok[use].sum() // len(use))))
        span = float(np.mean([np.where(valid[r], end[r], -np.inf).max() for r in use]))
        # from the last instruction of a launch to the first of the next, on the constant-rate clock
        last_real = np.where(valid, T[..., 4], 0).max(axis=(1, 2))
        gap = float(np.mean((real0[1:] - last_real[:-1])[1:]) * 0.01)
    if args.raw:
        np.savez_compressed(args.raw, **{f"stamp{k}": v for k, v in raw.items()})
    out = dict(workload=f"config {cfg.cid} {name} {m}x{n}, EC-CSR-{args.delta_bits}, {copies} cold copies, "
                        f"{R} launches back to back per stamped point", stamp_clock_mhz=round(mhz, 1),
               us_per_launch_stamps_off=round(us_plain, 3),
               us_per_launch_one_stamp=round(float(np.median(us_traced)), 3),
               kernel_span_us=round(span, 3), gap_to_next_launch_us=round(gap, 3), stamps=rows)
    print(f"# {out['workload']}")
    print(f"# stamp clock {mhz:.1f} MHz; {us_plain:.3f} us per launch with the stamps off, "
          f"{out['us_per_launch_one_stamp']:.3f} us with one stamp per wavefront (event-timed); first instruction to "
          f"last {span:.3f} us; last instruction to the next launch's first {gap:.3f} us")
    print(f"{'point in the kernel':40s} {'first':>8s} {'median':>8s} {'last':>8s} {'WG-last':>8s}   "
          "(us after the launch's first wavefront started; WG-last = slowest wavefront of the median workgroup)")
    for r in rows:
        print(f"{r['label']:40s} {r['first_us']:8.3f} {r['median_us']:8.3f} {r['last_us']:8.3f} "
              f"{r['last_wave_of_wg_median_us']:8.3f}")
    if args.json:
        os.makedirs(os.path.dirname(os.path.abspath(args.json)), exist_ok=True)
        with open(args.json, "w") as f:
            json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
