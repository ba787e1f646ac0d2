#!/usr/bin/env python3
"""Bench of the EC-SpMV hot path on one MI355X.

Workload (default): the LLaMA-13B-shaped decoder layer at 70 % sparsity -- seven back-to-back SpMVs
(q/k/v/o 5120x5120, gate/up 13824x5120, down 5120x13824) on one stream.  A "step" is one such layer.  The steps
rotate through several independently seeded layers whose EC-CSR images total more than 1 GB, so that no matrix is
served from the 256 MB Infinity Cache (cold-cache timing).  Inputs are synthetic (workloads/generators.py) and are
resident in HBM before the timed region starts.

`--launch` says how the SpMVs of a step are submitted in the timed region: `single` (default) = one launch each,
as the workload is stated; `groups` / `all` = the batched entry point (one launch per group of projections that are
independent in a decoder layer / one launch for all seven).  All three are always measured and reported in
`by_launch_mode`; `value` and `roofline` are those of the mode given by `--launch`.

Beside the headline figures the default run adds, as further keys of the same line: the spread of the step times
(`per_step_us`), one matrix hot in cache, the plain-read ceiling, the plain CSR kernel, the other delta width, several
right-hand sides, FP32 values, and the other workload configs (`other_configs`, each in a child process).

`ablation` (default run): the shape of the paper's Section 8.3 study on the same matrices and the same kernel: 16-bit
absolute columns (index compression off), 8-bit and 4-bit delta indices, each without block extraction and with blocks of
up to 2 / up to 8 rows: bytes per stored entry, entries per granularity, microseconds per step for `single` and `groups`.
`parity_checked`: for every leg that is timed, the y (of copy 0) that the timed launches left behind, checked against the
FP64 oracle's band after the timed regions (part of the cpu_baseline leg, which computes the oracle's y anyway).

Prints ONE JSON line: whole-job effective HBM GB/s (bytes that must be read or written per SpMV: EC-CSR values,
deltas and tables + x + y, divided by time), microseconds per SpMV, the roofline of the SpMV kernel and the CPU
oracle's rate on the host cores as a baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload config id (workloads/generators.py)")
    ap.add_argument("--copies", type=int, default=0, help="seeded copies in the rotation set (0 = enough for the config's cold-cache size)")
    ap.add_argument("--max-granularity", type=int, default=0)
    ap.add_argument("--delta-bits", type=int, default=4, choices=[4, 8, 16],
                    help="width of the delta indices: 4 = EC-CSR-4 (default: the smaller and faster format at the "
                         "sparsities of the configs), 8 = EC-CSR-8; the other one is timed in the extras")
    ap.add_argument("--panels", type=int, default=0)
    ap.add_argument("--threads-per-wg", type=int, default=0)
    ap.add_argument("--launch", choices=["single", "groups", "all"], default="single",
                    help="how the SpMVs of a step are submitted in the timed region: one launch each (single), "
                         "one launch per group of projections that are independent in a decoder layer (groups: "
                         "q+k+v, o, gate+up, down), or one launch for the whole step (all)")
    ap.add_argument("--profile-run", action="store_true",
                    help="only the warm-up and the timed region of the chosen launch mode (for rocprofv3, so that "
                         "the kernel statistics cover exactly the launches the bench times)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip hot-cache, CSR and streaming-read legs")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the runs of the other workload configs")
    ap.add_argument("--detail", type=str, default="", help="write per-shape details to this JSON file")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy three times (known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def algorithmic_bytes(st) -> int:
    """Bytes one SpMV must move: EC-CSR values + deltas + tables, x once, y once."""
    return int(st.value_bytes + st.delta_bytes + st.meta_bytes + 2 * st.n + 2 * st.m)


def kernel_source_sha() -> str:
    """SHA-256 (first 16 hex digits) over the sources the SpMV kernel is built from: a stored counter reading is only
    valid for the kernel it was taken with."""
    import hashlib
    h = hashlib.sha256()
    for f in ("kernels.hip", "ecspmv_format.h", "launch.h", "encoder.cpp"):
        with open(os.path.join(ROOT, "paper_2507_12205_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def main():
    args = parse_args()
    if args.profile_run:
        args.no_extras = args.no_cpu_baseline = True
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU; --gpus {args.gpus} is not supported "
              "(every run uses one GPU; across GPUs the path would shard by row panels), exiting", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    import paper_2507_12205_amd as E
    from paper_2507_12205_amd import device as D
    from workloads import generators as gen
    E.binding.lib()

    cfg = gen.config(args.config)
    nshapes = len(cfg.shapes)
    opts = E.make_opts(max_granularity=args.max_granularity, num_panels=args.panels,
                       threads_per_wg=args.threads_per_wg, delta_bits=args.delta_bits)
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    sh = int(stream.cuda_stream)

    # ---- build the rotation set -------------------------------------------------------------------------
    t_prep = time.time()
    est_layer_bytes = sum(2.5 * cfg.density * m * n for _, m, n in cfg.shapes)     # a lower bound: the set is never short
    copies = args.copies or max(2, int(np.ceil(max(cfg.rotation_bytes, 1) * 1.05 / est_layer_bytes)))
    mats = []      # [copy][shape] -> dict

    def make(job):
        copy, sid = job
        W = gen.make_matrix(cfg, sid, seed=0, copy=copy)
        A = E.ecspmv_build_dense(W, opts)
        return copy, sid, W, A

    jobs = [(c, s) for c in range(copies) for s in range(nshapes)]
    keep_dense = {}
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(make, jobs))
    build_seconds = 0.0
    for copy, sid, W, A in results:
        while len(mats) <= copy:
            mats.append([None] * nshapes)
        st = A.ecspmv_stats()
        build_seconds += st.build_seconds
        D.upload(A, stream=stream)
        m, n = W.shape
        x = gen.make_vector(n, seed=0, cid=cfg.cid, shape_id=sid, copy=copy)
        mats[copy][sid] = dict(A=A, st=st, x=torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16),
                               y=torch.full((m,), float("nan"), dtype=torch.float16, device="cuda"),
                               bytes=algorithmic_bytes(st),
                               name=cfg.shapes[sid][0], m=m, n=n)
        if copy == 0:
            keep_dense[sid] = (W, x)
    del results
    torch.cuda.synchronize()
    t_prep = time.time() - t_prep
    image_total = sum(e["st"].image_bytes for layer in mats for e in layer)
    layer_bytes = [sum(e["bytes"] for e in layer) for layer in mats]

    # what the timed launches leave in y is kept (copy 0, on the host) and checked against the oracle at the end
    parity_cases = []

    def keep_for_parity(label, layer, dense, fp32=False):
        torch.cuda.synchronize()
        for sid, e in enumerate(layer):
            W, x = dense[sid]
            parity_cases.append(dict(label=label, name=cfg.shapes[sid][0], W=W, x=x, y=e["y"].cpu().numpy(), fp32=fp32))

    def group_of(names):
        # projections of a decoder layer that do not depend on one another share a launch
        groups, cur, key = [], [], None
        fam = {"q": "qkv", "k": "qkv", "v": "qkv", "gate": "gu", "up": "gu"}
        for i, nm in enumerate(names):
            kf = fam.get(nm, f"solo{i}")
            if cur and kf != key:
                groups.append(cur)
                cur = []
            cur.append(i)
            key = kf
        if cur:
            groups.append(cur)
        return groups

    def batches_for(layer, mode):
        names = [e["name"] for e in layer]
        if mode == "all":
            groups = [list(range(len(layer)))]
        else:
            groups = group_of(names)
        return [E.Batch([layer[i]["A"] for i in g], [layer[i]["x"].data_ptr() for i in g],
                        [layer[i]["y"].data_ptr() for i in g]) for g in groups]

    batched = {mode: [batches_for(layer, mode) for layer in mats] for mode in ("groups", "all")}

    def run_layer(layer, mode=None):
        mode = mode or args.launch
        if mode == "single":
            for e in layer:
                e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
        else:
            for b in batched[mode][mats.index(layer)]:
                b.ecspmv_run_batch(sh)

    # ---- timed region: K steps, cold cache (rotation) ---------------------------------------------------
    # part of the set-up, not of the W warm-up steps: about 20 ms of the same work, so that the clocks have left
    # their idle state before anything is timed (the warm-up steps alone are half a millisecond)
    if not args.profile_run:
        for w in range(300):
            run_layer(mats[w % copies])
        torch.cuda.synchronize()
    for w in range(args.warmup):
        run_layer(mats[w % copies])
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for s in range(args.steps):
        run_layer(mats[(args.warmup + s) % copies])
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = ev0.elapsed_time(ev1)
    total_ms = max(gpu_ms, 0.0) if gpu_ms > 0 else wall * 1e3
    keep_for_parity(f"EC-CSR-{args.delta_bits} {args.launch}", mats[0], keep_dense)
    nlaunch = args.steps * nshapes
    moved = sum(layer_bytes[(args.warmup + s) % copies] for s in range(args.steps))
    value = moved / (total_ms * 1e-3) / 1e9
    us_per_spmv = total_ms * 1e3 / nlaunch

    # ---- per-shape cold timings: one event-bracketed region per shape class, rotating over every matrix of that
    # shape in the set (only classes whose images together exceed the 256 MB Infinity Cache count as cold)
    classes = {}
    for layer in mats:
        for e in layer:
            classes.setdefault((e["m"], e["n"]), []).append(e)
    per_shape = {}
    for (m, n), lst in ([] if args.profile_run else classes.items()):
        lst = list(lst)
        # a class whose images in the rotation set do not reach 512 MB gets further seeded copies, for this timing only
        sid0 = next(i for i, (_, m_, n_) in enumerate(cfg.shapes) if (m_, n_) == (m, n))
        extra = copies
        while sum(int(e["st"].image_bytes) for e in lst) <= (512 << 20) and extra < copies + 64:
            W = gen.make_matrix(cfg, sid0, seed=0, copy=extra)
            A = E.ecspmv_build_dense(W, opts)
            D.upload(A, stream=stream)
            st = A.ecspmv_stats()
            xv = gen.make_vector(n, seed=0, cid=cfg.cid, shape_id=sid0, copy=extra)
            lst.append(dict(A=A, st=st, x=torch.from_numpy(xv.view(np.int16)).cuda().view(torch.float16),
                            y=torch.empty(m, dtype=torch.float16, device="cuda"), bytes=algorithmic_bytes(st)))
            extra += 1
        tot_img = sum(int(e["st"].image_bytes) for e in lst)
        reps = max(2, (args.steps * nshapes) // (4 * len(lst)))
        for e in lst:
            e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            for e in lst:
                e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
        b.record(stream)
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / (reps * len(lst))
        byt = sum(e["bytes"] for e in lst) / len(lst)
        per_shape[f"{m}x{n}"] = dict(us=round(us, 3), gbps=round(byt / us / 1e3, 1), bytes=int(byt),
                                     cold=bool(tot_img > (512 << 20)), matrices=len(lst),
                                     rotation_mib=round(tot_img / 2**20))
        del lst
    # kernel launches of the timed region in the chosen launch mode
    launches_per_step = {"single": nshapes, "groups": len(batched["groups"][0]), "all": 1}[args.launch]
    n_ev = args.steps * launches_per_step
    avg_launch_us = total_ms * 1e3 / n_ev
    achieved = value
    byte_sum = moved

    # HBM traffic per launch as counted by rocprofv3 (FETCH_SIZE + WRITE_SIZE runs, see profiles/): measured in
    # separate profiler runs of this same command, so it is read from the committed summary, not sampled here
    traffic, traffic_stale = None, None
    tpath = os.path.join(ROOT, "profiles", "ecspmv_kernel_config3_hbm_traffic.json")
    default_build = not (args.max_granularity or args.panels or args.threads_per_wg or args.delta_bits != 4)
    if args.config == 3 and default_build and os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        # the counters were read from a particular build of the kernel: the figure is passed on only for that build
        traffic_stale = tj.get("kernel_source_sha16") != kernel_source_sha()
        if not traffic_stale:
            traffic = {"single": tj.get("traffic_bytes_per_launch"),
                       "groups": tj.get("traffic_bytes_per_launch_groups"),
                       "all": tj.get("traffic_bytes_per_step_launch_all")}.get(args.launch)

    out = {
        "metric": "effective HBM GB/s of cold-cache EC-CSR SpMV (EC-CSR bytes + x + y per SpMV / time)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(total_ms / args.steps, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 values, f32 accumulate", "data": "synthetic",
        "config": {"workload": f"config {cfg.cid} ({cfg.name}): {nshapes} SpMVs per step, "
                               + ", ".join(f"{nm} {m}x{n}" for nm, m, n in cfg.shapes)
                               + f"; density {cfg.density}; rotation of {copies} seeded copies, "
                               f"{image_total / 2**20:.0f} MiB of EC-CSR images (cold cache)",
                   "spmv_per_step": nshapes, "rotation_copies": copies,
                   "format": f"EC-CSR-{mats[0][0]['st'].delta_bits}"},
        "us_per_spmv": round(us_per_spmv, 3),
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_stale": traffic_stale,
                     "kernel": "ecspmv_kernel", "avg_launch_us": round(avg_launch_us, 3),
                     "bytes_per_launch": round(byte_sum / n_ev),
                     "timing": "HIP events on the launch stream around the whole timed region / launches (gaps included)"},
    }

    # ---- storage: EC-CSR bytes against CSR bytes ----------------------------------------------------------
    nnz = sum(e["st"].nnz for e in mats[0])
    img = sum(e["st"].image_bytes for e in mats[0])
    need = sum(e["bytes"] for e in mats[0])
    c32 = sum(e["st"].csr32_bytes for e in mats[0])
    c16 = sum(e["st"].csr16_bytes for e in mats[0])
    by_g = [int(sum(e["st"].nnz_by_g[k] for e in mats[0])) for k in range(5)]
    out["storage"] = {"nnz_per_step": int(nnz), "eccsr_image_bytes": int(img), "eccsr_needed_bytes": int(need),
                      "csr32_bytes": int(c32), "csr16_bytes": int(c16), "eccsr_over_csr32": round(img / c32, 4),
                      "bytes_per_nnz": round(img / nnz, 4), "nnz_by_granularity_1_2_4_8_16": by_g,
                      "pad_elements": int(sum(e["st"].pad_elements for e in mats[0])),
                      "build_seconds_total": round(build_seconds, 2), "prep_seconds": round(t_prep, 1)}

    detail = per_shape
    out["per_shape_cold"] = per_shape

    # the same steps submitted with fewer launches (cold rotation, same events)
    # the paper's own figures, with the hardware they were measured on: context, not a target (other machine, other
    # matrices: SparseGPT-pruned LLaMA2 / OPT weights)
    out["paper_context"] = {
        "hardware": "NVIDIA RTX 3080 Ti / 3090 / 4090",
        "speedup_over_best_fp16_baseline": {"max": 6.44, "geomean": 2.43, "baseline": "DASP", "where": "abstract, Section 8.1"},
        "speedup_over_best_fp32_baseline": {"max": 4.36, "geomean": 1.38, "baseline": "AlphaSparse", "where": "Section 8.1"},
        "storage_reduction_vs_csr32_pct_at_70_80_90_sparsity": {
            "fp16_ec_csr_8": [52.0, 49.9, 45.8], "fp16_ec_csr_4": [55.4, 53.5, 41.3],
            "fp32_ec_csr_8": [38.9, 37.3, 33.7], "fp32_ec_csr_4": [40.9, 38.2, 22.7], "where": "Section 8.2"},
        "here_storage_reduction_vs_csr32_pct": round(100.0 * (1.0 - img / c32), 1),
        "ablation_gain_pct": {"index_compression": 15.4, "block_extraction": 15.7, "load_balancing_up_to": 10.12,
                              "where": "Section 8.3, RTX 3080 Ti, FP32"},
    }
    out["launch_mode"] = args.launch
    out["launches_per_step"] = launches_per_step
    alt = {}
    for mode in (() if args.profile_run else ("single", "groups", "all")):
        for e in mats[0]:
            e["y"].fill_(float("nan"))
        for w in range(min(args.warmup, copies)):
            run_layer(mats[w % copies], mode)
        torch.cuda.synchronize()
        ev0.record(stream)
        for s_ in range(args.steps):
            run_layer(mats[(args.warmup + s_) % copies], mode)
        ev1.record(stream)
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1)
        keep_for_parity(f"EC-CSR-{args.delta_bits} {mode}", mats[0], keep_dense)
        nl = {"single": nshapes, "groups": len(batched["groups"][0]), "all": 1}[mode]
        alt[mode] = {"launches_per_step": nl, "us_per_step": round(ms * 1e3 / args.steps, 3),
                     "us_per_spmv": round(ms * 1e3 / (args.steps * nshapes), 3),
                     "gbps": round(moved / (ms * 1e-3) / 1e9, 1),
                     "pct_of_hbm_peak": round(100.0 * moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)}
    out["by_launch_mode"] = alt
    # roofline of the same kernel when one launch carries the whole step (bytes per launch / launch time)
    step_bytes = moved / args.steps
    out["roofline_by_launch_mode"] = {
        mode: {"bytes_per_launch": round(step_bytes / a["launches_per_step"]),
               "avg_launch_us": round(a["us_per_step"] / a["launches_per_step"], 3),
               "achieved": a["gbps"], "frac": round(a["gbps"] / HBM_PEAK_GBPS, 4)} for mode, a in alt.items()}

    if not args.no_extras:
        # spread over the rotation: every step of the chosen launch mode bracketed by its own pair of events (the
        # events add to each step, so these sit above the aggregate figure)
        nst = min(args.steps, 100)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(nst + 1)]
        for s in range(copies):
            run_layer(mats[s % copies])
        torch.cuda.synchronize()
        evs[0].record(stream)
        for s in range(nst):
            run_layer(mats[s % copies])
            evs[s + 1].record(stream)
        torch.cuda.synchronize()
        per = sorted(evs[s].elapsed_time(evs[s + 1]) * 1e3 for s in range(nst))
        out["per_step_us"] = {"launch_mode": args.launch, "steps": nst, "min": round(per[0], 3),
                              "median": round(per[nst // 2], 3), "max": round(per[-1], 3)}

        # clocks while the GPU is busy with the same work, as rocm-smi reports them (context; skipped if unreadable)
        try:
            import subprocess
            smi = subprocess.Popen(["rocm-smi", "--showclocks", "--json"], stdout=subprocess.PIPE,
                                   stderr=subprocess.DEVNULL, text=True)
            t_stop = time.time() + 10.0
            while smi.poll() is None and time.time() < t_stop:
                for s in range(50):
                    run_layer(mats[s % copies])
                torch.cuda.synchronize()
            if smi.poll() is None:
                smi.kill()
            txt = smi.communicate(timeout=5)[0]
            js = [ln for ln in txt.splitlines() if ln.startswith("{")]
            if js:
                card = next(iter(json.loads(js[-1]).values()))
                out["gpu_clocks_under_load"] = {k.strip(" :"): v.strip("()") for k, v in card.items() if "speed" in k}
        except Exception:
            pass

        # hot cache: one matrix over and over (its image fits the 256 MB Infinity Cache), first matrix of every shape
        reps = max(10, args.steps // 2)
        hot, seen = {}, set()
        for e in mats[0]:
            if (e["m"], e["n"]) in seen:
                continue
            seen.add((e["m"], e["n"]))
            for _ in range(5):
                e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
            torch.cuda.synchronize()
            ev0.record(stream)
            for _ in range(reps):
                e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
            ev1.record(stream)
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1)
            hot[f'{e["name"]} {e["m"]}x{e["n"]}'] = {"us_per_spmv": round(ms * 1e3 / reps, 3),
                                                      "gbps": round(e["bytes"] * reps / (ms * 1e-3) / 1e9, 1)}
        first = next(iter(hot))
        out["hot_cache"] = {"matrix": first, **hot[first], "per_shape": hot}

        # streaming-read ceiling over the very same images, same rotation
        chk = torch.zeros(1024, dtype=torch.int32, device="cuda")
        for nwg in (256, 512, 1024):
            for layer in mats[:2]:
                for e in layer:
                    E.ecspmv_stream_read(e["A"].d_image.data_ptr(), int(e["st"].image_bytes), chk.data_ptr(), nwg, sh)
            torch.cuda.synchronize()
            ev0.record(stream)
            tot = 0
            for s in range(min(args.steps, 4 * copies)):
                for e in mats[s % copies]:
                    E.ecspmv_stream_read(e["A"].d_image.data_ptr(), int(e["st"].image_bytes), chk.data_ptr(), nwg, sh)
                    tot += int(e["st"].image_bytes)
            ev1.record(stream)
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1)
            out.setdefault("stream_read_ceiling_gbps", {})[f"{nwg}wg"] = round(tot / (ms * 1e-3) / 1e9, 1)
        # ... and in one launch per step: buffers of one step's bytes each, rotated the same way
        step_bytes = sum(int(e["st"].image_bytes) for e in mats[0]) // 16 * 16
        big = [torch.randint(0, 255, (step_bytes,), dtype=torch.uint8, device="cuda") for _ in range(copies)]
        chk4 = torch.zeros(4096, dtype=torch.int32, device="cuda")
        for nwg in (512, 4096):
            for s in range(2 * copies):
                E.ecspmv_stream_read(big[s % copies].data_ptr(), step_bytes, chk4.data_ptr(), nwg, sh)
            torch.cuda.synchronize()
            ev0.record(stream)
            reps = min(args.steps, 8 * copies)
            for s in range(reps):
                E.ecspmv_stream_read(big[s % copies].data_ptr(), step_bytes, chk4.data_ptr(), nwg, sh)
            ev1.record(stream)
            torch.cuda.synchronize()
            out["stream_read_ceiling_gbps"][f"one_launch_per_step_{nwg}wg"] = round(
                step_bytes * reps / (ev0.elapsed_time(ev1) * 1e-3) / 1e9, 1)
        del big

        # the floor under lone launches: a launch that reads nothing, and the fastest plain read found (one contiguous
        # slice per workgroup) of as many bytes as an SpMV of each shape has to move, one launch each, cold (rotation
        # over 640 MB of buffers); the sum over the step's shapes is what seven lone launches cannot go below
        nul = torch.zeros(4096, dtype=torch.int32, device="cuda")
        floor = {}
        for nwg, thr in ((256, 1024), (512, 512)):
            E.ecspmv_empty_launch(nul.data_ptr(), nwg, thr, 50, sh)
            torch.cuda.synchronize()
            ev0.record(stream)
            E.ecspmv_empty_launch(nul.data_ptr(), nwg, thr, 1000, sh)
            ev1.record(stream)
            torch.cuda.synchronize()
            floor[f"empty_launch_{nwg}x{thr}_us"] = round(ev0.elapsed_time(ev1), 3)      # ms per 1000 = us per launch
        pool = torch.randint(0, 255, (640 << 20,), dtype=torch.uint8, device="cuda")
        reads, step_floor = {}, 0.0
        for (m, n), lst in classes.items():
            nbytes = int(sum(e["bytes"] for e in lst) / len(lst)) // 256 * 256
            nbuf = pool.numel() // nbytes
            best = None
            for nwg, thr in ((256, 1024), (512, 512), (1024, 512), (1024, 256), (2048, 256)):
                for r in range(nbuf):
                    E.ecspmv_stream_read_sliced(pool.data_ptr() + r * nbytes, nbytes, nul.data_ptr(), nwg, thr, sh)
                torch.cuda.synchronize()
                ev0.record(stream)
                reps = 3 * nbuf
                for r in range(reps):
                    E.ecspmv_stream_read_sliced(pool.data_ptr() + (r % nbuf) * nbytes, nbytes, nul.data_ptr(), nwg, thr, sh)
                ev1.record(stream)
                torch.cuda.synchronize()
                us = ev0.elapsed_time(ev1) * 1e3 / reps
                if best is None or us < best[0]:
                    best = (us, nwg, thr)
            spmv_us = per_shape.get(f"{m}x{n}", {}).get("us")
            reads[f"{m}x{n}"] = {"bytes": nbytes, "read_us": round(best[0], 3), "workgroups": best[1], "threads": best[2],
                                 "spmv_us": spmv_us, "spmv_over_read": round(spmv_us / best[0], 3) if spmv_us else None}
            step_floor += best[0] * sum(1 for e in mats[0] if (e["m"], e["n"]) == (m, n))
        # the same for the launches of mode `groups` (the bytes of the SpMVs that share a launch, read in one launch)
        gsum, glist = 0.0, []
        for g in group_of([e["name"] for e in mats[0]]):
            nbytes = int(sum(mats[0][i]["bytes"] for i in g)) // 256 * 256
            nbuf = max(2, pool.numel() // nbytes)
            best = None
            for nwg, thr in ((256, 1024), (512, 512), (1024, 512), (1024, 256), (2048, 256)):
                for r in range(nbuf):
                    E.ecspmv_stream_read_sliced(pool.data_ptr() + r * nbytes, nbytes, nul.data_ptr(), nwg, thr, sh)
                torch.cuda.synchronize()
                ev0.record(stream)
                reps = 3 * nbuf
                for r in range(reps):
                    E.ecspmv_stream_read_sliced(pool.data_ptr() + (r % nbuf) * nbytes, nbytes, nul.data_ptr(), nwg, thr, sh)
                ev1.record(stream)
                torch.cuda.synchronize()
                us = ev0.elapsed_time(ev1) * 1e3 / reps
                if best is None or us < best:
                    best = us
            glist.append({"spmvs": "+".join(mats[0][i]["name"] for i in g), "bytes": nbytes, "read_us": round(best, 3)})
            gsum += best
        floor["plain_read_group_launches_cold"] = glist
        floor["step_of_group_launches_us"] = round(gsum, 3)
        floor["step_of_group_launches_pct_of_hbm_peak"] = round(100.0 * layer_bytes[0] / (gsum * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2)
        del pool
        floor["plain_read_lone_launch_cold"] = reads
        floor["step_of_lone_launches_us"] = round(step_floor, 3)
        floor["step_of_lone_launches_pct_of_hbm_peak"] = round(100.0 * layer_bytes[0] / (step_floor * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2)
        out["launch_floor"] = floor

        # plain CSR kernel on the same matrices (first two copies, rotation > 512 MB of CSR data)
        csr_layers = []
        for c in range(min(copies, 2)):
            layer = []
            for sid in range(nshapes):
                W = keep_dense[sid][0] if c == 0 else gen.make_matrix(cfg, sid, seed=0, copy=c)
                C = E.ecspmv_csr_build_dense(W)
                D.csr_upload(C, stream=stream)
                layer.append((C, mats[c][sid]))
            csr_layers.append(layer)
        for layer in csr_layers:
            for C, e in layer:
                C.ecspmv_csr_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
        torch.cuda.synchronize()
        ev0.record(stream)
        reps = max(4, args.steps // 4)
        for s in range(reps):
            for C, e in csr_layers[s % len(csr_layers)]:
                C.ecspmv_csr_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
        ev1.record(stream)
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1)
        csr_bytes = sum(int(e["st"].csr32_bytes) + 2 * e["n"] + 2 * e["m"] for _, e in csr_layers[0])
        out["csr_kernel"] = {"us_per_spmv": round(ms * 1e3 / (reps * nshapes), 3),
                             "gbps_of_csr32_bytes": round(csr_bytes * reps / (ms * 1e-3) / 1e9, 1),
                             "speedup_eccsr_over_csr": round((ms * 1e3 / (reps * nshapes)) / us_per_spmv, 3)}

    if not args.no_extras:
        # the other delta width on the same matrices: a rotation of up to three copies (> 512 MB of images)
        other_bits = 8 if args.delta_bits == 4 else 4
        oopts = E.make_opts(max_granularity=args.max_granularity, num_panels=args.panels,
                            threads_per_wg=args.threads_per_wg, delta_bits=other_bits)
        ncp = min(copies, 3)

        def make_other(job):
            copy, sid = job
            W = keep_dense[sid][0] if copy == 0 else gen.make_matrix(cfg, sid, seed=0, copy=copy)
            return copy, sid, E.ecspmv_build_dense(W, oopts)

        olayers = [[None] * nshapes for _ in range(ncp)]
        with ThreadPoolExecutor(max_workers=4) as ex:
            for copy, sid, A in ex.map(make_other, [(c, s_) for c in range(ncp) for s_ in range(nshapes)]):
                D.upload(A, stream=stream)
                olayers[copy][sid] = dict(A=A, st=A.ecspmv_stats(), x=mats[copy][sid]["x"], y=mats[copy][sid]["y"])
        obatch = [E.Batch([e["A"] for e in layer], [e["x"].data_ptr() for e in layer],
                          [e["y"].data_ptr() for e in layer]) for layer in olayers]
        obytes = [sum(algorithmic_bytes(e["st"]) for e in layer) for layer in olayers]
        res = {}
        for mode in ("single", "all"):
            def go(layer_i):
                if mode == "single":
                    for e in olayers[layer_i]:
                        e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
                else:
                    obatch[layer_i].ecspmv_run_batch(sh)
            for e in olayers[0]:
                e["y"].fill_(float("nan"))
            for w in range(ncp):
                go(w)
            torch.cuda.synchronize()
            ev0.record(stream)
            for s_ in range(args.steps):
                go(s_ % ncp)
            ev1.record(stream)
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1)
            keep_for_parity(f"EC-CSR-{other_bits} {mode}", olayers[0], keep_dense)
            mv = sum(obytes[s_ % ncp] for s_ in range(args.steps))
            res[mode] = {"us_per_step": round(ms * 1e3 / args.steps, 3), "gbps": round(mv / (ms * 1e-3) / 1e9, 1),
                         "pct_of_hbm_peak": round(100.0 * mv / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)}
        onnz = sum(e["st"].nnz for e in olayers[0])
        oimg = sum(e["st"].image_bytes for e in olayers[0])
        out["other_delta_width"] = {"format": f"EC-CSR-{other_bits}", "rotation_copies": ncp,
                                    "bytes_per_nnz": round(oimg / onnz, 4),
                                    "eccsr_over_csr32": round(oimg / sum(e["st"].csr32_bytes for e in olayers[0]), 4),
                                    "nnz_by_granularity_1_2_4_8_16":
                                        [int(sum(e["st"].nnz_by_g[k] for e in olayers[0])) for k in range(5)],
                                    "by_launch_mode": res}
        del olayers, obatch

    if not args.no_extras:
        # a few right-hand sides at once (ecspmv_run_multi): lone launches per shape class, cold rotation over up to
        # three copies; images with 512 panels so that x (2*n*nb bytes) and the partial sums fit LDS more often
        mopts = E.make_opts(max_granularity=min(args.max_granularity or 4, 4), num_panels=512,
                            delta_bits=args.delta_bits)
        ncp = min(copies, 3)

        def make_multi(job):
            copy, sid = job
            W = keep_dense[sid][0] if copy == 0 else gen.make_matrix(cfg, sid, seed=0, copy=copy)
            return copy, sid, E.ecspmv_build_dense(W, mopts)

        mclasses = {}
        with ThreadPoolExecutor(max_workers=4) as ex:
            for copy, sid, A in ex.map(make_multi, [(c, s_) for c in range(ncp) for s_ in range(nshapes)]):
                D.upload(A, stream=stream)
                _, m_, n_ = cfg.shapes[sid]
                mclasses.setdefault((m_, n_), []).append((A, A.ecspmv_stats(), copy, sid))
        multi = {}
        for (m_, n_), lst in mclasses.items():
            row = {}
            for nb in (1, 2, 4, 8):
                Xh = np.stack([gen.make_vector(n_, seed=0, cid=cfg.cid, shape_id=0, copy=100 + b) for b in range(nb)], axis=1)
                X = torch.from_numpy(np.ascontiguousarray(Xh if nb > 1 else Xh[:, 0]).view(np.int16)).cuda().view(torch.float16)
                Y = torch.full((m_, nb) if nb > 1 else (m_,), float("nan"), dtype=torch.float16, device="cuda")
                try:
                    for A, _, _, _ in lst:
                        A.ecspmv_run_multi(X.data_ptr(), Y.data_ptr(), nb, sh)
                except E.EcspmvError as err:
                    if err.status != E.binding.ERR_UNSUPPORTED:
                        raise
                    row[f"nb{nb}"] = None                       # x and the partial sums do not fit LDS
                    continue
                torch.cuda.synchronize()
                reps = max(2, (args.steps * nshapes) // (4 * len(lst)))
                ev0.record(stream)
                for _ in range(reps):
                    for A, _, _, _ in lst:
                        A.ecspmv_run_multi(X.data_ptr(), Y.data_ptr(), nb, sh)
                ev1.record(stream)
                torch.cuda.synchronize()
                us = ev0.elapsed_time(ev1) * 1e3 / (reps * len(lst))
                # Y now holds what the last matrix of the rotation wrote: checked per column at the end
                _, _, lcopy, lsid = lst[-1]
                Wl = keep_dense[lsid][0] if lcopy == 0 else gen.make_matrix(cfg, lsid, seed=0, copy=lcopy)
                Yh = Y.cpu().numpy().reshape(m_, nb)
                for b in range(nb):
                    parity_cases.append(dict(label=f"multi_rhs nb={nb}", name=f"{m_}x{n_} column {b}", W=Wl, x=Xh[:, b].copy(),
                                             y=Yh[:, b].copy(), fp32=False))
                byt = sum(algorithmic_bytes(st) + (nb - 1) * 2 * (n_ + m_) for _, st, _, _ in lst) / len(lst)
                row[f"nb{nb}"] = {"us": round(us, 3), "gbps": round(byt / us / 1e3, 1),
                                  "cold": bool(sum(int(st.image_bytes) for _, st, _, _ in lst) > (300 << 20))}
            base = row.get("nb1")
            for nb in (2, 4, 8):
                if base and row.get(f"nb{nb}"):
                    row[f"nb{nb}"]["speedup_over_nb_single_launches"] = round(nb * base["us"] / row[f"nb{nb}"]["us"], 2)
            multi[f"{m_}x{n_}"] = row
        out["multi_rhs"] = {"format": f"EC-CSR-{mats[0][0]['st'].delta_bits}", "panels": 512, "per_shape": multi}
        del mclasses

    if not args.no_extras:
        # FP32 values (the paper's other precision): the same patterns with FP32 values, x and y; rotation of up to
        # three copies, one launch each and one launch per step
        fopts = E.make_opts(max_granularity=args.max_granularity, num_panels=args.panels,
                            threads_per_wg=args.threads_per_wg, delta_bits=args.delta_bits)
        ncp = min(copies, 3)

        def make_f32(job):
            copy, sid = job
            W = keep_dense[sid][0] if copy == 0 else gen.make_matrix(cfg, sid, seed=0, copy=copy)
            return copy, sid, E.ecspmv_build_dense_f32(W.astype(np.float32), fopts)

        flayers = [[None] * nshapes for _ in range(ncp)]
        with ThreadPoolExecutor(max_workers=3) as ex:
            for copy, sid, A in ex.map(make_f32, [(c, s_) for c in range(ncp) for s_ in range(nshapes)]):
                D.upload(A, stream=stream)
                st = A.ecspmv_stats()
                x32 = gen.make_vector(int(st.n), seed=0, cid=cfg.cid, shape_id=sid, copy=copy).astype(np.float32)
                flayers[copy][sid] = dict(A=A, st=st, x=torch.from_numpy(x32).cuda(),
                                          y=torch.full((int(st.m),), float("nan"), dtype=torch.float32, device="cuda"))
        fbatch = [E.Batch([e["A"] for e in layer], [e["x"].data_ptr() for e in layer],
                          [e["y"].data_ptr() for e in layer]) for layer in flayers]
        fbytes = [sum(int(e["st"].value_bytes + e["st"].delta_bytes + e["st"].meta_bytes + 4 * e["st"].n + 4 * e["st"].m)
                      for e in layer) for layer in flayers]
        res = {}
        for mode in ("single", "all"):
            def go(layer_i):
                if mode == "single":
                    for e in flayers[layer_i]:
                        e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
                else:
                    fbatch[layer_i].ecspmv_run_batch(sh)
            for e in flayers[0]:
                e["y"].fill_(float("nan"))
            for w in range(ncp):
                go(w)
            torch.cuda.synchronize()
            ev0.record(stream)
            for s_ in range(args.steps):
                go(s_ % ncp)
            ev1.record(stream)
            torch.cuda.synchronize()
            ms = ev0.elapsed_time(ev1)
            keep_for_parity(f"FP32 values {mode}", flayers[0],
                            {sid: (keep_dense[sid][0].astype(np.float32), keep_dense[sid][1].astype(np.float32))
                             for sid in range(nshapes)}, fp32=True)
            mv = sum(fbytes[s_ % ncp] for s_ in range(args.steps))
            res[mode] = {"us_per_step": round(ms * 1e3 / args.steps, 3), "gbps": round(mv / (ms * 1e-3) / 1e9, 1),
                         "pct_of_hbm_peak": round(100.0 * mv / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)}
        fnnz = sum(e["st"].nnz for e in flayers[0])
        fimg = sum(e["st"].image_bytes for e in flayers[0])
        out["fp32_values"] = {"format": f"EC-CSR-{flayers[0][0]['st'].delta_bits}, FP32 values, x, y", "rotation_copies": ncp,
                              "bytes_per_nnz": round(fimg / fnnz, 4),
                              "eccsr_over_csr32": round(fimg / sum(e["st"].csr32_bytes for e in flayers[0]), 4),
                              "nnz_by_granularity_1_2_4_8_16":
                                  [int(sum(e["st"].nnz_by_g[k] for e in flayers[0])) for k in range(5)],
                              "by_launch_mode": res}
        del flayers, fbatch

    if not args.no_extras:
        # The shape of the paper's Section 8.3 ablation, measured on this workload with this kernel: index width
        # (16-bit absolute columns = no index compression, 8-bit deltas, 4-bit deltas) x block extraction (none, up to
        # 2 rows, up to 8 rows).  Cold rotation of three copies (> 512 MB of images for every variant).
        ncp = min(copies, 3)
        abl = []
        for bits, mg in ((16, 1), (16, 2), (16, 8), (8, 1), (8, 2), (8, 8), (4, 1), (4, 8)):
            aopts = E.make_opts(max_granularity=mg, delta_bits=bits)

            def make_abl(job):
                copy, sid = job
                W = keep_dense[sid][0] if copy == 0 else gen.make_matrix(cfg, sid, seed=0, copy=copy)
                return copy, sid, E.ecspmv_build_dense(W, aopts)

            alayers = [[None] * nshapes for _ in range(ncp)]
            with ThreadPoolExecutor(max_workers=4) as ex:
                for copy, sid, A in ex.map(make_abl, [(c, s_) for c in range(ncp) for s_ in range(nshapes)]):
                    D.upload(A, stream=stream)
                    alayers[copy][sid] = dict(A=A, st=A.ecspmv_stats(), x=mats[copy][sid]["x"], y=mats[copy][sid]["y"],
                                              name=cfg.shapes[sid][0])
            abatch = [[E.Batch([layer[i]["A"] for i in g], [layer[i]["x"].data_ptr() for i in g],
                               [layer[i]["y"].data_ptr() for i in g]) for g in group_of([e["name"] for e in layer])]
                      for layer in alayers]
            abytes = [sum(algorithmic_bytes(e["st"]) for e in layer) for layer in alayers]
            row = {"index_bits": bits, "max_granularity": mg,
                   "bytes_per_nnz": round(sum(e["st"].image_bytes for e in alayers[0]) / sum(e["st"].nnz for e in alayers[0]), 4),
                   "needed_bytes_per_nnz": round(abytes[0] / sum(e["st"].nnz for e in alayers[0]), 4),
                   "nnz_by_granularity_1_2_4_8_16": [int(sum(e["st"].nnz_by_g[k] for e in alayers[0])) for k in range(5)],
                   "x_access_cost_per_nnz": round(sum(e["st"].x_access_cost for e in alayers[0]) / sum(e["st"].nnz for e in alayers[0]), 4)}
            for mode in ("single", "groups"):
                def go(layer_i):
                    if mode == "single":
                        for e in alayers[layer_i]:
                            e["A"].ecspmv_run(e["x"].data_ptr(), e["y"].data_ptr(), sh)
                    else:
                        for b in abatch[layer_i]:
                            b.ecspmv_run_batch(sh)
                for e in alayers[0]:
                    e["y"].fill_(float("nan"))
                for w in range(ncp):
                    go(w)
                torch.cuda.synchronize()
                ev0.record(stream)
                for s_ in range(args.steps):
                    go(s_ % ncp)
                ev1.record(stream)
                torch.cuda.synchronize()
                ms = ev0.elapsed_time(ev1)
                keep_for_parity(f"ablation index {bits} bits, g <= {mg}, {mode}", alayers[0], keep_dense)
                mv = sum(abytes[s_ % ncp] for s_ in range(args.steps))
                row[f"us_per_step_{mode}"] = round(ms * 1e3 / args.steps, 3)
                row[f"pct_of_hbm_peak_{mode}"] = round(100.0 * mv / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)
            abl.append(row)
            del alayers, abatch
        out["ablation"] = {"workload": f"config {cfg.cid}, cold rotation of {ncp} copies, the same ecspmv_kernel for every row",
                           "rows": abl}

    if not args.no_extras and not args.no_other_configs:
        # the other workload configs under the same protocol (own cold rotation, the same three launch modes), each
        # in a child process that runs this file with --config
        import subprocess
        others = {}
        for cid in [c for c in (1, 2, 3, 4) if c != args.config]:
            cmd = [sys.executable, os.path.abspath(__file__), "--config", str(cid), "--no-extras", "--no-cpu-baseline",
                   "--delta-bits", str(args.delta_bits), "--steps", str(args.steps), "--warmup", str(args.warmup)]
            r = subprocess.run(cmd, capture_output=True, text=True, timeout=900)
            if r.returncode != 0 or not r.stdout.strip():
                others[str(cid)] = {"error": r.stderr[-300:]}
                continue
            d = json.loads(r.stdout.strip().splitlines()[-1])
            others[str(cid)] = {"workload": d["config"]["workload"], "bytes_per_nnz": d["storage"]["bytes_per_nnz"],
                                "eccsr_over_csr32": d["storage"]["eccsr_over_csr32"],
                                "nnz_by_granularity_1_2_4_8_16": d["storage"]["nnz_by_granularity_1_2_4_8_16"],
                                "by_launch_mode": d["by_launch_mode"]}
        out["other_configs"] = others

    if args.calibrate_copy:
        src = torch.randint(0, 127, (256 << 20,), dtype=torch.int8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = int(src.numel())

    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        # the oracle as it stands over one step's matrices, again and again for about ten seconds of wall time (the
        # dense FP16 matrices of a step are 0.4 GB, so every pass streams them from DRAM); the median pass counts
        times, cores, t_all = [], 1, time.perf_counter()
        while len(times) < 3 or (time.perf_counter() - t_all < 10.0 and len(times) < 1000):
            t = time.perf_counter()
            for sid in range(nshapes):
                W, x = keep_dense[sid]
                _, _, cores = orc.spmv_oracle_threads(W, x)
            times.append(time.perf_counter() - t)
        tmed, t_cpu = float(np.median(times)), time.perf_counter() - t_all
        # the y every timed leg left behind (copy 0), against the oracle's band
        refs, checked = {}, {}
        for pc in parity_cases:
            key = (id(pc["W"]), pc["x"].tobytes()[:64], pc["fp32"])
            if key not in refs:
                refs[key] = orc.spmv_oracle_f32(pc["W"], pc["x"]) if pc["fp32"] else orc.spmv_oracle(pc["W"], pc["x"])
            y_ref, S = refs[key]
            ok, ratio = orc.within_band(pc["y"], y_ref, S, 2e-3, 1e-6)
            ok = ok and not np.isnan(pc["y"].astype(np.float64)).any()
            c = checked.setdefault(pc["label"], {"ok": True, "worst_error_over_limit": 0.0, "vectors": 0})
            c["ok"] = bool(c["ok"] and ok)
            c["worst_error_over_limit"] = round(max(c["worst_error_over_limit"], ratio), 4)
            c["vectors"] += 1
            if not ok:
                print(f"bench.py: PARITY FAILED for {pc['label']} / {pc['name']}: worst error / limit = {ratio}", file=sys.stderr)
        out["parity_checked"] = {"band": "|y - y_ref| <= 2e-3 * sum_j |W_ij x_j| + 1e-6, FP64 oracle, every row of every "
                                         "matrix of copy 0 as left by the timed launches",
                                 "all_ok": bool(all(c["ok"] for c in checked.values())), "legs": checked}
        out["cpu_baseline"] = {"value": round(layer_bytes[0] / tmed / 1e9, 3), "unit": "GB/s", "cores": int(cores),
                               "kind": "oracle",
                               "sample": f"one step ({nshapes} dense-masked FP16 matrices of copy 0), FP64 oracle, "
                                         f"median of {len(times)} passes in {t_cpu:.0f} s, {tmed * 1e3:.0f} ms per step; "
                                         "rate = the same EC-CSR+x+y bytes / time",
                               "us_per_spmv": round(tmed * 1e6 / nshapes, 1)}

    if args.detail:
        os.makedirs(os.path.dirname(os.path.abspath(args.detail)), exist_ok=True)
        with open(args.detail, "w") as f:
            json.dump({"summary": out, "per_shape": detail,
                       "stats_copy0": [e["st"].as_dict() for e in mats[0]]}, f, indent=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
