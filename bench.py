#!/usr/bin/env python3
"""Benchmark of the whole scheduling path on one MI355X.

A step is one pass of the hot path over one batch of synthetic timing samples of the
workload: dependency-bitset propagation (``tictac_build_deps``), TIC priorities
(``tictac_tic_priority``), and TAC orders for all B samples together with the simulation of
every sample under its TAC order (``tictac_tac_simulate``, the fused form of
``tictac_tac_priority`` + ``tictac_simulate``; the two separate calls are timed as well).  The timing arrays
are resident in device memory before the timed region starts.

Prints one JSON line: timing-sample schedules per second, the roofline record of the
dominant kernel (TAC), the dependency-propagation bandwidth on the stress preset, the
side legs on the same samples (random, TIC and TAC orders compared, several channels, the
time-oracle estimator, the order search) and the CPU oracle timed on a bounded sample of the
same workload.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np


def parse() -> argparse.Namespace:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="resnet50", choices=["tiny", "resnet50", "vgg16", "inception3", "stress"])
    ap.add_argument("--batch", type=int, default=0, help="override B of the preset (0 = preset's)")
    ap.add_argument("--cpu-samples", type=int, default=1024, help="samples the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-deps-bench", action="store_true", help="skip the propagation timing on the stress preset")
    ap.add_argument("--no-compare", action="store_true",
                    help="skip the comparison of random, TIC and TAC orders (efficiency, straggler effect)")
    ap.add_argument("--deps-batch", type=int, default=8,
                    help="independent instances of the stress graph propagated concurrently on streams of their own "
                         "(a run beyond the configuration: one graph alone is bound by the latency of its level chain); 0 = skip")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain elementwise kernel that reads 1 GiB and writes 1 GiB, the known-size "
                         "reference that hardware byte counters of a profiler run are scaled by")
    return ap.parse_args()


# HBM bytes per launch of the fused TAC + simulation kernel, FETCH_SIZE + WRITE_SIZE of the two
# counter runs summarised in profiles/bench_resnet50_hbm_counters.md (scaled by the copy probe).
# Only valid for the kernel and workload those runs measured; None otherwise.
TAC_TRAFFIC_BYTES = {("resnet50", 65536): 730.35e6 + 94.49e6}

# peaks of MI355X used for the roofline records
HBM_PEAK_GBS = 8000.0
FP64_VECTOR_PEAK_TFLOPS = 78.6


def tac_algorithmic_ops(nnz_ops: int, R: int, N: int) -> float:
    """Operations per timing sample that the method itself needs in its incremental form:
    one add per compute op (class totals), for every (op, recv) incidence one integer
    decrement and one float64 subtract when that recv is removed, and four float64
    operations (two min, two compares) per comparator step of the R(R+1)/2 steps of the
    selection scans."""
    return float(N + 2 * nnz_ops + 4 * (R * (R + 1) // 2))


def main() -> int:
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on one GPU only (timing samples are independent and would shard "
              "by sample with no collective); run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_1803_03288_amd import binding as tt, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    tt.lib()

    d = wl.preset(args.workload)
    B = args.batch or d.batch
    t0 = time.time()
    op, rv = wl.timing_samples(d, 0, B)
    gop, grv = torch.from_numpy(op).cuda(), torch.from_numpy(rv).cuda()
    torch.cuda.synchronize()
    print(f"[bench] workload {d.name}: N={d.n_compute} R={d.n_recv} E={d.n_edges} B={B}; "
          f"inputs generated and uploaded in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    tac_ms, sim_ms, sep_tac_ms = [], [], []

    def step(record: bool):
        h = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
        tt.tic_priority(h)
        e0, e1 = ev(), ev()
        e0.record()
        res = tt.tac_simulate(h, gop, grv, want_rank=True)     # order, rank, ..., makespan, E, U, L, S
        e1.record()
        if record:
            step.events.append((e0, e1))
        return h, res[4:]
    step.events = []

    for _ in range(args.warmup):
        h, out = step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        h, out = step(True)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    for e0, e1 in step.events:
        tac_ms.append(e0.elapsed_time(e1))
    # the two calls made separately, for reference (same outputs as the fused call)
    for i in range(4):
        e0, e1, e2 = ev(), ev(), ev()
        e0.record()
        order = tt.tac_priority(h, gop, grv, want_rank=True)[0]
        e1.record()
        tt.simulate(h, order, gop, grv)
        e2.record()
        torch.cuda.synchronize()
        if i:
            sep_tac_ms.append(e0.elapsed_time(e1))
            sim_ms.append(e1.elapsed_time(e2))
    ms_per_step = dt / args.steps * 1e3
    value = B / (dt / args.steps)
    mean_eff = float(out[1].mean())

    # ---- roofline record of the dominant kernel (TAC), from the HIP events above ----
    dep_gpu = h.deps().cpu().numpy().view(np.uint64)
    nnz_ops = int(np.unpackbits(dep_gpu[d.compute_ids()].view(np.uint8), axis=1).sum())
    tac_s = float(np.mean(tac_ms)) * 1e-3
    ops_per_launch = tac_algorithmic_ops(nnz_ops, d.n_recv, d.n_compute) * B
    achieved = ops_per_launch / tac_s / 1e12
    roofline = {"kernel": "tac_reg_kernel (TAC + simulation fused)", "bound": "alu", "achieved": achieved, "peak": FP64_VECTOR_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / FP64_VECTOR_PEAK_TFLOPS,
                "traffic": TAC_TRAFFIC_BYTES.get((args.workload, B)),
                "ms_per_launch": tac_s * 1e3,
                "hbm_GBs": (8.0 * (d.n_compute + d.n_recv) + 8.0 * d.n_recv) * B / tac_s / 1e9}
    sim_s = float(np.mean(sim_ms)) * 1e-3
    simulate = {"separate_tac_ms": float(np.mean(sep_tac_ms)), "ms_per_launch": sim_s * 1e3,
                "hbm_GBs": (8.0 * (d.n_compute + d.n_recv) + 4.0 * d.n_recv + 16.0) * B / sim_s / 1e9}
    simulate["frac_of_hbm_peak"] = simulate["hbm_GBs"] / HBM_PEAK_GBS

    # ---- no scheduling (a random order per sample) against TIC and TAC on the same samples ----
    comparison = None
    if not args.no_compare and d.n_recv > 0:
        t0 = time.time()
        rnd = torch.from_numpy(wl.random_orders(d, 0, B)).cuda()
        tic_order = tt.tic_priority(h)[1]
        legs = {"random": tt.simulate(h, rnd, gop, grv), "tic": tt.simulate(h, tic_order, gop, grv), "tac": out}
        comparison = {}
        for name_, r_ in legs.items():
            m_, e_ = r_[0], r_[1]
            qm_ = torch.quantile(m_, torch.tensor([0.05, 0.5, 0.95], dtype=torch.float64, device="cuda"))
            qe_ = torch.quantile(e_, torch.tensor([0.05, 0.5, 0.95], dtype=torch.float64, device="cuda"))
            rec = {"mean_makespan_s": float(m_.mean()), "mean_efficiency": float(e_.mean()),
                   "min_efficiency": float(e_.min()),
                   "makespan_s_p05_p50_p95": [float(x) for x in qm_], "efficiency_p05_p50_p95": [float(x) for x in qe_]}
            for w_ in (2, 4, 8, 16):
                s_ = tt.straggler_effect(m_, w_)
                rec[f"straggler_w{w_}"] = {"mean": float(s_.mean()), "max": float(s_.max())}
            comparison[name_] = rec
        torch.cuda.synchronize()
        print(f"[bench] order comparison in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    # ---- the same samples with the recvs dealt round-robin over four channels (TAC orders) ----
    channels = None
    if not args.no_compare and 0 < d.n_recv <= 512 and h.n_classes <= 512:
        chan4 = (np.arange(d.n_recv) % 4).astype(np.int32)
        tac_order = tt.tac_priority(h, gop, grv)[0]
        cms = []
        for i in range(5):
            a, b = ev(), ev()
            a.record()
            rc_ = tt.simulate_channels(h, 4, chan4, tac_order, gop, grv)
            b.record()
            torch.cuda.synchronize()
            if i >= 1:
                cms.append(a.elapsed_time(b))
        c_s = float(np.mean(cms)) * 1e-3
        c_bytes = (8.0 * (d.n_compute + d.n_recv) + 4.0 * d.n_recv + 16.0) * B
        channels = {"n_channels": 4, "ms_per_launch": c_s * 1e3, "hbm_GBs": c_bytes / c_s / 1e9,
                    "frac_of_hbm_peak": c_bytes / c_s / 1e9 / HBM_PEAK_GBS,
                    "mean_makespan_s": float(rc_[0].mean()), "mean_efficiency": float(rc_[1].mean())}

    # ---- order search: every sample climbs from its random order through 1024 proposed exchanges ----
    search = None
    if not args.no_compare and 0 < d.n_recv <= 512 and h.n_classes <= 512:
        n_moves = 1024
        mv = torch.from_numpy(np.random.default_rng(d.seed + 77).integers(0, d.n_recv, size=(n_moves, 2))
                              .astype(np.int32)).cuda()
        rnd = torch.from_numpy(wl.random_orders(d, 0, B)).cuda()
        sms = []
        for i in range(4):
            a, b = ev(), ev()
            a.record()
            sr_ = tt.order_search(h, rnd, mv, gop, grv)
            b.record()
            torch.cuda.synchronize()
            if i >= 1:
                sms.append(a.elapsed_time(b))
        s_s = float(np.mean(sms)) * 1e-3
        from_tac = tt.order_search(h, tt.tac_priority(h, gop, grv)[0], mv, gop, grv)
        search = {"n_moves": n_moves, "start": "random order per sample", "ms_per_launch": s_s * 1e3,
                  "sample_moves_per_s": n_moves * B / s_s,
                  "mean_makespan_start_s": float(sr_[2].mean()), "mean_makespan_end_s": float(sr_[1].mean()),
                  "mean_exchanges_kept": float(sr_[3].double().mean()),
                  "from_tac": {"mean_makespan_start_s": float(from_tac[2].mean()),
                               "mean_makespan_end_s": float(from_tac[1].mean()),
                               "samples_improved": int((from_tac[3] > 0).sum())}}
        del rnd, sr_, from_tac

    # ---- the same samples stored as float32 (converted on load, float64 arithmetic) ----
    f32 = None
    if not args.no_compare and d.n_recv > 0:
        gop32, grv32 = gop.float(), grv.float()
        rec32 = {}
        for leg in ("tac_simulate", "simulate"):
            fms = []
            for i in range(5):
                a, b = ev(), ev()
                a.record()
                if leg == "tac_simulate":
                    r32 = tt.tac_simulate(h, gop32, grv32)
                else:
                    r32s = tt.simulate(h, r32[0], gop32, grv32)
                b.record()
                torch.cuda.synchronize()
                if i >= 1:
                    fms.append(a.elapsed_time(b))
            rec32[leg + "_ms"] = float(np.mean(fms))
        m32, m64 = r32[4], out[0]
        f32 = dict(rec32, hbm_bytes_per_sample=4.0 * (d.n_compute + d.n_recv),
                   max_rel_makespan_difference_from_float64_input=float(((m32 - m64).abs() / m64).max()),
                   orders_equal_to_float64_input=float((r32[0] == tt.tac_priority(h, gop, grv)[0]).all(dim=1).double().mean()))
        del gop32, grv32, r32, r32s

    # ---- time oracle estimator: minimum over five measured runs of the whole op_time array ----
    time_oracle = None
    if not args.no_compare:
        K_ = 5
        runs_ = gop.unsqueeze(0).repeat(K_, 1, 1)          # [5][B][N], device
        tms = []
        for i in range(5):
            a, b = ev(), ev()
            a.record()
            est_ = tt.time_oracle_min(runs_)
            b.record()
            torch.cuda.synchronize()
            if i >= 1:
                tms.append(a.elapsed_time(b))
        t_s = float(np.mean(tms)) * 1e-3
        t_bytes = (K_ + 1) * 8.0 * gop.numel()
        time_oracle = {"runs": K_, "values": gop.numel(), "ms_per_launch": t_s * 1e3, "hbm_GBs": t_bytes / t_s / 1e9,
                       "frac_of_hbm_peak": t_bytes / t_s / 1e9 / HBM_PEAK_GBS}
        del runs_, est_

    # ---- a plain device copy on the same box, the practical ceiling next to the published peak ----
    cx = torch.zeros(1 << 26, dtype=torch.float64, device="cuda")      # 512 MiB read + 512 MiB written
    cy = torch.empty_like(cx)
    copy_ms = []
    for i in range(6):
        a, b = ev(), ev()
        a.record()
        torch.add(cx, 1.0, out=cy)
        b.record()
        torch.cuda.synchronize()
        if i >= 2:
            copy_ms.append(a.elapsed_time(b))
    copy_GBs = 2.0 * cx.numel() * 8 / (float(np.mean(copy_ms)) * 1e-3) / 1e9
    del cx, cy
    simulate["frac_of_device_copy"] = simulate["hbm_GBs"] / copy_GBs

    # ---- dependency-bitset propagation bandwidth on the stress preset ----
    dep_bitset = None
    if not args.no_deps_bench:
        ds = wl.preset("stress")
        hs = tt.build_deps(ds.n_ops, ds.row_ptr, ds.col_idx, ds.recv_ids)
        times = []
        for i in range(7):
            a, b = ev(), ev()
            a.record()
            hs.recompute_deps()
            b.record()
            torch.cuda.synchronize()
            if i >= 2:
                times.append(a.elapsed_time(b))
        k1_s = float(np.mean(times)) * 1e-3
        alg_bytes = ds.n_ops * ds.words * 8 + 4 * (ds.n_ops + 1 + ds.n_edges)
        dep_bitset = {"workload": "stress", "n_ops": ds.n_ops, "words": ds.words, "levels": hs.n_levels,
                      "us_per_launch": k1_s * 1e6, "GB/s": alg_bytes / k1_s / 1e9,
                      "frac_of_hbm_peak": alg_bytes / k1_s / 1e9 / HBM_PEAK_GBS,
                      "frac_of_device_copy": alg_bytes / k1_s / 1e9 / copy_GBs,
                      "device_copy_GB/s": copy_GBs}
        if args.deps_batch > 1:
            # beyond the configuration: G instances of the same graph, each on its own stream
            G = args.deps_batch
            hb = [hs] + [tt.build_deps(ds.n_ops, ds.row_ptr, ds.col_idx, ds.recv_ids) for _ in range(G - 1)]
            streams = [torch.cuda.Stream() for _ in range(G)]
            torch.cuda.synchronize()
            bt = []
            for i in range(5):
                t0 = time.perf_counter()
                for hh, st in zip(hb, streams):
                    with torch.cuda.stream(st):
                        hh.recompute_deps()
                torch.cuda.synchronize()
                if i >= 2:
                    bt.append(time.perf_counter() - t0)
            bs = float(np.mean(bt))
            dep_bitset["batched"] = {"instances": G, "us_total": bs * 1e6, "GB/s": G * alg_bytes / bs / 1e9,
                                     "frac_of_hbm_peak": G * alg_bytes / bs / 1e9 / HBM_PEAK_GBS,
                                     "note": "G independent graphs on G streams, wall clock; beyond the configuration"}
            for hh in hb[1:]:
                hh.close()
        hs.close()

    if args.copy_probe:
        x = torch.zeros(1 << 27, dtype=torch.float64, device="cuda")
        y = torch.empty_like(x)
        torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
        del x, y

    # ---- the oracle on the host cores, bounded sample of the same workload ----
    cpu = None
    if args.cpu_samples > 0:
        import oracle   # the CPU-baseline leg is the only user of the oracle here
        k = min(args.cpu_samples, B)
        t0 = time.perf_counter()
        dep = oracle.find_dependencies(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
        oracle.tic(dep, d.recv_ids)
        eo = oracle.tac(dep, d.recv_ids, op[:k], rv[:k])[0]
        em = oracle.simulate(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids, eo, op[:k], rv[:k])[0]
        cdt = time.perf_counter() - t0
        cpu = {"value": k / cdt, "unit": "schedules/s", "cores": 1, "kind": "oracle",
               "sample": f"first {k} of {B} samples of {d.name}: deps + TIC + TAC + simulate, {cdt:.1f}s"}
        order_gpu = tt.tac_priority(h, gop[:k].contiguous(), grv[:k].contiguous())[0].cpu().numpy()
        cpu["orders_match_gpu"] = bool(np.array_equal(order_gpu, eo))

    line = {
        "metric": "timing-sample schedules/sec (TAC+simulate) on 1 MI355X; dep-bitset HBM GB/s",
        "value": value, "unit": "schedules/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{d.name} preset (seed {d.seed}): N={d.n_compute} compute ops, R={d.n_recv} recvs, "
                               f"B={B} timing samples; step = build_deps + TIC + fused TAC/simulate"},
        "roofline": roofline, "simulate": simulate, "dep_bitset": dep_bitset, "order_comparison": comparison, "simulate_channels": channels, "time_oracle_min": time_oracle, "order_search": search, "float32_storage": f32,
        "cpu_baseline": cpu,
        "mean_scheduling_efficiency": mean_eff,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
