#!/usr/bin/env python3
"""Benchmark of the whole scheduling path on one MI355X.

A step is one pass of the hot path over one batch of synthetic timing samples of a workload:
dependency-bitset propagation (``tictac_build_deps``), TIC priorities (``tictac_tic_priority``), and
TAC orders for all B samples together with the simulation of every sample under its TAC order
(``tictac_tac_simulate``, the fused form of ``tictac_tac_priority`` + ``tictac_simulate``; the two
separate calls are timed as well).  The timing arrays are resident in device memory before the timed
region starts.

The headline (``value``, timed over exactly ``--steps`` steps after ``--warmup``) is the Inception-v3-shaped
preset at its full batch, the largest preset on which the CPU oracle can run whole samples; the line
also carries one record per preset, all five at their full batch (``per_config``), the roofline record
of the dominant kernel, the dependency-propagation bandwidth on the stress preset, side legs on the
headline samples (random, TIC and TAC orders compared, several channels, the time-oracle estimator,
the order search, float32 storage) and the CPU oracle timed on a bounded sample of the headline
workload, on one host core and on all of them.
"""

from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

PRESETS = ["tiny", "resnet50", "vgg16", "inception3", "stress"]
HEADLINE = "inception3"

# peaks of MI355X used for the roofline records
HBM_PEAK_GBS = 8000.0
FP64_VECTOR_PEAK_TFLOPS = 78.6      # 256 compute units x 4 SIMD x 16 lanes x 2 (fused multiply-add) x 2.4 GHz


def parse() -> argparse.Namespace:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=HEADLINE, choices=PRESETS, help="the preset that the headline is timed on")
    ap.add_argument("--batch", type=int, default=0, help="override B of the headline preset (0 = the preset's)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="CPU work per leg of the oracle baseline, in seconds of one core (0 = skip)")
    ap.add_argument("--no-per-config", action="store_true", help="skip the records of the other presets")
    ap.add_argument("--no-deps-bench", action="store_true", help="skip the propagation timing on the stress preset")
    ap.add_argument("--no-compare", action="store_true", help="skip the side legs on the headline samples")
    ap.add_argument("--deps-batch", type=int, default=32,
                    help="independent instances of the stress graph propagated by one launch (a run beyond the "
                         "configuration: one graph alone is bound by the latency of its level chain); 0 = skip")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain elementwise kernel that reads 1 GiB and writes 1 GiB, the known-size "
                         "reference that hardware byte counters of a profiler run are scaled by")
    return ap.parse_args()


def tac_algorithmic_ops(nnz_ops: int, R: int, N: int) -> float:
    """Operations per timing sample that the method itself needs in its incremental form: one add per
    compute op (class totals), for every (op, recv) incidence one integer decrement and one float64
    subtract when that recv is removed, and four float64 operations (two min, two compares) per
    comparator step of the R(R+1)/2 steps of the selection scans."""
    return float(N + 2 * nnz_ops + 4 * (R * (R + 1) // 2))


def traffic_from_profiles(workload: str, B: int):
    """HBM bytes per launch of the fused TAC + simulation kernel from the counter runs summarised in
    profiles/tac_fused_hbm_counters.md (FETCH_SIZE + WRITE_SIZE, scaled by the copy probe).  None when
    the file has no row for this workload and batch, or when the kernel sources have changed since."""
    path = os.path.join(ROOT, "profiles", "tac_fused_hbm_counters.md")
    if not os.path.exists(path):
        return None
    text = open(path).read()
    m = re.search(r"kernel sources sha256/16:\s*([0-9a-f]{16})", text)
    if not m or m.group(1) != kernel_sources_hash():
        return None
    for line in text.splitlines():
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[0] == workload and cells[1].replace(" ", "") == str(B):
            try:
                return float(cells[2]) + float(cells[3])
            except ValueError:
                return None
    return None


def kernel_sources_hash() -> str:
    h = hashlib.sha256()
    for f in ("k3_tac_reg.hip", "k3_tac_sliced.hip", "k3_tac.hip", "device_utils.h"):
        h.update(open(os.path.join(ROOT, "paper_1803_03288_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


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
    ev = lambda: torch.cuda.Event(enable_timing=True)
    log = lambda msg: print(f"[bench] {msg}", file=sys.stderr, flush=True)

    def timed(fn, reps: int, skip: int = 1) -> float:
        """mean milliseconds of fn() between HIP events on the current stream, the first `skip` calls left out"""
        ms = []
        for i in range(reps + skip):
            a, b = ev(), ev()
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            if i >= skip:
                ms.append(a.elapsed_time(b))
        return float(np.mean(ms))

    popcount8 = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device="cuda")

    def dep_nnz(h, d) -> int:
        """sum of |dep| over the compute ops, from the handle's bitsets"""
        deps = h.deps()
        if deps.numel() == 0:
            return 0
        comp = torch.from_numpy(d.compute_ids().astype(np.int64)).cuda()
        total = 0
        for r0 in range(0, comp.numel(), 16384):
            total += int(popcount8[deps[comp[r0:r0 + 16384]].contiguous().view(torch.uint8).long()].sum())
        return total

    def measure(name: str, B: int, steps: int, warmup: int):
        """K timed steps of the whole path on one preset, and the kernel-level figures of its TAC launch."""
        d = wl.preset(name)
        t0 = time.time()
        op, rv = wl.timing_samples(d, 0, B)
        gop, grv = torch.from_numpy(op).cuda(), torch.from_numpy(rv).cuda()
        torch.cuda.synchronize()
        log(f"{d.name}: N={d.n_compute} R={d.n_recv} E={d.n_edges} B={B}; inputs generated and uploaded in {time.time() - t0:.1f}s")
        events = []

        def step(record: bool):
            h = tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)
            tt.tic_priority(h)
            e0, e1 = ev(), ev()
            e0.record()
            res = tt.tac_simulate(h, gop, grv, want_rank=True)     # order, rank, ..., makespan, E, U, L, S
            e1.record()
            if record:
                events.append((e0, e1))
            return h, res

        for _ in range(warmup):
            h, res = step(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            h, res = step(True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        tac_ms = float(np.median([a.elapsed_time(b) for a, b in events]))
        build_ms = timed(lambda: tt.build_deps(d.n_ops, d.row_ptr, d.col_idx, d.recv_ids), 3)
        tic_ms = timed(lambda: tt.tic_priority(h), 3)
        k1_ms = timed(h.recompute_deps, 5, skip=2)
        nnz = dep_nnz(h, d)
        ops = tac_algorithmic_ops(nnz, d.n_recv, d.n_compute) * B
        hbm_bytes = (8.0 * (d.n_compute + d.n_recv) + 8.0 * d.n_recv + 40.0) * B       # rows in; order, rank and five doubles out
        rec = {
            "workload": f"{d.name} preset (seed {d.seed}): N={d.n_compute} compute ops, R={d.n_recv} recvs, B={B} timing samples",
            "schedules_per_s": B / (dt / steps), "ms_per_step": dt / steps * 1e3, "steps": steps,
            "tac_simulate_ms": tac_ms, "tac_simulate_schedules_per_s": B / (tac_ms * 1e-3),
            "build_deps_ms": build_ms, "tic_priority_ms": tic_ms, "dep_propagation_us": k1_ms * 1e3,
            "classes": h.n_classes, "levels": h.n_levels, "dep_incidences": nnz,
            "alu": {"algorithmic_Tops_per_s": ops / (tac_ms * 1e-3) / 1e12,
                    "frac_of_fp64_vector_peak": ops / (tac_ms * 1e-3) / 1e12 / FP64_VECTOR_PEAK_TFLOPS},
            "hbm": {"compulsory_GBs": hbm_bytes / (tac_ms * 1e-3) / 1e9,
                    "frac_of_hbm_peak": hbm_bytes / (tac_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "mean_scheduling_efficiency": float(res[5].mean()), "mean_makespan_s": float(res[4].mean()),
        }
        first_sample[name] = (d, op[0].copy(), rv[0].copy(), res[0][0].cpu().numpy())
        return d, h, op, rv, gop, grv, res, rec

    # ---- every preset at its full batch (the headline one last, with the driver's step counts) ----
    per_config = {}
    first_sample = {}           # per preset: the graph, sample 0 and its TAC order from the GPU (for the CPU leg)
    if not args.no_per_config:
        for name in PRESETS:
            if name == args.workload:
                continue
            dd = wl.preset(name)
            k = 3 if name in ("stress",) else 5
            out = measure(name, dd.batch, k, 2)
            per_config[name] = out[-1]
            log(f"{name}: {out[-1]['schedules_per_s']:.4g} schedules/s, fused call {out[-1]['tac_simulate_ms']:.3f} ms")
            del out
            torch.cuda.empty_cache()

    d0 = wl.preset(args.workload)
    B = args.batch or d0.batch
    d, h, op, rv, gop, grv, res, head = measure(args.workload, B, args.steps, args.warmup)
    per_config[args.workload] = head
    out = res[4:]
    value, ms_per_step = head["schedules_per_s"], head["ms_per_step"]
    tac_s = head["tac_simulate_ms"] * 1e-3

    # ---- roofline record of the dominant kernel (the fused TAC + simulation launch), from the HIP events ----
    achieved = head["alu"]["algorithmic_Tops_per_s"]
    K = (max(h.n_classes, 1) + 63) // 64
    kernel_name = "tac_reg_kernel" if (d.n_recv <= 384 and K <= 8) else "tac_sliced_kernel"
    roofline = {"kernel": f"{kernel_name} (TAC + simulation fused)", "bound": "alu", "achieved": achieved,
                "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / FP64_VECTOR_PEAK_TFLOPS,
                "traffic": traffic_from_profiles(args.workload, B), "ms_per_launch": tac_s * 1e3,
                "hbm_GBs": head["hbm"]["compulsory_GBs"], "hbm_frac": head["hbm"]["frac_of_hbm_peak"],
                "note": "algorithmic operations N + 2 nnz + 4 R(R+1)/2 per sample (mostly integer and compare work) over the "
                        "fp64 vector peak; the kernel is bound by instruction issue of a dependent chain of R rounds per sample"}

    # ---- the two calls made separately, for reference (same outputs as the fused call) ----
    sep_tac_ms = timed(lambda: tt.tac_priority(h, gop, grv, want_rank=True), 3)
    order_tac = tt.tac_priority(h, gop, grv, want_rank=True)[0]
    sim_ms = timed(lambda: tt.simulate(h, order_tac, gop, grv), 3)
    sim_s = sim_ms * 1e-3
    simulate = {"separate_tac_ms": sep_tac_ms, "ms_per_launch": sim_ms,
                "hbm_GBs": (8.0 * (d.n_compute + d.n_recv) + 4.0 * d.n_recv + 16.0) * B / sim_s / 1e9}
    simulate["frac_of_hbm_peak"] = simulate["hbm_GBs"] / HBM_PEAK_GBS

    small = 0 < d.n_recv <= 512 and h.n_classes <= 512
    # ---- no scheduling (a random order per sample) against TIC and TAC on the same samples ----
    comparison = None
    if not args.no_compare and d.n_recv > 0:
        t0 = time.time()
        rnd = torch.from_numpy(wl.random_orders(d, 0, B)).cuda()
        tic_order = tt.tic_priority(h)[1]
        legs = {"random": tt.simulate(h, rnd, gop, grv), "tic": tt.simulate(h, tic_order, gop, grv), "tac": out}
        comparison = {}
        q3 = torch.tensor([0.05, 0.5, 0.95], dtype=torch.float64, device="cuda")
        for name_, r_ in legs.items():
            m_, e_ = r_[0], r_[1]
            rec = {"mean_makespan_s": float(m_.mean()), "mean_efficiency": float(e_.mean()), "min_efficiency": float(e_.min()),
                   "makespan_s_p05_p50_p95": [float(x) for x in torch.quantile(m_, q3)],
                   "efficiency_p05_p50_p95": [float(x) for x in torch.quantile(e_, q3)]}
            for w_ in (2, 4, 8, 16):
                s_ = tt.straggler_effect(m_, w_)
                rec[f"straggler_w{w_}"] = {"mean": float(s_.mean()), "max": float(s_.max())}
            comparison[name_] = rec
        comparison["tac_better_than_tic_samples"] = int((legs["tac"][0] < legs["tic"][0]).sum())
        comparison["tic_better_than_tac_samples"] = int((legs["tic"][0] < legs["tac"][0]).sum())
        del rnd, legs
        torch.cuda.synchronize()
        log(f"order comparison in {time.time() - t0:.1f}s")

    # ---- the same samples with the recvs dealt round-robin over four channels (TAC orders) ----
    channels = None
    if not args.no_compare and small:
        chan4 = (np.arange(d.n_recv) % 4).astype(np.int32)
        c_ms = timed(lambda: tt.simulate_channels(h, 4, chan4, order_tac, gop, grv), 3)
        rc_ = tt.simulate_channels(h, 4, chan4, order_tac, gop, grv)
        c_bytes = (8.0 * (d.n_compute + d.n_recv) + 4.0 * d.n_recv + 16.0) * B
        channels = {"n_channels": 4, "ms_per_launch": c_ms, "hbm_GBs": c_bytes / (c_ms * 1e-3) / 1e9,
                    "frac_of_hbm_peak": c_bytes / (c_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                    "mean_makespan_s": float(rc_[0].mean()), "mean_efficiency": float(rc_[1].mean())}

    # ---- send ops: the same graph with a send behind R compute ops drawn at random, on an uplink ----
    sends_leg = None
    if not args.no_compare and small:
        rng_s = np.random.default_rng(d.seed + 99)
        k_s = d.n_recv
        behind = np.sort(rng_s.choice(d.compute_ids(), size=k_s, replace=False)).astype(np.int32)
        row2 = np.concatenate([d.row_ptr, d.row_ptr[-1] + 1 + np.arange(k_s, dtype=np.int32)]).astype(np.int32)
        col2 = np.concatenate([d.col_idx, behind]).astype(np.int32)
        send_ids = np.arange(d.n_ops, d.n_ops + k_s, dtype=np.int32)
        h2 = tt.build_deps(d.n_ops + k_s, row2, col2, d.recv_ids)
        Bs = min(B, 16384)
        # a send moves what a recv moves (the gradient of a parameter has the parameter's size)
        send_t = grv[:Bs].index_select(1, torch.from_numpy(rng_s.permutation(d.n_recv)).cuda())
        op2 = torch.cat([gop[:Bs], send_t], dim=1).contiguous()
        rv2 = grv[:Bs].contiguous()
        ord2 = order_tac[:Bs].contiguous()
        q_ms = timed(lambda: tt.simulate_sends(h2, send_ids, ord2, op2, rv2), 2)
        rs_ = tt.simulate_sends(h2, send_ids, ord2, op2, rv2)
        sends_leg = {"n_send": int(k_s), "samples": int(Bs), "ms_per_launch": q_ms, "samples_per_s": Bs / (q_ms * 1e-3),
                     "ns_per_op_and_sample": q_ms * 1e6 / Bs / (d.n_compute + k_s),
                     "mean_makespan_s": float(rs_[0].mean()), "mean_efficiency": float(rs_[1].mean()),
                     "mean_makespan_without_sends_s": float(out[0][:Bs].mean()),
                     "note": "compute device followed op by op (lowest ready op id first), TAC orders"}
        h2.close()
        del op2, rv2, ord2, send_t

    # ---- order search: every sample climbs from its random order through proposed exchanges ----
    search = None
    if not args.no_compare and small:
        n_moves = 1024 if d.n_recv <= 200 else 256
        mv = torch.from_numpy(np.random.default_rng(d.seed + 77).integers(0, d.n_recv, size=(n_moves, 2)).astype(np.int32)).cuda()
        rnd = torch.from_numpy(wl.random_orders(d, 0, B)).cuda()
        s_ms = timed(lambda: tt.order_search(h, rnd, mv, gop, grv), 2)
        sr_ = tt.order_search(h, rnd, mv, gop, grv)
        from_tac = tt.order_search(h, order_tac, mv, gop, grv)
        search = {"n_moves": n_moves, "start": "random order per sample", "ms_per_launch": s_ms,
                  "sample_moves_per_s": n_moves * B / (s_ms * 1e-3),
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
        r32 = tt.tac_simulate(h, gop32, grv32)
        f32 = {"tac_simulate_ms": timed(lambda: tt.tac_simulate(h, gop32, grv32), 3),
               "simulate_ms": timed(lambda: tt.simulate(h, r32[0], gop32, grv32), 3),
               "hbm_bytes_per_sample": 4.0 * (d.n_compute + d.n_recv),
               "max_rel_makespan_difference_from_float64_input": float(((r32[4] - out[0]).abs() / out[0]).max()),
               "orders_equal_to_float64_input": float((r32[0] == order_tac).all(dim=1).double().mean())}
        del gop32, grv32, r32

    # ---- time oracle estimator: minimum over five measured runs of the first 2^26 values of op_time ----
    time_oracle = None
    if not args.no_compare:
        K_ = 5
        one = gop.reshape(-1)[: 1 << 26]
        runs_ = one.unsqueeze(0).repeat(K_, 1)
        t_ms = timed(lambda: tt.time_oracle_min(runs_), 4)
        t_bytes = (K_ + 1) * 8.0 * one.numel()
        time_oracle = {"runs": K_, "values": one.numel(), "ms_per_launch": t_ms, "hbm_GBs": t_bytes / (t_ms * 1e-3) / 1e9,
                       "frac_of_hbm_peak": t_bytes / (t_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del runs_, one

    # ---- a plain device copy on the same box, the practical ceiling next to the published peak ----
    cx = torch.zeros(1 << 26, dtype=torch.float64, device="cuda")      # 512 MiB read + 512 MiB written
    cy = torch.empty_like(cx)
    copy_ms = timed(lambda: torch.add(cx, 1.0, out=cy), 4, skip=2)
    copy_GBs = 2.0 * cx.numel() * 8 / (copy_ms * 1e-3) / 1e9
    # (the propagation only writes: the rate of a plain fill on the same box stands beside it)
    fill_ms = timed(lambda: cy.fill_(1.0), 4, skip=2)
    fill_GBs = cy.numel() * 8 / (fill_ms * 1e-3) / 1e9
    del cx, cy
    simulate["frac_of_device_copy"] = simulate["hbm_GBs"] / copy_GBs

    # ---- dependency-bitset propagation bandwidth on the stress preset ----
    dep_bitset = None
    if not args.no_deps_bench:
        ds = wl.preset("stress")
        hs = tt.build_deps(ds.n_ops, ds.row_ptr, ds.col_idx, ds.recv_ids)
        k1_ms = timed(hs.recompute_deps, 8, skip=2)
        alg_bytes = ds.n_ops * ds.words * 8 + 4 * (ds.n_ops + 1 + ds.n_edges)
        gbs = alg_bytes / (k1_ms * 1e-3) / 1e9
        dep_bitset = {"workload": "stress", "n_ops": ds.n_ops, "words": ds.words, "levels": hs.n_levels,
                      "us_per_launch": k1_ms * 1e3, "GB/s": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS,
                      "target_frac_of_hbm_peak": 0.5, "target_met": bool(gbs / HBM_PEAK_GBS >= 0.5),
                      "us_per_level": k1_ms * 1e3 / max(hs.n_levels, 1),
                      "note": "one graph is a chain of dependent levels: its time is levels x per-level latency, not bytes",
                      "frac_of_device_copy": gbs / copy_GBs, "device_copy_GB/s": copy_GBs,
                      "device_fill_GB/s": fill_GBs}
        if args.deps_batch > 1 and hasattr(tt, "recompute_deps_batch"):
            # beyond the configuration: G instances of the graph, propagated by one launch
            for G in sorted({max(2, args.deps_batch // 2), args.deps_batch, args.deps_batch * 2}):
                hb = [hs] + [tt.build_deps(ds.n_ops, ds.row_ptr, ds.col_idx, ds.recv_ids) for _ in range(G - 1)]
                b_ms = timed(lambda: tt.recompute_deps_batch(hb), 5, skip=2)
                dep_bitset.setdefault("batched", []).append(
                    {"instances": G, "us_per_launch": b_ms * 1e3, "GB/s": G * alg_bytes / (b_ms * 1e-3) / 1e9,
                     "frac_of_hbm_peak": G * alg_bytes / (b_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "target_met": bool(G * alg_bytes / (b_ms * 1e-3) / 1e9 / HBM_PEAK_GBS >= 0.5),
                     "frac_of_device_fill": G * alg_bytes / (b_ms * 1e-3) / 1e9 / fill_GBs,
                     "note": "G independent graphs in one launch, HIP events; beyond the configuration"})
                for hh in hb[1:]:
                    hh.close()
        hs.close()

    if args.copy_probe:
        x = torch.zeros(1 << 27, dtype=torch.float64, device="cuda")
        y = torch.empty_like(x)
        torch.add(x, 1.0, out=y)
        torch.cuda.synchronize()
        del x, y

    # ---- the oracle on the host cores, bounded samples of the headline workload ----
    cpu = None
    if args.cpu_seconds > 0:
        import oracle   # the CPU-baseline leg is the only user of the oracle here
        args_ = (d.n_ops, d.row_ptr, d.col_idx, d.recv_ids)

        def oracle_path(rows):
            dep_ = oracle.find_dependencies(*args_)
            oracle.tic(dep_, d.recv_ids)
            eo_ = oracle.tac(dep_, d.recv_ids, op[rows], rv[rows])[0]
            oracle.simulate(*args_, eo_, op[rows], rv[rows])
            return eo_

        t0 = time.perf_counter()
        oracle_path(slice(0, 1))
        per_sample = max(time.perf_counter() - t0, 1e-4)
        k1 = int(max(1, min(B, args.cpu_seconds / per_sample)))
        t0 = time.perf_counter()
        eo = oracle_path(slice(0, k1))
        dt1 = time.perf_counter() - t0
        cores = len(os.sched_getaffinity(0))
        per_thread = max(1, k1 // 2)
        kall = min(B, cores * per_thread)
        bounds = np.linspace(0, kall, cores + 1).astype(int)
        t0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(lambda i: oracle_path(slice(int(bounds[i]), int(bounds[i + 1]))), range(cores)))
        dta = time.perf_counter() - t0
        cpu = {"value": kall / dta, "unit": "schedules/s", "cores": cores, "kind": "oracle",
               "sample": f"first {kall} of {B} samples of {d.name}, dealt to {cores} host threads (each: deps + TIC + TAC + simulate), {dta:.1f}s",
               "one_core": {"value": k1 / dt1, "unit": "schedules/s", "cores": 1,
                            "sample": f"first {k1} of {B} samples of {d.name}: deps + TIC + TAC + simulate, {dt1:.1f}s"}}
        order_gpu = tt.tac_priority(h, gop[:k1].contiguous(), grv[:k1].contiguous())[0].cpu().numpy()
        cpu["orders_match_gpu"] = bool(np.array_equal(order_gpu, eo))

        # What the rounds of Algorithm 3 look like on each preset, from the oracle's Algorithm 1 on sample 0 (along
        # the order the GPU produced): how many outstanding recvs have P > 0 when the minimum is taken.  With one
        # such recv the selection is forced, with none it is the minimum of M+, otherwise the comparator decides.
        def round_kinds(name_):
            dd, op0, rv0, order0 = first_sample[name_]
            R_ = dd.n_recv
            if R_ == 0:
                return None
            dep_ = oracle.find_dependencies(dd.n_ops, dd.row_ptr, dd.col_idx, dd.recv_ids)
            tfull = np.zeros(dd.n_ops)
            tfull[dd.compute_ids()] = op0
            tfull[dd.recv_ids] = rv0
            ks = list(range(R_)) if R_ <= 400 else sorted(set(np.linspace(0, R_ - 1, 24).astype(int).tolist()))

            def one(k):
                alive = np.ones(R_, dtype=np.uint8)
                alive[order0[:k]] = 0
                P_ = oracle.update_properties(dep_, dd.recv_ids, tfull, alive)[1]
                return int(((P_ > 0) & (alive > 0)).sum())

            with ThreadPoolExecutor(cores) as ex:
                q = np.array(list(ex.map(one, ks)))
            return {"rounds_looked_at": len(ks), "of_rounds": R_, "recvs_with_P_mean": float(q.mean()),
                    "share_forced": float((q == 1).mean()), "share_two": float((q == 2).mean()),
                    "share_three_or_more": float((q >= 3).mean()), "share_none": float((q == 0).mean())}

        for name_ in per_config:
            t0 = time.time()
            per_config[name_]["round_kinds_from_oracle"] = round_kinds(name_)
            log(f"round kinds of {name_} in {time.time() - t0:.1f}s")

    line = {
        "metric": "timing-sample schedules/sec (TAC+simulate) on 1 MI355X; dep-bitset HBM GB/s",
        "value": value, "unit": "schedules/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": head["workload"] + "; step = build_deps + TIC + fused TAC/simulate"},
        "roofline": roofline, "cpu_baseline": cpu, "per_config": per_config,
        "simulate": simulate, "dep_bitset": dep_bitset, "order_comparison": comparison, "simulate_channels": channels, "simulate_sends": sends_leg,
        "time_oracle_min": time_oracle, "order_search": search, "float32_storage": f32,
        "mean_scheduling_efficiency": head["mean_scheduling_efficiency"],
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
