#!/usr/bin/env python3
"""Benchmark of the certified sub-vocabulary LM-head path on one MI355X.

A "step" is one csv_decode_step call (bounds -> select -> gathered GEMV -> certification -> fallback) on one
batch of synthetic hidden states; inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c2]
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

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def step_bytes(r, C, rows_union: float, any_fallback_frac: float, k: int, mu_bytes: int = 4) -> float:
    """Algorithmic bytes of one batch step: centroids + cluster metadata, h, each distinct opened row of W with its
    bias, the whole of W with bias when any sequence falls back, and the outputs."""
    return (C * r.d * mu_bytes + 12 * C + r.B * r.d * 2 + rows_union * (2 * r.d + 4)
            + any_fallback_frac * r.V * (2 * r.d + 4) + r.B * (8 * k + 16))


def brief(name: str, steps: int = 64, warmup: int = 10) -> dict:
    """One of the other workloads, measured the same way but briefly: `steps` timed steps after `warmup`, the
    dense product at the same batch, and how the steps ended (32 steps with a synchronisation each)."""
    import numpy as np
    import torch

    import synth
    import paper_2511_21702_amd as csv

    r = synth.CONFIGS[name]
    head = synth.make_head(r, threads=16)
    h_bits = synth.make_hidden(r, head["centers"], steps=steps + warmup)
    dW = csv.bits_to_device(head["W_bits"])
    db = torch.from_numpy(head["b"]).cuda()
    idx = csv.csv_build_index(dW, db, r.C, init_labels=head["labels"].astype(np.int32))
    del dW
    ws = csv.CsvWorkspace(idx, r.B, r.K_max_rows)
    dh = csv.bits_to_device(h_bits)
    buf = csv.make_step_buffers(idx, r.B, r.k, r.eps, r.K_max_rows)
    sp = torch.cuda.current_stream().cuda_stream
    hp = [dh[s].data_ptr() for s in range(steps + warmup)]
    for s in range(warmup):
        csv.csv_decode_step_raw(ws, idx, hp[s], r.B, buf, sp)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for s in range(warmup, warmup + steps):
        csv.csv_decode_step_raw(ws, idx, hp[s], r.B, buf, sp)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t1
    nstat, n_fb, anyfb, rows, ncert = min(32, steps), 0, 0, 0, 0
    for s in range(warmup, warmup + nstat):
        csv.csv_decode_step_raw(ws, idx, hp[s], r.B, buf, sp)
        torch.cuda.synchronize()
        fl = buf.flags.cpu().numpy()
        fb = (fl & csv.FLAG_FALLBACK) != 0
        n_fb += int(fb.sum()); anyfb += int(fb.any())
        rows += int(buf.n_rows.cpu().numpy()[~fb].sum()); ncert += int((~fb).sum())
    full_out = torch.empty((r.B, r.V), dtype=torch.float32, device="cuda")
    for s in range(2):
        csv.csv_full_logits(ws, idx, dh[s], out=full_out)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for s in range(8):
        csv.csv_full_logits(ws, idx, dh[s], out=full_out)
    torch.cuda.synchronize()
    full_ms = (time.perf_counter() - t1) * 1e3 / 8
    ms = wall * 1e3 / steps
    out = {"workload": f"{r.name}: V={r.V} d={r.d} C={r.C} B={r.B} k={r.k} eps={r.eps:g} K_max={r.K_max_rows}",
           "steps": steps, "ms_per_step": ms, "steps_per_s": 1e3 / ms, "seq_steps_per_s": r.B * 1e3 / ms,
           "fallback_rate": n_fb / (nstat * r.B), "steps_with_fallback": anyfb / nstat,
           "mean_rows_per_certified_seq": rows / max(ncert, 1),
           "full_gemv_ms": full_ms, "speedup_vs_full_gemv": full_ms / ms}
    del buf, full_out, dh
    ws.free(); idx.free()
    torch.cuda.empty_cache()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c2")
    ap.add_argument("--max-rounds", type=int, default=0, help="fallback levels: scoring rounds allowed (0 = the two-round schedule)")
    ap.add_argument("--delta-clusters", type=int, default=0, help="fallback levels: clusters per partial expansion (0 = off)")
    ap.add_argument("--bf16-centroids", action="store_true", help="index option: centroids stored as bfloat16 (half the bound kernel's bytes)")
    ap.add_argument("--bias-table", type=int, default=0, help="index option: top-m bias table (Section III, bias binning), m = 2..8")
    ap.add_argument("--spherical", action="store_true", help="index option: unit directions and the angular bound (Section III, spherical clustering)")
    ap.add_argument("--relax", action="store_true", help="fallback levels: accept the softmax bound at 2 eps before falling back")
    ap.add_argument("--alg1", action="store_true", help="Algorithm 1's own order (one cluster per iteration, the reference mode) instead of the round-based schedule; use with --cpu-steps 0")
    ap.add_argument("--cpu-steps", type=int, default=-1, help="oracle steps to time (-1: sized to ~15 s, 0: skip)")
    ap.add_argument("--kmeans", type=int, default=-1, metavar="ITERS",
                    help="time the offline index build instead: Lloyd's k-means with ITERS iterations from the default seeding "
                         "rule on the config's head (Section IV, offline preprocessing); prints its own JSON line and exits")
    ap.add_argument("--others", type=int, default=-1,
                    help="also measure the other four workloads briefly (field other_configs): 1 yes, 0 no, -1 only in the default run (c2, no options)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE`: launch a device-to-device copy of known size, "
                         "the bound kernel and a few whole steps, then exit (no timing, no JSON)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every figure is one GPU's throughput); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import synth
    import paper_2511_21702_amd as csv

    r = synth.CONFIGS[args.config]
    K, W = args.steps, args.warmup
    t0 = time.time()
    head = synth.make_head(r, threads=16)
    h_bits = synth.make_hidden(r, head["centers"])
    log(f"[bench] {r.name}: V={r.V} d={r.d} C={r.C} B={r.B} generated in {time.time() - t0:.1f}s")
    dW = csv.bits_to_device(head["W_bits"])
    db = torch.from_numpy(head["b"]).cuda()
    if args.kmeans >= 0:
        csv.csv_build_index(dW, db, r.C, iters=0).free()           # warm-up (module load, allocations)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kidx = csv.csv_build_index(dW, db, r.C, iters=args.kmeans)
        torch.cuda.synchronize()
        sec = time.perf_counter() - t1
        e = kidx.export()
        # how well the planted clusters were found: share of tokens whose cluster holds mostly tokens of their planted cluster
        lab = np.empty(r.V, dtype=np.int64)
        off = np.concatenate([[0], np.cumsum(e["n"])])
        for c in range(r.C):
            lab[e["perm"][off[c]:off[c + 1]]] = c
        pairs = np.stack([lab, head["labels"].astype(np.int64)], 1)
        uniq, cnt = np.unique(pairs, axis=0, return_counts=True)
        purity = sum(cnt[uniq[:, 0] == c].max() for c in np.unique(lab)) / r.V
        flops = 2.0 * r.V * r.C * r.d * (args.kmeans + 1)
        print(json.dumps({"metric": "offline k-means index build", "config": {"workload": f"{r.name}: V={r.V} d={r.d} C={r.C}"},
                          "lloyd_iterations": args.kmeans, "assignments": args.kmeans + 1, "seconds": sec,
                          "distance_product_TFLOPs_useful": flops / sec / 1e12,
                          "note": "whole build: every assignment (MFMA distance product, three bf16 pieces per float32 centroid value), "
                                  "host-side layout, row gather, centroid means; then radii and metadata",
                          "empty_clusters": int((e["n"] == 0).sum()), "largest_cluster": int(e["n"].max()), "purity_vs_planted": float(purity)}))
        return 0
    idx = csv.csv_build_index(dW, db, r.C, init_labels=head["labels"].astype(np.int32), centroid_bf16=args.bf16_centroids,
                              bias_table_m=args.bias_table, spherical=args.spherical)
    del dW
    ws = csv.CsvWorkspace(idx, r.B, r.K_max_rows)
    dh = csv.bits_to_device(h_bits)
    nh = h_bits.shape[0]
    lad = dict(max_rounds=args.max_rounds, delta_clusters=args.delta_clusters, relax=args.relax, schedule=1 if args.alg1 else 0)
    buf = csv.make_step_buffers(idx, r.B, r.k, r.eps, r.K_max_rows, **lad)
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    hp = [dh[s % nh].data_ptr() for s in range(max(K, W) + W)]

    def run(n, first=0):
        for s in range(first, first + n):
            csv.csv_decode_step_raw(ws, idx, hp[s], r.B, buf, sp)

    if args.traffic_probe:
        # calibration: a plain copy of 256 MiB reads 256 MiB and writes 256 MiB
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        U_out = torch.empty((r.B, r.C), dtype=torch.float32, device="cuda")
        hn_out = torch.empty(r.B, dtype=torch.float32, device="cuda")
        full_out = torch.empty((r.B, r.V), dtype=torch.float32, device="cuda")
        for s in range(8):
            dst.copy_(src)
        for s in range(32):
            csv.lib.csv_bounds(ws._h, idx._h, hp[s], r.B, U_out.data_ptr(), hn_out.data_ptr(), sp)
        run(32)
        for s in range(4):
            csv.csv_full_logits(ws, idx, dh[s % nh], out=full_out)
        torch.cuda.synchronize()
        log("[bench] traffic probe done: 8 copies of 256 MiB, 32 bound launches, 32 steps, 4 full products")
        return 0

    # ---------------- timed region: W warm-up steps, then exactly K steps, sync on both sides
    run(W)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    run(K, W)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_ms = e0.elapsed_time(e1)
    ms_per_step = wall * 1e3 / K
    log(f"[bench] {K} steps: wall {wall * 1e3:.2f} ms, stream {gpu_ms:.2f} ms -> {K / wall:.0f} steps/s")
    # the same region a few more times (not part of `value`): how much a region of this length varies from run to run
    rep_ms = []
    for _ in range(9):
        t1 = time.perf_counter()
        run(K, W)
        torch.cuda.synchronize()
        rep_ms.append((time.perf_counter() - t1) * 1e3 / K)
    repeats = {"n": len(rep_ms), "median": float(np.median(rep_ms)), "min": float(min(rep_ms)), "max": float(max(rep_ms))}

    # ---------------- per-stage HIP-event timing over the same K steps (second pass, same stream)
    ws.profile_begin(K)
    run(K, W)
    torch.cuda.synchronize()
    stage_ms, nrec = ws.profile_end()
    stage_us = {n: 1e3 * v / max(nrec, 1) for n, v in stage_ms.items()}

    # ---------------- statistics pass: per-step sync, latency percentiles, rows / fallbacks
    fb0 = int(buf.fallback_count.item())
    lat, rows_sum, rows_union_sum, anyfb, ncl_sum, rounds_hist = [], 0, 0.0, 0, 0, {i: 0 for i in range(9)}
    n_relaxed = 0
    buf_s = csv.make_step_buffers(idx, r.B, r.k, r.eps, r.K_max_rows, want_sel=True, **lad)
    sizes = head["sizes"]
    nstat = min(K, 256)
    for s in range(W, W + nstat):
        t1 = time.perf_counter()
        csv.csv_decode_step_raw(ws, idx, hp[s], r.B, buf_s, sp)
        torch.cuda.synchronize()
        lat.append(time.perf_counter() - t1)
        fl = buf_s.flags.cpu().numpy()
        nr = buf_s.n_rows.cpu().numpy()
        nc = buf_s.n_clusters.cpu().numpy()
        fb = (fl & csv.FLAG_FALLBACK) != 0
        n_relaxed += int(((fl & csv.FLAG_SOFTMAX_RELAXED) != 0).sum())
        anyfb += bool(fb.any())
        rows_sum += int(nr[~fb].sum())
        ncl_sum += int(nc[~fb].sum())
        sel = buf_s.sel_clusters.cpu().numpy()
        opened = set()
        for b in np.flatnonzero(~fb):
            opened.update(sel[b, :nc[b]].tolist())
        rows_union_sum += float(sizes[list(opened)].sum()) if opened else 0.0
        for v in buf_s.rounds.cpu().numpy():
            rounds_hist[int(v)] = rounds_hist.get(int(v), 0) + 1
    n_seq = nstat * r.B
    fb_rate = int(buf_s.fallback_count.item()) / n_seq
    # bound tightness xi = (largest logit of a cluster) / (its bound), Section III-A "Bound Quality Analysis", averaged over
    # the clusters the certified sequences opened; logits and bounds from the library's own entry points, a few steps
    lab = torch.from_numpy(head["labels"].astype(np.int64)).cuda()
    xi_sum, xi_n = 0.0, 0
    for s in range(W, W + min(8, nstat)):
        csv.csv_decode_step_raw(ws, idx, hp[s], r.B, buf_s, sp)
        Lf = csv.csv_full_logits(ws, idx, dh[s % nh])
        Ub, _ = csv.csv_bounds(ws, idx, dh[s % nh])
        cmax = torch.full((r.B, r.C), float("-inf"), device="cuda").scatter_reduce_(1, lab.expand(r.B, -1), Lf, "amax")
        torch.cuda.synchronize()
        fl = buf_s.flags.cpu().numpy(); nc = buf_s.n_clusters.cpu().numpy(); sel = buf_s.sel_clusters.cpu().numpy()
        ratio = (cmax / Ub).cpu().numpy()
        for b in np.flatnonzero((fl & csv.FLAG_FALLBACK) == 0):
            v = ratio[b, sel[b, :nc[b]]]
            v = v[np.isfinite(v)]
            xi_sum += float(v.sum()); xi_n += v.size
    xi = xi_sum / xi_n if xi_n else None
    del lab
    lat = np.sort(np.array(lat))

    # ---------------- full-vocabulary baseline at the same B (in-repo kernel)
    full_out = torch.empty((r.B, r.V), dtype=torch.float32, device="cuda")
    nfull = max(8, min(K, 64))
    for s in range(3):
        csv.csv_full_logits(ws, idx, dh[s % nh], out=full_out)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for s in range(nfull):
        csv.csv_full_logits(ws, idx, dh[s % nh], out=full_out)
    torch.cuda.synchronize()
    full_ms = (time.perf_counter() - t1) * 1e3 / nfull
    full_bytes = r.V * (2 * r.d + 8) + r.B * r.d * 2

    # ---------------- roofline
    # At small batches a step is a short chain of dependent launches (bounds -> round 0 with certification), none of
    # which can be timed alone from the host without adding more than it lasts, so the unit priced against the HBM
    # roofline is the whole step: algorithmic bytes of a step / the step time of the timed region above.  The
    # launch that takes most of a step's time is named next to it, with its own bytes and its share of the step
    # (step time minus the bound launch timed back to back; per-kernel durations from rocprofv3 are in profiles/).
    # When most steps contain a fallback the full-vocabulary product dominates and is timed as a launch of its own.
    mean_rows_seq = rows_sum / max(1, n_seq - int(round(fb_rate * n_seq)))
    mu_b = 2 if args.bf16_centroids else 4
    bound_bytes = r.C * r.d * mu_b + 12 * r.C + r.B * r.d * 2 + 4 * r.B * r.C
    rows_step = rows_sum / nstat
    round0_bytes = rows_step * (2 * r.d + 16) + r.B * r.d * 2 + r.B * (4 * r.C * 2) + r.B * (8 * r.k + 16)
    full_bytes_launch = r.V * (2 * r.d + 8) + r.B * r.d * 2
    bstep = step_bytes(r, r.C, rows_union_sum / nstat, anyfb / nstat, r.k, mu_b)
    eff_gbs = bstep / (ms_per_step * 1e-3) / 1e9
    sharing = rows_sum / rows_union_sum if rows_union_sum else None     # sum_b |S_b| / |union_b S_b|

    U_out = torch.empty((r.B, r.C), dtype=torch.float32, device="cuda")
    hn_out = torch.empty(r.B, dtype=torch.float32, device="cuda")

    def time_bounds(nrep, flush=None):
        """Average duration of one launch of the bound kernel(s): back to back (warm: the centroids stay in the
        256 MB last-level cache between launches), or each launch preceded by a read of a buffer larger than
        that cache and timed by its own pair of events (cold: the centroids come from HBM)."""
        for s in range(10):
            csv.lib.csv_bounds(ws._h, idx._h, hp[s], r.B, U_out.data_ptr(), hn_out.data_ptr(), sp)
        torch.cuda.synchronize()
        if flush is None:
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record(stream)
            for s in range(nrep):
                csv.lib.csv_bounds(ws._h, idx._h, hp[s % len(hp)], r.B, U_out.data_ptr(), hn_out.data_ptr(), sp)
            a1.record(stream)
            torch.cuda.synchronize()
            return a0.elapsed_time(a1) * 1e3 / nrep
        tot = 0.0
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nrep)]
        for s in range(nrep):
            flush.sum()                                   # streams the whole buffer through the caches
            evs[s][0].record(stream)
            csv.lib.csv_bounds(ws._h, idx._h, hp[s % len(hp)], r.B, U_out.data_ptr(), hn_out.data_ptr(), sp)
            evs[s][1].record(stream)
        torch.cuda.synchronize()
        # a pair of events around nothing costs a few microseconds of its own: measured and taken off
        e0_, e1_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        empty = []
        for s in range(20):
            flush[:1 << 20].sum()
            e0_.record(stream); e1_.record(stream)
            torch.cuda.synchronize()
            empty.append(e0_.elapsed_time(e1_))
        base = float(np.median(empty))
        tot = float(np.median([a.elapsed_time(b) for a, b in evs])) - base
        return tot * 1e3

    bound_name = "bound1_kernel" if r.B == 1 else ("bound_kernel" if r.B <= 4 else "bound_mfma_kernel + bound_finish_kernel")
    bound_warm_us = time_bounds(200)
    flush_buf = torch.empty(768 << 20, dtype=torch.uint8, device="cuda").zero_()
    bound_cold_us = time_bounds(30, flush_buf)
    del flush_buf
    kernels = {
        bound_name: {"bytes_per_launch": bound_bytes, "back_to_back_us": bound_warm_us,
                     "GBps_back_to_back": bound_bytes / bound_warm_us / 1e3,
                     "cold_us": bound_cold_us, "GBps_cold": bound_bytes / max(bound_cold_us, 1e-3) / 1e3,
                     "note": "back to back the centroids are served by the 256 MB last-level cache; cold = after 768 MB "
                             "of other traffic, one launch between its own events (event cost taken off)"},
    }
    if anyfb / nstat > 0.5:
        nrep = 20
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for s in range(nrep):
            csv.csv_full_logits(ws, idx, dh[s % nh], out=full_out)
        ev1.record(stream)
        torch.cuda.synchronize()
        dom_us = ev0.elapsed_time(ev1) * 1e3 / nrep
        roof = {"bound": "hbm", "kernel": "full-vocabulary product for all B sequences (full_mfma_kernel / full_gemv_kernel), the launch "
                                          "that dominates a step when most steps contain a fallback; timed back to back",
                "achieved": full_bytes_launch / dom_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "bytes_per_launch": full_bytes_launch, "avg_launch_us": dom_us}
    else:
        step_us = ms_per_step * 1e3
        rest_us = max(step_us - bound_warm_us, 1e-3)
        kernels["round 0 and what follows it (step_kernel, or round0_kernel + tail launches)"] = {
            "bytes_per_launch": round0_bytes, "in_step_us": rest_us, "share_of_step": rest_us / step_us,
            "GBps": round0_bytes / rest_us / 1e3, "frac_of_peak": round0_bytes / rest_us / 1e3 / HBM_PEAK_GBS,
            "note": "step time minus the bound launch timed back to back: a chain of dependent round trips "
                    "(bounds -> seed cluster -> its rows -> logits -> top-k, certificates), latency-bound"}
        roof = {"bound": "hbm", "kernel": f"whole decode step: {bound_name} + round-0/certification launch (dependent launches of one step)",
                "achieved": eff_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "bytes_per_launch": bstep, "avg_launch_us": step_us}
    roof["frac"] = roof["achieved"] / HBM_PEAK_GBS
    # measured HBM bytes per step: taken from the committed rocprofv3 --pmc summary of this workload (not measured in this run)
    traffic, tsrc = None, None
    tfile = os.path.join(ROOT, "profiles", f"decode_step_{r.name}_hbm_traffic.txt")
    if os.path.exists(tfile):
        for line in open(tfile):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == ("full_product" if anyfb / nstat > 0.5 else "decode_step"):
                traffic, tsrc = int(f[2]), os.path.relpath(tfile, ROOT)
    roof["traffic"] = traffic
    roof["traffic_source"] = tsrc
    roof["kernels"] = kernels

    # ---------------- CPU baseline: the oracle as it stands, on a bounded sample of the same workload
    cpu = None
    if args.cpu_steps != 0:
        from oracle import csv_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        W64 = O.bf16_to_f64(head["W_bits"])
        if args.spherical:
            oidx = O.build_index_angular(head["W_bits"], head["b"], head["labels"], r.C)
        else:
            oidx = O.build_index(head["W_bits"], head["b"], head["labels"], r.C, centroid_bf16=args.bf16_centroids,
                                 bias_table_m=args.bias_table)
        t1 = time.perf_counter()
        olad = dict(max_rounds=max(args.max_rounds, 2), delta_clusters=args.delta_clusters, relax=args.relax)
        O.decode_step(W64, head["b"], oidx, h_bits[0], r.k, r.eps, r.K_max_rows, **olad)
        one = time.perf_counter() - t1
        n_cpu = args.cpu_steps if args.cpu_steps > 0 else int(max(1, min(1024, 15.0 / max(one, 1e-3))))
        t1 = time.perf_counter()
        for s in range(n_cpu):
            O.decode_step(W64, head["b"], oidx, h_bits[(1 + s) % nh], r.k, r.eps, r.K_max_rows, **olad)
        cpu_s = time.perf_counter() - t1
        cpu = {"value": n_cpu / cpu_s, "unit": "steps/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{n_cpu} consecutive batch steps of {r.name} (B={r.B}) through oracle.decode_step, float64, numpy/BLAS"}
        log(f"[bench] oracle: {n_cpu} steps in {cpu_s:.1f}s on {cores} threads")

    out = {
        "metric": "certified decode steps/sec + effective HBM GB/s, V=128256 d=4096 B=1",
        "value": K / wall, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{r.name}: V={r.V} d={r.d} C={r.C} B={r.B} k={r.k} eps={r.eps:g} K_max={r.K_max_rows} "
                               f"combine=ALL, bf16 W and h, float32 accumulation, planted clusters"
                               + (", bf16 centroids" if args.bf16_centroids else "")
                               + (f", top-{args.bias_table} bias table" if args.bias_table >= 2 else "")
                               + (", angular index" if args.spherical else "")
                               + (", Algorithm 1's order (one cluster per iteration)" if args.alg1 else "")
                               + (f", fallback levels max_rounds={args.max_rounds} delta_clusters={args.delta_clusters} relax={int(args.relax)}"
                                  if (args.max_rounds or args.delta_clusters or args.relax) else ""), "batch": r.B},
        "roofline": roof,
        "cpu_baseline": cpu,
        "effective_hbm_GBps": eff_gbs, "algorithmic_bytes_per_step": bstep,
        "stream_ms_per_step": gpu_ms / K,
        "repeat_ms_per_step": repeats,
        "seq_steps_per_s": K * r.B / wall,
        "stage_us": stage_us,
        "latency_us": {"p50": float(lat[len(lat) // 2] * 1e6), "p95": float(lat[int(len(lat) * 0.95)] * 1e6)},
        "fallback_rate": fb_rate, "steps_with_fallback": anyfb / nstat,
        "mean_rows_per_certified_seq": mean_rows_seq, "mean_clusters_per_certified_seq": ncl_sum / max(1, n_seq - int(round(fb_rate * n_seq))),
        "sub_vocab_ratio": mean_rows_seq / r.V, "rounds_hist": {k: v for k, v in rounds_hist.items() if v or k <= 2},
        "relaxed_rate": n_relaxed / n_seq,
        "sharing_factor": sharing,
        "bound_tightness_xi": xi,
        "full_gemv": {"ms_per_step": full_ms, "steps_per_s": 1e3 / full_ms, "GBps": full_bytes / (full_ms * 1e-3) / 1e9},
        "speedup_vs_full_gemv": full_ms / ms_per_step,
    }
    plain = not (args.bf16_centroids or args.bias_table or args.spherical or args.max_rounds or args.delta_clusters or args.relax or args.alg1)
    if args.others == 1 or (args.others < 0 and args.config == "c2" and plain and args.cpu_steps != 0):
        # the main workload's buffers go first: the largest of the others needs 2.4 GB for W' alone
        del buf, buf_s, full_out, dh
        ws.free(); idx.free()
        torch.cuda.empty_cache()
        others = {}
        t_o = time.time()
        for name in ("c1", "c3", "c4", "c5"):
            if name == args.config:
                continue
            others[name] = brief(name)
            log(f"[bench] {name}: {others[name]['ms_per_step'] * 1e3:.1f} us/step, dense {others[name]['full_gemv_ms'] * 1e3:.1f} us ({time.time() - t_o:.0f}s so far)")
        out["other_configs"] = others
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
