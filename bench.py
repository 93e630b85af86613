#!/usr/bin/env python3
"""Benchmark of the CollectiveKV decode hot path (fused gather + concat + attend) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--also cfg2_f32,cfg2_bf16,cfg3]

One step = one ckv_attend over the whole batch of the workload (main kernel + merge of split
histories), inputs resident in HBM.  Prints ONE JSON line:
  value        users/s = B / step time (events on the launch stream around exactly K steps)
  roofline     algorithmic bytes E per launch / mean duration of the main attention kernel over the K timed
               launches (events recorded by the library on the launch stream around every launch), against
               the 8 TB/s HBM peak; beside the mean: median, minimum and quartiles of the K launches, the
               merge kernel's time, the counter-measured HBM traffic where a profile of the workload is
               committed (a constant read from profiles/hbm_traffic.json, labelled as such), and the
               matrix-core rate
  steady_state the same per-launch statistics over a further block of launches after the timed steps (the
               first ~50 back-to-back launches of a process run at lower clocks); not part of `value`
  parity       the GPU output of the timed configuration against the CPU oracle on a seeded sample of users
  cpu_baseline the CPU oracle timed on a sample of the same workload's users, on this host's cores (and on one of them)
  also         the same figures for the other workloads (not the headline)
  prefill      the prefill stage (router argmax + projection into the packed cache): positions/s and
               matrix-core TFLOP/s against the dense peak of its matrix instruction
  offloaded    latency of one decode batch with the compressed cache read in place from pinned host memory, against the
               resident cache and against loading the batch's full-width keys (the paper's latency-table scenario), for a
               one-query and a many-candidate shape
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "users/sec and effective HBM GB/s (% of peak) for fused gather+concat+attend"
DESCRIBE = {
    "cfg1": "config 1 tiny: B=4 L=50 H=1 d=56+8 P=256 Nq=1 softmax fp32",
    "cfg2_f32": "config 2 SASRec-like: B=1024 L=200 H=2 d=56+8 P=4096 Nq=1 softmax fp32",
    "cfg2_bf16": "config 2 SASRec-like: B=1024 L=200 H=2 d=56+8 P=4096 Nq=1 softmax bf16",
    "cfg3": "config 3 HSTU-style: B=512 L=1024 H=4 d=60+4 P=16384 Zipf(1.1) Nq=64 SiLU/L bf16",
    "cfg3_ck": "config 3 with only the keys shared (CollectiveK): V is an ordinary 64-column cache",
    "cfg3_cv": "config 3 with only the values shared (CollectiveV): K is an ordinary 64-column cache",
    "cfg4": "config 4 long ragged: B=128 L~U[2048,8192] H=8 d=120+8 P=65536 Nq=128 softmax bf16",
    "cfg3_plain": "config 3 with an ordinary K/V cache (d_g = 0): the same decode without compression",
    "cfg4_plain": "config 4 with an ordinary K/V cache (d_g = 0): the same decode without compression",
    "d256_u4": "256-column heads (Table 1's width, CR 0.020): B=128 L~U[2048,8192] H=4 d=252+4 P=32768 Nq=128 softmax bf16",
    "d256_u10": "256-column heads (Table 1's width, CR 0.043): B=128 L~U[2048,8192] H=4 d=246+10 P=32768 Nq=128 softmax bf16",
    "tgt256_u1": "target attention over 256-column heads, d_u = 1 (Table 1's CR 0.008): B=1024 L~U[200,2000] H=1 d=255+1 P=16384 Nq=1 softmax bf16",
    "tgt256_u10": "target attention over 256-column heads, d_u = 10 (Table 1's CR 0.043): B=1024 L~U[200,2000] H=1 d=246+10 P=16384 Nq=1 softmax bf16",
    "cfg3_f32_d256": "config 3's shape with 256-column fp32 heads: B=128 L=1024 H=4 d=252+4 P=16384 Zipf(1.1) Nq=64 SiLU/L fp32",
    "cfg5": "config 5 large batch: B=8192 L~U[512,2048] H=4 d=62+2 P=1048576 Zipf(1.05) Nq=16 softmax bf16",
}


def compulsory_bytes(w, ab):
    """Compressed stream + every distinct touched pool row once + q + out."""
    e = 4 if w["dtype"] == 0 else 2
    rows = 0
    share = w.get("share", 0)
    for h in range(w["H"]):
        rows += (len(np.unique(w["idx_k"][:, h])) if share in (0, 1) else 0) + (len(np.unique(w["idx_v"][:, h])) if share in (0, 2) else 0)
    return ab["compressed"] + rows * w["d_g"] * e + ab["q_out"]


def launch_stats(ms):
    """Mean, median, minimum, maximum and quartiles of per-launch milliseconds."""
    ms = np.asarray(ms, dtype=np.float64)
    q = np.percentile(ms, [25, 50, 75])
    return {"launches": int(ms.size), "mean": float(ms.mean()), "median": float(q[1]), "min": float(ms.min()),
            "max": float(ms.max()), "p25": float(q[0]), "p75": float(q[2])}


def parity(w, out, budget_s):
    """The GPU output `out` (fp64 [B][H][Nq][d_a]) against the oracle on a seeded sample of users sized to
    about budget_s of oracle time: worst element against the rule of tests/parity.py and the norm-wise error."""
    from oracle import oracle
    from tests.parity import compare
    order = np.random.default_rng(1).permutation(w["B"]).astype(np.int32)
    n = min(w["B"], max(1, oracle.threads() // max(1, w["H"])))
    while True:
        users = np.sort(order[:n])
        t0 = time.time()
        ref, rss, sss, acs, asum = oracle.attend(w, users=users, with_scales=True, with_asum=True)
        dt = time.time() - t0
        if n >= w["B"] or dt >= 0.4 * budget_s:
            break
        n = int(min(w["B"], max(2 * n, n * 0.8 * budget_s / max(dt, 1e-3))))
    st = compare(out[users], ref[users], rss[users], w["dtype"], sss[users], acs[users], asum[users])
    return {"users_checked": int(n), "of": int(w["B"]), "elements": st["elements"], "tol": st["tol"],
            "max_rel_err_normwise": st["norm_err"], "worst_element_over_bound": st["worst_ratio"],
            "ok": bool(st["finite"] and st["worst_ratio"] <= 1.0),
            "rule": "|g-r| <= tol*|r| + max(tol*rss, u_w*asum) + (d_a+1)*2^-24*sss + 8*2^-24*acs (rss: root-sum-square of the element's "
                    "summands, asum: sum of their magnitudes, u_w: unit roundoff of the storage type, sss: root-sum-square of the "
                    "first-order effects of the scores' rounding, acs: sqrt(n) (|r| + root-sum-square of the summands one by one), "
                    "for the rounding of the additions; all four from the oracle)"}


def measure(name, steps, warmup, traffic_table, steady=0, parity_budget_s=0.0, with_compulsory=True):
    import torch
    from paper_2601_19178_amd import ckv, session, workloads as wl

    w = wl.config(name)
    ab = wl.algorithmic_bytes(w)
    d_a = w["d_g"] + w["d_u"]
    flop = 4.0 * w["Nq"] * d_a * ab["position_heads"]
    t0 = time.time()
    s = session.Session(w)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    for _ in range(warmup):
        s.attend()
    torch.cuda.synchronize()
    ckv.ckv_set_timing(s.cache, steps)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(steps):
        s.attend()
    stop.record()
    torch.cuda.synchronize()
    ms_step = start.elapsed_time(stop) / steps
    k_ms, m_ms = ckv.ckv_kernel_times(s.cache, steps)
    assert len(k_ms) == steps
    kst, mst = launch_stats(k_ms), launch_stats(m_ms)
    ms_kernel = kst["mean"]
    bf16 = w["dtype"] == wl.BF16
    mfma = ckv.ckv_variant(s.cache).startswith("mfma")
    peak_tflops = MFMA_BF16_PEAK_TFLOPS if bf16 else MFMA_F32_PEAK_TFLOPS
    res = {
        "workload": name,
        "describe": DESCRIBE[name],
        "variant": ckv.ckv_variant(s.cache),
        "B": w["B"], "T": int(w["lengths"].sum()),
        "ms_per_step": ms_step,
        "kernel_ms": ms_kernel,
        "kernel_ms_median": kst["median"], "kernel_ms_min": kst["min"], "kernel_ms_p25": kst["p25"], "kernel_ms_p75": kst["p75"],
        "kernel_ms_max": kst["max"],
        "merge_ms": mst["mean"],
        "users_per_s": w["B"] / (ms_step * 1e-3),
        "E_bytes": ab["E"],
        "E_GBps_step": ab["E"] / (ms_step * 1e-3) / 1e9,
        "E_GBps_kernel": ab["E"] / (ms_kernel * 1e-3) / 1e9,
        "E_GBps_kernel_median": ab["E"] / (kst["median"] * 1e-3) / 1e9,
        # E counts a pool row every time it is gathered: where the gathered rows are served by the L2s this is
        # gather bandwidth, not HBM bandwidth (see hbm_traffic below)
        "effective_gather_frac_of_hbm_peak": ab["E"] / (ms_kernel * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "effective_gather_frac_of_hbm_peak_median": ab["E"] / (kst["median"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "flop": flop,
        "TFLOPs_kernel": flop / (ms_kernel * 1e-3) / 1e12,
        "mfma_frac_of_peak": (flop / (ms_kernel * 1e-3) / 1e12 / peak_tflops) if mfma else None,
        "build_cache_s": build_s,
    }
    if with_compulsory:
        res["C_bytes"] = compulsory_bytes(w, ab)
        res["C_GBps_kernel"] = res["C_bytes"] / (ms_kernel * 1e-3) / 1e9
    tr = traffic_table.get(name, {}).get("bytes_per_launch")
    res["hbm_traffic"] = {
        "bytes_per_launch": tr,
        "source": "profiles/hbm_traffic.json (static: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this workload, "
                  "scaled by the copy-kernel calibration; not measured in this run)" if tr else None,
        "GBps": (tr / (ms_kernel * 1e-3) / 1e9) if tr else None,
        "frac_of_hbm_peak": (tr / (ms_kernel * 1e-3) / 1e9 / HBM_PEAK_GBPS) if tr else None,
        "over_E": (tr / ab["E"]) if tr else None,
    }
    if steady > 0:
        # a further block of launches, untimed by the contract: the clocks have settled by now
        ckv.ckv_set_timing(s.cache, steady)
        for _ in range(2 * steady):
            s.attend()
        torch.cuda.synchronize()
        k2, m2 = ckv.ckv_kernel_times(s.cache, steady)
        st2 = launch_stats(k2)
        res["steady_state"] = {"after_launches": warmup + steps + steady, "kernel_ms": st2, "merge_ms_mean": float(np.mean(m2)),
                               "E_GBps_median": ab["E"] / (st2["median"] * 1e-3) / 1e9,
                               "effective_gather_frac_of_hbm_peak_median": ab["E"] / (st2["median"] * 1e-3) / 1e9 / HBM_PEAK_GBPS}
    ckv.ckv_set_timing(s.cache, 0)
    if parity_budget_s > 0:
        s.out.fill_(float("nan"))
        s.attend()
        res["parity"] = parity(w, s.output(), parity_budget_s)
    return res, w, s


MFMA_BF16_PEAK_TFLOPS = 2500.0
MFMA_F32_PEAK_TFLOPS = 157.3


def measure_prefill(name, steps, warmup, with_cpu=False):
    """Prefill stage (router GEMM + argmax, projection) recomputed into a resident handle: one step = one
    ckv_prefill_into over all T positions.  Every launch is bracketed by its own event pair on the launch stream."""
    import torch
    from paper_2601_19178_amd import ckv, session, workloads as wl

    r = wl.prefill_config(name)
    decode = {"prefill_cfg2": "cfg2_bf16", "prefill_cfg3": "cfg3", "prefill_cfg2_f32": "cfg2_f32"}[name]
    peak = MFMA_F32_PEAK_TFLOPS if r["dtype"] == wl.F32 else MFMA_BF16_PEAK_TFLOPS
    w = wl.config(decode)
    s = session.Session(w, prefill=r)
    for _ in range(warmup):
        s.prefill_again()
    torch.cuda.synchronize()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for a, b in pairs:
        a.record()
        s.prefill_again()
        b.record()
    stop.record()
    torch.cuda.synchronize()
    ms_step = start.elapsed_time(stop) / steps
    ms_kernel = float(np.mean([a.elapsed_time(b) for a, b in pairs]))
    flops = wl.prefill_flops(r)
    res = {
        "workload": name,
        "describe": f"prefill of {decode}'s cache: T={r['T']} H={r['H']} d_e={r['d_e']} d_u={r['d_u']} P={r['P']} {'fp32' if r['dtype'] == wl.F32 else 'bf16'}",
        "kernel": ckv.ckv_prefill_kernel_name(s.shape, s.router),
        "ms_per_step": ms_step, "kernel_ms": ms_kernel,
        "positions_per_s": r["T"] / (ms_step * 1e-3),
        "users_per_s": w["B"] / (ms_step * 1e-3),
        "flop": flops,
        "roofline": {"bound": "mfma", "achieved": flops / (ms_kernel * 1e-3) / 1e12, "peak": peak,
                     "unit": "TFLOP/s", "frac": flops / (ms_kernel * 1e-3) / 1e12 / peak, "traffic": None},
    }
    s.close()
    if with_cpu:
        from oracle import oracle
        n, dt = 256, 0.0
        for _ in range(2):  # a first small sample sizes the second one to about five seconds of oracle time
            rs = dict(r)
            rs["S"] = np.ascontiguousarray(r["S"][:n])
            rs["T"] = n
            t0 = time.time()
            oracle.prefill(rs)
            dt = time.time() - t0
            if dt >= 2.0 or n >= r["T"]:
                break
            n = int(min(r["T"], max(n, n * 5.0 / max(dt, 1e-3))))
        res["cpu_baseline"] = {"value": n / dt, "unit": "positions/s", "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"first {n} of {r['T']} positions, all heads, both routers, {dt:.1f} s wall"}
    return res


def cpu_baseline(w, budget_s=15.0):
    """The oracle as it stands, timed on a bounded sample of users (all heads, all queries)."""
    from oracle import oracle
    threads = oracle.threads()
    order = np.random.default_rng(0).permutation(w["B"]).astype(np.int32)
    n = min(w["B"], max(1, threads // max(1, w["H"])))
    t0 = time.time()
    oracle.attend(w, users=order[:n])
    dt = time.time() - t0
    for _ in range(3):  # grow the sample until it takes about budget_s (or covers every user)
        if dt >= 0.6 * budget_s or n >= w["B"]:
            break
        n = int(min(w["B"], max(n + 1, n * budget_s / max(dt, 1e-3))))
        t0 = time.time()
        oracle.attend(w, users=order[:n])
        dt = time.time() - t0
    # and on one thread, on a sample a sixteenth as large (a few seconds)
    n1 = max(1, n // max(threads, 1))
    oracle.set_threads(1)
    try:
        t0 = time.time()
        oracle.attend(w, users=order[:n1])
        dt1 = time.time() - t0
    finally:
        oracle.set_threads(threads)
    return {"value": n / dt, "unit": "users/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {w['B']} users (seeded choice), all heads and queries, {dt:.1f} s wall",
            "single_thread": {"value": n1 / dt1, "unit": "users/s", "cores": 1,
                              "sample": f"{n1} of {w['B']} users, all heads and queries, {dt1:.1f} s wall"}}


OFFLOADED_SHAPES = {
    # target attention as in the paper's latency table: one query per user, streaming kernel
    "target": dict(L=(200, 200), H=2, d_a=64, d_u=8, P=10000, idx="uniform", Nq=1, mode=0, sigma_pool=0.125),
    # the same over 256-column heads with d_u = 4 (Table 1's width, CR 0.020) and longer histories: wide-row streaming kernel
    "target256": dict(L=(1000, 1000), H=1, d_a=256, d_u=4, P=16384, idx="uniform", Nq=1, mode=0, sigma_pool=0.0625),
    # many candidates per user, HSTU-style weighting: matrix-core kernel (config 3's shape per user)
    "candidates": dict(L=(1024, 1024), H=4, d_a=64, d_u=4, P=16384, idx=("zipf", 1.1), Nq=64, mode=1, sigma_pool=0.125),
}


def offloaded_sweep(batches=(1, 8, 32, 64, 128, 256, 512), reps=30, kinds=("target", "target256", "candidates")):
    """Decode latency of one request batch per shape of OFFLOADED_SHAPES (bf16): compressed cache read in place from
    pinned host memory, compressed cache resident in HBM, and the time to load the same batch's full-width keys from
    pinned host memory (the standard-KV-cache baseline)."""
    import torch
    from paper_2601_19178_amd import ckv, session, workloads as wl

    def median_ms(fn):
        ts = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record(); torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return float(np.median(ts[reps // 3:]))

    rows = []
    for kind in kinds:
        sh = OFFLOADED_SHAPES[kind]
        for B in batches:
            w = wl.make(B=B, dtype=wl.BF16, seed=2000 + B, **sh)
            ab = wl.algorithmic_bytes(w)
            T = int(w["lengths"].sum())
            full_keys = torch.empty(T * sh["H"] * sh["d_a"], dtype=torch.bfloat16).pin_memory()
            dev_keys = torch.empty_like(full_keys, device="cuda")
            row = {"shape": kind, "batch": B, "compressed_bytes": ab["compressed"], "full_key_bytes": full_keys.numel() * 2}
            for name, off in (("resident_ms", False), ("offloaded_ms", True)):
                s = session.Session(w, offloaded=off)
                row["kernel"] = ckv.ckv_variant(s.cache)
                for _ in range(5):
                    s.attend()
                row[name] = median_ms(s.attend)
                s.close()
            row["full_key_load_ms"] = median_ms(lambda: dev_keys.copy_(full_keys, non_blocking=True))
            row["offloaded_GBps_over_host_link"] = ab["compressed"] / (row["offloaded_ms"] * 1e-3) / 1e9
            rows.append(row)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps; the GPU needs ~50 back-to-back launches to reach its steady clocks")
    ap.add_argument("--workload", default="cfg4", choices=sorted(DESCRIBE))
    ap.add_argument("--also", default="cfg1,cfg2_f32,cfg2_bf16,cfg3,cfg5,cfg3_ck,d256_u4,cfg3_f32_d256,tgt256_u1,tgt256_u10", help="comma list of further workloads ('' for none)")
    ap.add_argument("--steady", type=int, default=200,
                    help="launches of the extra steady-state block per workload, reported under 'steady_state' (0: none)")
    ap.add_argument("--parity-budget", type=float, default=6.0,
                    help="seconds of oracle time per workload for the parity figures in the line (0: none)")
    ap.add_argument("--prefill", default="prefill_cfg2,prefill_cfg3,prefill_cfg2_f32",
                    help="comma list of prefill workloads reported under 'prefill' (prefill_cfg2, prefill_cfg3, prefill_cfg2_f32; '' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--offloaded-batches", default="1,64,512",
                    help="batch sizes of the offloaded-cache latencies reported under 'offloaded' in the line ('' for none)")
    ap.add_argument("--offloaded-sweep", action="store_true",
                    help="latency of one decode batch with the compressed cache in pinned host memory vs resident vs "
                         "loading a full-width key cache, batch 1..512 (the paper's latency-table scenario)")
    ap.add_argument("--calibrate-copy-mb", type=int, default=0,
                    help="only run the library's plain copy kernel on this many MiB (counter calibration) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the hot path has no CPU fallback")

    if args.calibrate_copy_mb > 0:
        from paper_2601_19178_amd import ckv
        nbytes = args.calibrate_copy_mb << 20
        src = torch.full((nbytes,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.zeros_like(src)
        stream = torch.cuda.current_stream().cuda_stream
        for _ in range(args.steps):
            ckv.ckv_copy(dst, src, nbytes, stream)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": nbytes, "launches": args.steps}))
        return

    if args.offloaded_sweep:
        print(json.dumps({"offloaded_sweep": offloaded_sweep()}))
        return

    traffic_table = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic_table = json.load(f)
    pb = 0.0 if args.no_cpu_baseline else args.parity_budget
    head, w, sess = measure(args.workload, args.steps, args.warmup, traffic_table, steady=args.steady, parity_budget_s=pb)
    base = None if args.no_cpu_baseline else cpu_baseline(w)
    sess.close()
    del w, sess
    also = []
    for name in [x for x in args.also.split(",") if x and x != args.workload]:
        r, w2, s2 = measure(name, args.steps, args.warmup, traffic_table, steady=args.steady, parity_budget_s=pb)
        s2.close()
        del w2, s2
        also.append(r)

    prefill = [measure_prefill(n, max(10, args.steps // 4), max(5, args.warmup // 4), with_cpu=not args.no_cpu_baseline)
               for n in args.prefill.split(",") if n]
    ob = tuple(int(x) for x in args.offloaded_batches.split(",") if x)
    offloaded = offloaded_sweep(batches=ob, reps=21) if ob else None

    line = {
        "metric": METRIC,
        "value": head["users_per_s"],
        "unit": "users/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if "bf16" in head["variant"] else "f32",
        "data": "synthetic (seeded; shapes and index/value distributions of BASELINE.json's configs)",
        "config": {"workload": head["describe"], "name": head["workload"], "kernel": head["variant"],
                   "B": head["B"], "T": head["T"]},
        "effective_GBps": head["E_GBps_step"],
        "pct_of_hbm_peak": 100.0 * head["E_GBps_step"] / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": head["E_GBps_kernel"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": head["effective_gather_frac_of_hbm_peak"], "traffic": head["hbm_traffic"]["bytes_per_launch"],
                     "traffic_source": head["hbm_traffic"]["source"], "traffic_frac_of_peak": head["hbm_traffic"]["frac_of_hbm_peak"],
                     "kernel": head["variant"], "kernel_ms": head["kernel_ms"], "kernel_ms_median": head["kernel_ms_median"],
                     "kernel_ms_min": head["kernel_ms_min"], "kernel_ms_p25": head["kernel_ms_p25"],
                     "kernel_ms_p75": head["kernel_ms_p75"], "merge_ms": head["merge_ms"],
                     "frac_median": head["effective_gather_frac_of_hbm_peak_median"],
                     "E_bytes": head["E_bytes"], "C_bytes": head.get("C_bytes"), "C_GBps": head.get("C_GBps_kernel"),
                     "mfma_TFLOPs": head["TFLOPs_kernel"], "mfma_frac_of_peak": head["mfma_frac_of_peak"]},
        "steady_state": head.get("steady_state"),
        "parity": head.get("parity"),
        "cpu_baseline": base,
        "also": also,
        "prefill": prefill,
        "offloaded": offloaded,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
