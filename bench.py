"""Benchmark of the centroid-cache hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_large]

The default workload is the large compute-bound lookup (1,048,576 centroids x 1,024, batches of 16,384);
--workload c2_mid | c4_stream | c5_merge give the mid-size lookup (with the offline passes timed beside it),
the streaming lookup with updates between micro-batches, and the all-pairs merge.

A step is one pass of the online path over one batch of synthetic queries that already
sit in GPU memory: siso_lookup (query norms, similarity against every cached centroid,
top-1, hit test) followed by siso_update_hits (hit queries fold into their centroid).
The offline merge pass (pair search + group merge) is timed once after the steps and
reported beside them; it is not part of a step because it runs once per cache refresh,
not once per batch.  Prints one JSON line.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # dense bf16 MFMA, MI355X
PEAK_FP8_TFLOPS = 5000.0   # dense fp8 MFMA
PEAK_HBM_GBS = 8000.0      # HBM3E


def measured_traffic(workload):
    """Bytes per launch of the dominant kernel from the committed counter summary, or None when the
    kernel source has changed since the counters were taken."""
    import hashlib

    h = hashlib.sha256()
    for f in ("lookup_mfma.hip", "siso_internal.h"):
        with open(os.path.join(ROOT, "paper_2508_18736_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    sha = h.hexdigest()[:16]
    try:
        with open(os.path.join(ROOT, "profiles", "traffic_counters.txt")) as fh:
            for line in fh:
                t = line.split()
                if len(t) == 6 and t[0] == workload and t[1] == sha:
                    return (float(t[2]) * float(t[3]) + float(t[4]) * float(t[5])) * 1024.0
    except OSError:
        pass
    return None


def add_measured_peak(siso, roof):
    """Beside the published peak: what a bare MFMA loop (random operands, as real data) or a bare streaming
    read reaches on this very chip, measured now with the library's probe, and the fraction of that."""
    try:
        if roof["bound"] == "mfma":
            roof["measured_peak"] = siso.probe(0)
            roof["measured_peak_constant_operands"] = siso.probe(1)
        else:
            roof["measured_peak"] = siso.probe(2)
        roof["frac_of_measured_peak"] = roof["achieved"] / roof["measured_peak"]
    except Exception as e:  # the probe is an extra: the line stands without it
        roof["measured_peak"] = None
        roof["measured_peak_error"] = str(e)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c3_large", choices=["c2_mid", "c3_large", "c4_stream", "c5_merge"])
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU work given to the oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-merge", action="store_true")
    ap.add_argument("--two-calls", action="store_true", help="a step as siso_lookup + siso_update_hits instead of siso_lookup_update")
    ap.add_argument("--storage", default="bf16", choices=["bf16", "fp8"],
                    help="fp8: the 8-bit storage variant of the cache (lookups only: a step is siso_lookup)")
    ap.add_argument("--option", action="append", default=[], help="name=value for siso_set_option")
    ap.add_argument("--path", type=int, default=0, help="siso_set_lookup_path (0 = auto)")
    ap.add_argument("--operands", default="workload", choices=["workload", "signs", "ones", "zeros"],
                    help="diagnosis of the power limit: the same shapes, launches and bytes with operand values that switch "
                         "fewer bits in the matrix cores (+-1.0 with the workload's signs, all 1.0, all 0.0)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a known-size reference for byte counters)")
    return ap.parse_args()


def cpu_baseline(wl, n_batch, seconds):
    """The oracle, as it stands, on a bounded sample of the same queries."""
    import oracle

    oracle.build()
    threads = oracle.threads()
    k = min(4 * threads, n_batch)
    oracle.lookup_rows(wl.centroids, wl.queries[:k], wl.thresholds[0], wl.dtype)  # thread start-up, page-in
    t0 = time.perf_counter()
    oracle.lookup_rows(wl.centroids, wl.queries[:k], wl.thresholds[0], wl.dtype)
    per_q = (time.perf_counter() - t0) / k
    # (in the streaming workload the sample runs over several batches, against the centroids as loaded)
    m = int(max(2, min(wl.n, seconds / max(per_q, 1e-9))))
    t0 = time.perf_counter()
    oracle.lookup_rows(wl.centroids, wl.queries[:m], wl.thresholds[0], wl.dtype)
    dt = time.perf_counter() - t0
    return {"value": m / dt, "unit": "queries/s", "cores": threads, "kind": "oracle",
            "sample": f"first {m} queries of the workload against all {wl.K} centroids, {dt:.1f} s"}


def cpu_baseline_pairs(wl, theta, seconds):
    """The oracle's pair search on the first m rows; its cost grows with the square of the rows, so the
    rate for the whole triangle is the measured one scaled by (m / K)."""
    import oracle

    oracle.build()
    threads = oracle.threads()

    def run(m):
        oc = oracle.OracleCache(wl.dim, m, wl.dtype)
        oc.load(wl.centroids[:m])
        t0 = time.perf_counter()
        oc.merge(theta, cap=0)
        return time.perf_counter() - t0

    run(1024)
    t = run(4096)
    m = int(min(wl.K, max(4096, 4096 * (seconds / max(t, 1e-6)) ** 0.5)))
    dt = run(m)
    return {"value": m / dt * (m / wl.K), "unit": "rows/s", "cores": threads, "kind": "oracle",
            "sample": f"all pairs of the first {m} rows in {dt:.1f} s ({m / dt:.0f} rows/s); the work grows with the "
                      f"square of the rows, so the rate for all {wl.K} rows is that times {m}/{wl.K}"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2508_18736_amd import siso
    from paper_2508_18736_amd import workloads as W
    from paper_2508_18736_amd.siso import to_dev, to_host

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    name = args.workload
    t0 = time.perf_counter()
    wl = W.FULL_CONFIGS[name]()
    gen_s = time.perf_counter() - t0
    d, K = wl.dim, wl.K
    fp8 = args.storage == "fp8"
    if fp8 and name == "c5_merge":
        print("bench.py: the 8-bit storage variant serves lookups only", file=sys.stderr)
        sys.exit(2)
    cache = siso.SisoCache(d, K, siso.FP8 if fp8 else siso.BF16)
    cache.set_lookup_path(args.path)
    for o in args.option:
        k, v = o.split("=")
        cache.set_option(k, int(v))
    def operands(t):
        if args.operands == "signs":
            return torch.where(t > 0, 1.0, -1.0).to(t.dtype)
        if args.operands == "ones":
            return torch.ones_like(t)
        if args.operands == "zeros":
            return torch.zeros_like(t)
        return t

    cents = operands(to_dev(wl.centroids, "bf16"))
    cache.load(cents)
    del cents
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 18, dtype=torch.float32, device="cuda:0")
        dst = src.clone()  # reads and writes copy_probe_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    out = {"n_gpus": 1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.storage,
           "data": "synthetic" if args.operands == "workload" else f"synthetic shapes, operand values replaced ({args.operands})"}
    merge_info = None

    if name == "c5_merge":
        steps = args.steps or 10
        warmup = args.warmup if args.warmup is not None else 2
        theta = wl.thresholds[0]
        cap = wl.meta["expected_pairs"] + 1024
        for _ in range(warmup):
            cache.merge(theta, cap)
        cache.profile_enable(True)
        cache.profile_read()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            pairs, total = cache.merge(theta, cap)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        kern_ms, launches = cache.profile_read()
        flop = float(K) * K * d  # upper triangle only
        avg_s = kern_ms / 1e3 / max(launches, 1)
        cache.set_option("second_set", 1)  # the one-time allocation of the arrays the survivors are gathered into
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        cache.merge_apply(pairs)
        apply_s = time.perf_counter() - t1
        # the same rows taken as a query log: community detection into a repository (second use of the pair search)
        repo = siso.SisoCache(d, K, siso.BF16)
        rows = to_dev(wl.centroids, "bf16")
        repo.cluster(rows, 0.86, 2)
        t1 = time.perf_counter()
        _, clusters, cluster_pairs = repo.cluster(rows, 0.86, 2)
        cluster_s = time.perf_counter() - t1
        out.update({"metric": "merge_centroid_rows_per_s", "value": K * steps / dt, "unit": "rows/s",
                    "steps": steps, "warmup": warmup, "ms_per_step": dt / steps * 1e3,
                    "config": {"workload": "c5_merge", "centroids": K, "dim": d, "threshold": theta,
                               "pairs": int(total), "groups_after_merge": cache.count,
                               "merge_apply_ms": apply_s * 1e3,
                               "cluster": {"vectors": K, "theta_c": 0.86, "min_size": 2, "clusters": clusters,
                                           "pairs": cluster_pairs, "ms": cluster_s * 1e3}},
                    "roofline": {"bound": "mfma", "achieved": flop / avg_s / 1e12, "peak": PEAK_BF16_TFLOPS,
                                 "unit": "TFLOP/s", "frac": flop / avg_s / 1e12 / PEAK_BF16_TFLOPS,
                                 "traffic": measured_traffic(name), "kernel_ms": avg_s * 1e3}})
        add_measured_peak(siso, out["roofline"])
        if not args.no_cpu_baseline:
            out["cpu_baseline"] = cpu_baseline_pairs(wl, theta, args.cpu_seconds)
        if args.operands != "workload":
            out["config"]["operands"] = args.operands
        print(json.dumps(out))
        return

    streaming = name == "c4_stream"
    nb = wl.batch if streaming else wl.n
    n_batches = wl.n // nb
    queries = operands(to_dev(wl.queries, "bf16"))
    # enough steps for a steady state (the first ones run on a chip that is still ramping its clocks up):
    # the whole stream of 4,096 batches; 200 mid-size batches; 10 large ones
    steps = args.steps or (4096 if streaming else 10 if name == "c3_large" else 200)
    warmup = args.warmup if args.warmup is not None else (64 if streaming else 2 if name == "c3_large" else 10)
    thetas = list(wl.thresholds)
    idx = torch.empty(nb, dtype=torch.int32, device="cuda:0")
    sim = torch.empty(nb, dtype=torch.float32, device="cuda:0")
    hit = torch.empty(nb, dtype=torch.uint8, device="cuda:0")

    two_calls = fp8 or args.two_calls
    master = None
    if fp8 and streaming:
        # the online loop with an 8-bit serving copy: the bf16 cache keeps the running means, the copy follows it
        master = siso.SisoCache(d, K, siso.BF16)
        master.load(to_dev(wl.centroids, "bf16"))
        master.reserve(nb)

    def step(i):
        q = queries[(i % n_batches) * nb:(i % n_batches + 1) * nb]
        if master is not None and args.two_calls:
            cache.lookup(q, thetas[i % len(thetas)], idx, sim, hit)
            master.update(q, idx, hit)
            cache.follow(master, idx, hit)
        elif master is not None:
            cache.lookup_update_with(master, q, thetas[i % len(thetas)], idx, sim, hit)
        elif two_calls:
            cache.lookup(q, thetas[i % len(thetas)], idx, sim, hit)
            if not fp8:
                cache.update(q, idx, hit)
        else:
            cache.lookup_update(q, thetas[i % len(thetas)], idx, sim, hit)

    for i in range(warmup):
        step(i)
    cache.profile_enable(32 if streaming else 1)  # events around every 32nd lookup kernel when steps are short
    cache.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kern_ms, launches = cache.profile_read()
    cache.profile_enable(False)
    hit_rate = float(hit.float().mean().item())
    avg_s = kern_ms / 1e3 / max(launches, 1)
    graph_ms = None
    if streaming and not args.two_calls and not args.no_merge:
        # the same steps once more, 64 of them captured in a HIP graph and replayed (the calls neither allocate nor
        # synchronise, and the one-kernel end of a step keeps nothing on the host between launches)
        side = torch.cuda.Stream()
        both = [c_ for c_ in (cache, master) if c_ is not None]
        for c_ in both:
            c_.set_stream(side)
        with torch.cuda.stream(side):
            step(0)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(64):
                step(i)
        for _ in range(4):
            graph.replay()
        torch.cuda.synchronize()
        reps = max(1, steps // 64)
        t1 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t1) / (reps * 64) * 1e3
        for c_ in both:
            c_.set_stream(torch.cuda.current_stream())
    flop = 2.0 * nb * K * d
    eb = 1.0 if fp8 else 2.0  # bytes per stored element
    peak_tflops = PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS
    if streaming:
        bytes_alg = K * d * eb + nb * d * eb + K * 4.0  # centroids + queries + inverse lengths, read once
        roof = {"bound": "hbm", "achieved": bytes_alg / avg_s / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": bytes_alg / avg_s / 1e9 / PEAK_HBM_GBS, "traffic": measured_traffic(name + ("_fp8" if fp8 else "")),
                "algorithmic_bytes": bytes_alg, "kernel_ms": avg_s * 1e3,
                "launches": launches,
                # the same bytes over the whole step (every kernel, launch and gap of it): the streaming target
                "step_frac": bytes_alg / (dt / steps) / 1e9 / PEAK_HBM_GBS}
        if graph_ms:
            roof["graph_replay_ms_per_step"] = graph_ms
            roof["graph_replay_step_frac"] = bytes_alg / (graph_ms / 1e3) / 1e9 / PEAK_HBM_GBS
    else:
        roof = {"bound": "mfma", "achieved": flop / avg_s / 1e12, "peak": peak_tflops, "unit": "TFLOP/s",
                "frac": flop / avg_s / 1e12 / peak_tflops, "traffic": measured_traffic(name + ("_fp8" if fp8 else "")),
                "algorithmic_bytes": K * d * eb + nb * d * eb + K * 4.0, "kernel_ms": avg_s * 1e3,
                "launches": launches}

    variants_info = None
    if not args.no_merge and name in ("c2_mid", "c3_large"):
        # the lookup variants on the same batch: the whole threshold sweep as one lookup (against one lookup per
        # threshold), and the 8 closest centroids of every query
        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t1) / reps * 1e3
        reps = 3 if name == "c3_large" else 20
        q0 = queries[:nb]
        sweep3 = [0.75, 0.85, 0.92]
        variants_info = {"sweep_thresholds": sweep3,
                         "sweep_one_lookup_multi_ms": timed(lambda: cache.lookup_multi(q0, sweep3), reps),
                         "sweep_three_lookups_ms": timed(lambda: [cache.lookup(q0, t, idx, sim, hit) for t in sweep3], reps),
                         "top8_ms": timed(lambda: cache.lookup_topk(q0, 8), reps)}

    t2h_info = None
    if not args.no_merge and not fp8 and name == "c2_mid":
        # threshold-to-hit-ratio table over a sample whose similarities spread over the sweep, then the
        # SLO-aware choice for one made-up operating point (LLM time 1 s, 1.2 requests/s, SLO 1.3 s)
        sweep = np.round(np.arange(0.98, 0.599, -0.02), 2).astype(np.float32)
        cents_now, _, _ = cache.export()
        sample = to_dev(W.spread_sample(to_host(cents_now, wl.dtype), wl.dtype, nb), wl.dtype)
        cache.t2h(sample, sweep)
        t1 = time.perf_counter()
        hits = cache.t2h(sample, sweep)
        t2h_s = time.perf_counter() - t1
        ratio = hits / float(nb)
        pick = siso.pick_threshold(sweep, ratio, 1.0, 1.2, 1.3)
        t2h_info = {"sample": nb, "thresholds": int(sweep.shape[0]), "ms": t2h_s * 1e3,
                    "hit_ratio_at_0.98_0.80_0.60": [float(ratio[0]), float(ratio[9]), float(ratio[19])],
                    "picked_theta": float(sweep[pick]) if pick >= 0 else None}

    if not args.no_merge and not fp8 and name == "c2_mid":
        theta_c = 0.90
        cap = 1 << 20
        cache.merge(theta_c, cap)
        cache.profile_enable(True)
        cache.profile_read()
        t1 = time.perf_counter()
        pairs, total = cache.merge(theta_c, cap)
        merge_s = time.perf_counter() - t1
        mk_ms, _ = cache.profile_read()
        cache.profile_enable(False)
        cache.set_option("second_set", 1)  # the one-time allocation of the arrays the survivors are gathered into
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        cache.merge_apply(pairs)
        apply_s = time.perf_counter() - t1
        merge_info = {"threshold": theta_c, "pairs": int(total), "pair_search_ms": merge_s * 1e3,
                      "pair_kernel_ms": mk_ms, "pair_kernel_tflops": float(K) * K * d / (mk_ms / 1e3) / 1e12,
                      "group_merge_ms": apply_s * 1e3, "centroids_after": cache.count}

    refresh_info = None
    if not args.no_merge and not fp8 and name == "c2_mid":
        # cache replacement (Algorithm 1) on a fresh copy of the cache: a repository of 10 % of its size, half of
        # it near cached centroids (they merge), half of it new directions (they join); room for 2 % more rows
        rng = np.random.Generator(np.random.Philox(key=4242))
        r = K // 10
        near = W.spread_sample(wl.centroids, wl.dtype, r // 2, sigma_lo=0.02, sigma_hi=0.1, seed=W.BASE_SEED + 8)
        fresh = W.to_storage(W.uniform_directions(W.BASE_SEED + 9, 7, r - r // 2, d), wl.dtype)
        repo = to_dev(np.concatenate([near, fresh])[rng.permutation(r)], wl.dtype)
        sizes = torch.from_numpy(rng.integers(1, 40, size=r).astype(np.float32)).to("cuda:0")
        c2 = siso.SisoCache(d, K + r, siso.BF16)
        c2.load(to_dev(wl.centroids, wl.dtype))
        c2.set_option("second_set", 1)
        c2.lookup(queries[:nb], 0.85)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        merged, added, evicted = c2.refresh(repo, sizes, 0.90, K + K // 50)
        refresh_s = time.perf_counter() - t1
        refresh_info = {"repository": r, "threshold": 0.9, "max_centroids": K + K // 50, "ms": refresh_s * 1e3,
                        "merged": merged, "added": added, "evicted": evicted, "centroids_after": c2.count}
        c2.close()

    out.update({"metric": "lookup_queries_per_s", "value": nb * steps / dt, "unit": "queries/s", "steps": steps,
                "warmup": warmup, "ms_per_step": dt / steps * 1e3,
                "config": {"workload": name, "centroids": K, "dim": d, "batch": nb, "thresholds": thetas,
                           "storage": args.storage,
                           "step": ("siso_lookup (8-bit copy) + siso_update_hits (bf16 master) + siso_fp8_follow" if master is not None and args.two_calls else
                                    "siso_fp8_lookup_update (8-bit copy, bf16 master)" if master is not None else
                                    "siso_lookup" if fp8 else "siso_lookup + siso_update_hits" if two_calls else "siso_lookup_update"), "hit_rate_last_batch": hit_rate,
                           "offline_merge": merge_info, "t2h": t2h_info, "refresh": refresh_info,
                           "variants": variants_info,
                           "generate_s": round(gen_s, 1)},
                "roofline": roof})
    add_measured_peak(siso, out["roofline"])
    if not args.no_cpu_baseline and not fp8:
        out["cpu_baseline"] = cpu_baseline(wl, nb, args.cpu_seconds)
    if args.operands != "workload":
        out["config"]["operands"] = args.operands
    print(json.dumps(out))


if __name__ == "__main__":
    main()
