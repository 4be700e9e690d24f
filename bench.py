#!/usr/bin/env python3
"""Benchmark of the MI355X retrieval library on synthetic workloads of the paper's shapes.

Default: the hyperscale shard (1e9 vectors x 96-byte PQ codes, nlist 65536; 1024 queries,
nprobe 128, k 100).  One step = one whole rago_ivfpq_search call (coarse GEMM, list selection,
table build, ADC scan, top-k merge) over the query batch, inputs resident in HBM.

Prints ONE JSON line (see README/DESIGN): whole-job queries/s, the scan kernel's roofline
figures measured live with HIP events inside the library, and the CPU oracle timed on a bounded
sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

CPU_SECONDS = 10.0       # oracle time spent on the cpu_baseline sample
HBM_PEAK_GBPS = 8000.0


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def scaled_cfg(cfg, f):
    if f == 1.0:
        return cfg
    import synth  # noqa: F401
    return cfg.scaled(n=max(10000, int(cfg.n * f)), nlist=max(64, int(cfg.nlist * f)),
                      components=max(16, int(cfg.components * f)), train_n=max(20000, int(cfg.train_n * f)))


def read_traffic(name):
    """HBM bytes per launch of the dominant kernel from a committed rocprofv3 --pmc summary, if present.

    Hardware byte counters cannot be read inside this run, so the figure is quoted with its source:
    the file and the kernel time of the counter run it was taken in."""
    p = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(p):
        return None
    vals = {}
    for line in open(p):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            try:
                vals[k.strip()] = float(v.strip().split()[0])
            except ValueError:
                pass
    if "FETCH_BYTES_PER_LAUNCH" not in vals or "WRITE_BYTES_PER_LAUNCH" not in vals:
        return None
    return {"file": "profiles/" + name, "fetch_bytes": vals["FETCH_BYTES_PER_LAUNCH"], "write_bytes": vals["WRITE_BYTES_PER_LAUNCH"],
            "kernel_ms": vals.get("KERNEL_MS_UNDER_COUNTERS")}


def read_stream_ceiling(rb, gib=4.0, reps=10):
    """GB/s of the library's plain read-stream kernel over `gib` GiB, timed here with HIP events
    (far larger than the 256 MiB Infinity Cache, so every repetition reads HBM)."""
    import torch
    buf = torch.empty(int(gib * (1 << 30)), dtype=torch.uint8, device="cuda").fill_(1)
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    for _ in range(3):
        rb.rago_debug_read_stream(buf, sink)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        rb.rago_debug_read_stream(buf, sink)
    e1.record()
    torch.cuda.synchronize()
    rate = buf.numel() * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del buf, sink
    torch.cuda.empty_cache()
    return rate


def hbm_roofline(kernel, useful_bytes, kernel_ms, ceiling, prof, what, extra=None):
    """The roofline object of a bandwidth-bound kernel.

    `achieved` = bytes the kernel moves to and from HBM per launch / its HIP-event time in this run.  The bytes are
    hardware counters (FETCH_SIZE + WRITE_SIZE per launch) from the committed rocprofv3 summary named in
    `traffic_source`, taken on this same command; hardware counters cannot be read inside this process, so the
    summary's own kernel time is quoted beside them.  Without a summary for the workload the kernel's own count of
    the bytes it streams stands in and `achieved_is` says so.  `useful` = bytes of database codes (or corpus rows)
    streamed per launch / the same time: never bytes counted once per query that shares them."""
    useful = useful_bytes / (kernel_ms * 1e-3) / 1e9 if kernel_ms > 0 else 0.0
    rec = {"bound": "hbm", "kernel": kernel, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "kernel_ms": kernel_ms,
           "useful": useful, "useful_is": what, "useful_bytes_per_launch": useful_bytes,
           "ceiling": ceiling, "ceiling_is": "plain read-stream kernel over 4 GiB, timed in this run", "traffic": None}
    if prof:
        total = prof["fetch_bytes"] + prof["write_bytes"]
        rec["traffic"] = total
        rec["achieved"] = total / (kernel_ms * 1e-3) / 1e9 if kernel_ms > 0 else 0.0
        rec["achieved_is"] = "FETCH_SIZE + WRITE_SIZE bytes per launch (rocprofv3 counters, scaled by a copy of known size) / the kernel's HIP-event time in this run"
        rec["traffic_source"] = {"file": prof["file"], "kernel_ms_in_that_run": prof["kernel_ms"],
                                 "fetch_bytes": prof["fetch_bytes"], "write_bytes": prof["write_bytes"]}
        if prof["kernel_ms"]:
            rec["traffic_source"]["rate_in_that_run"] = total / (prof["kernel_ms"] * 1e-3) / 1e9
    else:
        rec["achieved"] = useful
        rec["achieved_is"] = "no counter summary for this workload: the bytes the kernel streams by its own count / its HIP-event time"
    rec["frac"] = rec["achieved"] / HBM_PEAK_GBPS
    rec["frac_useful"] = useful / HBM_PEAK_GBPS
    rec["frac_of_ceiling"] = rec["achieved"] / ceiling if ceiling else None
    if extra:
        rec.update(extra)
    assert rec["frac"] <= 1.0 and rec["frac_useful"] <= 1.0, "an HBM fraction above 1 means bytes were counted that never crossed HBM"
    return rec


def host_subindex(index, probes_np):
    """Plain index on the host holding only the lists in `probes_np` (others empty)."""
    import numpy as np
    import torch
    off = index["list_offsets"].cpu().numpy()
    nlist = len(off) - 1
    lists = np.unique(probes_np)
    lens = np.zeros(nlist, np.int64)
    lens[lists] = off[lists + 1] - off[lists]
    new_off = np.zeros(nlist + 1, np.int64)
    new_off[1:] = np.cumsum(lens)
    m = index["codes"].shape[1]
    codes = np.empty((int(new_off[-1]), m), np.uint8)
    ids = np.empty(int(new_off[-1]), np.int64)
    for l in lists:
        a, b = int(off[l]), int(off[l + 1])
        codes[new_off[l]:new_off[l + 1]] = index["codes"][a:b].cpu().numpy()
        ids[new_off[l]:new_off[l + 1]] = index["ids"][a:b].cpu().numpy()
    return dict(centroids=index["centroids"].cpu().numpy(), codebooks=index["codebooks"].cpu().numpy(),
                list_offsets=new_off, codes=codes, ids=ids)


def run_ivfpq(args):
    import numpy as np
    import torch
    import synth
    from paper_2503_14649_amd import binding as rb

    base = {"hyper": synth.HYPER, "mid": synth.MID, "tiny": synth.TINY, "iter": synth.HYPER}[args.workload]
    cfg = scaled_cfg(base, args.scale)
    if args.ksub != 256 or args.m:
        cfg = cfg.scaled(ksub=args.ksub, m=args.m or cfg.m, name=f"{cfg.name}-m{args.m or cfg.m}x{args.ksub}")
    dev = "cuda:0"
    t0 = time.time()
    last = [0.0]

    def prog(b, n):
        if time.time() - last[0] > 20:
            last[0] = time.time()
            log(f"generated {b / 1e6:.0f}M / {n / 1e6:.0f}M vectors ({time.time() - t0:.0f}s)")

    log(f"building {cfg.name} index: n={cfg.n} d={cfg.d} m={cfg.m} nlist={cfg.nlist} on {dev}")
    index = synth.build_index(cfg, device=dev, keep_vectors=False, progress=prog)
    torch.cuda.synchronize()
    lens = (index["list_offsets"][1:] - index["list_offsets"][:-1])
    log(f"index built in {time.time() - t0:.0f}s; list length min/median/max = "
        f"{int(lens.min())}/{int(lens.median())}/{int(lens.max())}")
    nq, nprobe, k = cfg.nq, cfg.nprobe, cfg.k
    if args.workload == "iter":
        nprobe, k = synth.ITER_NPROBE, synth.ITER_K
    Q = synth.make_queries(cfg, max(nq, 16), device=dev)

    # ---- CPU-oracle sample (needs the plain codes, so fetch them before they are released)
    cpu = None
    sample_ref = None
    ns = min(args.cpu_queries, nq) if args.cpu_queries > 0 else 0
    if ns:
        import oracle
        Qs = Q[:ns].cpu().numpy()
        cen = index["centroids"].cpu().numpy()
        pr = oracle.select(oracle.coarse(Qs, cen, metric=args.metric), nprobe)
        sub = host_subindex(index, pr)
        log(f"oracle sample: {ns} queries, {sub['codes'].nbytes / 1e9:.2f} GB of codes on the host")
        oracle.ivfpq_search(Qs[:1], sub, nprobe, k, metric=args.metric)   # warm-up (library load, page-in)
        # the sample is searched again and again until about CPU_SECONDS of oracle time have been spent (a sample
        # with more queries would need more of the billion-vector index on the host)
        t1 = time.time()
        sample_ref = oracle.ivfpq_search(Qs, sub, nprobe, k, metric=args.metric)
        reps = 1
        while time.time() - t1 < CPU_SECONDS and reps < 200:
            oracle.ivfpq_search(Qs, sub, nprobe, k, metric=args.metric)
            reps += 1
        dt = time.time() - t1
        cpu = {"value": ns * reps / dt, "unit": "queries/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{ns} of {nq} queries on the full index (only the lists they probe copied to the host), searched {reps} "
                         f"times in {dt:.2f}s wall, OpenMP over queries"}
        log(f"oracle: {ns * reps / dt:.2f} queries/s on {oracle.num_threads()} threads")
        del sub

    torch.cuda.empty_cache()
    rb.rago_debug_force_scan_kernel(args.scan_kernel)
    h = rb.rago_index_wrap(index, 0, metric=args.metric)
    info = rb.rago_index_info(h)
    del index["codes"]
    torch.cuda.empty_cache()
    log(f"index wrapped ({info.code_bytes_resident / 1e9:.1f} GB of codes resident); total setup {time.time() - t0:.0f}s")

    if args.workload == "iter":
        return run_iter(args, rb, h, Q, cfg, cpu, index["centroids"])

    Qb = Q[:nq].contiguous()
    out = (torch.empty(nq, k, dtype=torch.int64, device=dev), torch.empty(nq, k, dtype=torch.float32, device=dev),
           torch.empty(nq, k, dtype=torch.int32, device=dev))
    if args.calib_copy_gib > 0:     # a copy of known size for scaling hardware byte counters
        a = torch.empty(int(args.calib_copy_gib * (1 << 30)), dtype=torch.uint8, device=dev).fill_(1)
        b = torch.empty_like(a)
        rb.rago_debug_copy(a, b)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()
    for _ in range(args.warmup):
        rb.rago_ivfpq_search(h, Qb, nprobe, k, out=out)
    torch.cuda.synchronize()
    rb.rago_debug_profile(h, True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        rb.rago_ivfpq_search(h, Qb, nprobe, k, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    stages, ncalls = rb.rago_debug_stage_ms(h)
    rb.rago_debug_profile(h, False)
    cnt = rb.rago_debug_counters(h)
    algo_bytes, streamed = cnt[2], cnt[1]
    scan_ms = stages["scan"]
    ceiling = read_stream_ceiling(rb) if args.ceiling else None
    parity = None
    if sample_ref is not None:
        gi, gis = out[0][:ns].cpu().numpy(), out[2][:ns].cpu().numpy()
        ov = float(np.mean([len(set(gi[q].tolist()) & set(sample_ref["ids"][q].tolist())) / k for q in range(ns)]))
        parity = {"queries": ns, "topk_id_overlap": ov,
                  "ids_bit_exact": bool(np.array_equal(gi, sample_ref["ids"])),
                  "iscores_bit_exact": bool(np.array_equal(gis, sample_ref["iscores"]))}
    mbytes = cfg.m // 2 if cfg.ksub == 16 else cfg.m
    prof = read_traffic(f"scan_m{mbytes}_{cfg.name}_pmc.txt") if args.scale == 1.0 and args.metric == "ip" and cfg.ksub == 256 else None
    scan_name = {1: "rago::scan_kernel", 2: "rago::narrow::scan_kernel", 3: "rago::wavescan::scan_kernel"}.get(cnt[6], "scan_kernel")
    roof = hbm_roofline(
        f"{scan_name}<{mbytes}>", streamed, scan_ms, ceiling, prof,
        "code bytes the scan kernel streams from HBM per launch (the library's own count: every pass over a list once, "
        "whatever number of queries it serves) / the kernel's HIP-event time",
        {"algorithmic_bytes_per_launch": algo_bytes, "code_bytes_streamed_per_launch": streamed,
         "algorithmic_rate": algo_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0,
         "algorithmic_rate_is": "sum over (query, probed list) pairs of list length x code bytes, per second of kernel time: "
                                "the user-visible rate, above the HBM rate by the reuse factor",
         "reuse_factor": algo_bytes / streamed if streamed else None, "launches_timed": ncalls})
    rec = {
        "metric": ("ivfpq_queries_per_s_1Bx96B_shard" if cfg.name == "hyper" and args.scale == 1.0 else f"ivfpq_queries_per_s_{cfg.name}")
                  + ("" if args.metric == "ip" else "_l2"),
        "value": nq / (ms * 1e-3), "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: n={cfg.n} d={cfg.d} m={cfg.m} nlist={cfg.nlist} nq={nq} nprobe={nprobe} k={k}",
                   "scale": args.scale, "similarity": args.metric, "ksub": cfg.ksub},
        "roofline": roof,
        "stage_ms": stages,
        "scan_tasks": cnt[0], "inexact_probe_queries": cnt[3],
        "list_len_min_med_max": [int(lens.min()), int(lens.median()), int(lens.max())],
        "cpu_baseline": cpu, "parity_sample": parity,
    }
    print(json.dumps(rec), flush=True)
    rb.rago_index_free(h)


def run_iter(args, rb, h, Q, cfg, cpu, cen_dev):
    """Iterative retrieval: 8 sequential rounds per request chain at batch 1 / 4 / 16."""
    import numpy as np
    import torch
    import synth
    nprobe, k = synth.ITER_NPROBE, synth.ITER_K
    g = torch.Generator(device="cuda").manual_seed(cfg.seed * 10 + 9)
    res = {}
    batches = tuple(int(x) for x in args.iter_batches.split(",")) if args.iter_batches else synth.ITER_BATCHES
    for b in batches:
        lat = []
        out = (torch.empty(b, k, dtype=torch.int64, device="cuda"), torch.empty(b, k, dtype=torch.float32, device="cuda"),
               torch.empty(b, k, dtype=torch.int32, device="cuda"))
        chains = max(args.steps, 100)       # request chains of 8 rounds each: median and p99 over >= 800 rounds
        rb.rago_debug_profile(h, False)
        for c in range(chains + 1):
            if c == 1:
                rb.rago_debug_profile(h, True)
            q = Q[:b].contiguous() if c == 0 else synth.make_queries(cfg, b, device="cuda", stream=20 + c)
            for r in range(synth.ITER_ROUNDS):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                rb.rago_ivfpq_search(h, q, nprobe, k, out=out)
                e1.record()
                torch.cuda.synchronize()
                if c > 0:
                    lat.append(e0.elapsed_time(e1))
                q = synth.drift_queries(q, synth.ITER_DRIFT, g)
        lat = np.array(lat)
        stages, _ = rb.rago_debug_stage_ms(h)
        rb.rago_debug_profile(h, False)
        # the same rounds with the whole search of one round captured once in a HIP graph and replayed
        # (the call only enqueues kernels on the caller's stream, so it can be captured as it is)
        q_static = Q[:b].clone()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            rb.rago_ivfpq_search(h, q_static, nprobe, k, out=out)
        glat, same = [], True
        for c in range(chains):
            q = synth.make_queries(cfg, b, device="cuda", stream=20 + c + 1)
            for r in range(synth.ITER_ROUNDS):
                q_static.copy_(q)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                graph.replay()
                e1.record()
                torch.cuda.synchronize()
                glat.append(e0.elapsed_time(e1))
                if c == 0 and r < 2:                 # replays against the eager call on the same queries
                    gi = out[0].clone()
                    ei = rb.rago_ivfpq_search(h, q, nprobe, k)[0]
                    same = same and bool(torch.equal(gi, ei))
                q = synth.drift_queries(q, synth.ITER_DRIFT, g)
        glat = np.array(glat)
        res[str(b)] = {"round_ms_median": float(np.median(lat)), "round_ms_p99": float(np.percentile(lat, 99)),
                       "queries_per_s": float(b / (np.median(lat) * 1e-3)), "stage_ms": stages,
                       "graph_round_ms_median": float(np.median(glat)), "graph_round_ms_p99": float(np.percentile(glat, 99)),
                       "graph_equals_eager": same}
    # ---- the same rounds with probes chosen through an upper level over the lists (two-level coarse search)
    tree = None
    if args.upper:
        nsuper, nsp = (int(x) for x in args.upper.split(","))
        t1 = time.time()
        upper = synth.build_upper_level(cen_dev, nsuper, seed=cfg.seed * 10 + 7)
        sizes = (upper["super_offsets"][1:] - upper["super_offsets"][:-1])
        rb.rago_index_set_upper_level(h, upper)
        log(f"upper level: {nsuper} groups in {time.time() - t1:.1f}s, lists per group min/median/max = "
            f"{int(sizes.min())}/{int(sizes.median())}/{int(sizes.max())}; keeping {nsp} groups per query")
        tree = {"nsuper": nsuper, "nsp": nsp, "group_size_min_med_max": [int(sizes.min()), int(sizes.median()), int(sizes.max())],
                "per_batch": {}}
        for b in batches:
            out = (torch.empty(b, k, dtype=torch.int64, device="cuda"), torch.empty(b, k, dtype=torch.float32, device="cuda"),
                   torch.empty(b, k, dtype=torch.int32, device="cuda"))
            lat, agree = [], []
            for c in range(max(args.steps, 100) + 1):
                q = synth.make_queries(cfg, b, device="cuda", stream=20 + c)
                for r in range(synth.ITER_ROUNDS):
                    rb.rago_index_set_upper_probe(h, nsp)
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    rb.rago_ivfpq_search(h, q, nprobe, k, out=out)
                    e1.record()
                    torch.cuda.synchronize()
                    if c > 0:
                        lat.append(e0.elapsed_time(e1))
                    if c == 1:                         # agreement of the results with the exhaustive list level
                        ti = out[0].clone()
                        rb.rago_index_set_upper_probe(h, 0)
                        ei = rb.rago_ivfpq_search(h, q, nprobe, k)[0]
                        agree.append(float(np.mean([len(set(ti[i].tolist()) & set(ei[i].tolist())) / k for i in range(b)])))
                    q = synth.drift_queries(q, synth.ITER_DRIFT, g)
            lat = np.array(lat)
            # (round 0 = queries near the data; later rounds drift away from it and their nearest lists scatter)
            tree["per_batch"][str(b)] = {"round_ms_median": float(np.median(lat)), "round_ms_p99": float(np.percentile(lat, 99)),
                                         "topk_overlap_with_exhaustive_coarse_round0": agree[0],
                                         "topk_overlap_with_exhaustive_coarse_all_rounds": float(np.mean(agree))}
        rb.rago_index_set_upper_probe(h, 0)
    rec = {"metric": "ivfpq_iterative_round_latency", "value": res[str(batches[0])]["round_ms_median"], "unit": "ms", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": res[str(batches[0])]["round_ms_median"], "higher_is_better": False,
           "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
           "config": {"workload": f"iterative on {cfg.name}: n={cfg.n} nlist={cfg.nlist} nprobe={nprobe} k={k} rounds=8 "
                                  f"batches=1/4/16 drift_sigma={synth.ITER_DRIFT}", "scale": args.scale,
                      "request_chains": max(args.steps, 100)},
           "per_batch": res, "upper_level": tree, "cpu_baseline": cpu}
    print(json.dumps(rec), flush=True)
    rb.rago_index_free(h)


def run_flat(args):
    import numpy as np
    import torch
    import synth
    from paper_2503_14649_amd import binding as rb
    cfg = synth.FLAT
    R = max(1, int(cfg.requests * min(1.0, args.scale * 4))) if args.scale < 1.0 else cfg.requests
    corpus, queries = synth.make_flat(cfg, requests=R, device="cuda:0")
    half = args.flat_format == "f16"
    if half:
        corpus, queries = corpus.to(torch.float16), queries.to(torch.float16)   # same embeddings, stored as binary16
    search = rb.rago_flat_search_f16 if half else rb.rago_flat_search
    if args.calib_copy_gib > 0:     # a copy of known size for scaling hardware byte counters
        a = torch.empty(int(args.calib_copy_gib * (1 << 30)), dtype=torch.uint8, device="cuda").fill_(1)
        b = torch.empty_like(a)
        rb.rago_debug_copy(a, b)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()
    out = (torch.empty(R, cfg.nq, cfg.k, dtype=torch.int64, device="cuda"),
           torch.empty(R, cfg.nq, cfg.k, dtype=torch.float32, device="cuda"))
    for _ in range(args.warmup):
        search(corpus, queries, cfg.k, out=out)
    torch.cuda.synchronize()
    rb.rago_debug_flat_profile(0, True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        search(corpus, queries, cfg.k, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    fst, _ = rb.rago_debug_flat_stage_ms(0)
    rb.rago_debug_flat_profile(0, False)
    scan_ms, merge_ms = fst["scan"], fst["merge"]
    algo = R * cfg.n * cfg.d * 2
    cpu = None
    if args.cpu_queries > 0:
        import oracle
        rs = min(2, R)
        cb = corpus[:rs].cpu().view(torch.int16).numpy().view(np.uint16)
        qb = queries[:rs].cpu().view(torch.int16).numpy().view(np.uint16)
        t1 = time.time()
        oi, osc = oracle.flat_search(cb, qb, cfg.k, fmt=args.flat_format)
        reps = 1
        while time.time() - t1 < CPU_SECONDS and reps < 200:
            oracle.flat_search(cb, qb, cfg.k, fmt=args.flat_format)
            reps += 1
        dt = time.time() - t1
        gi = out[0][:rs].cpu().numpy()
        ov = float(np.mean([len(set(gi[r, q].tolist()) & set(oi[r, q].tolist())) / cfg.k for r in range(rs) for q in range(cfg.nq)]))
        cpu = {"value": rs * reps / dt, "unit": "requests/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"{rs} of {R} requests, searched {reps} times in {dt:.2f}s wall", "topk_id_overlap": ov}
    ceiling = read_stream_ceiling(rb) if args.ceiling else None
    prof = read_traffic("flat_32x100k_pmc.txt") if R == cfg.requests and not half else None
    roof = hbm_roofline("flat_scan_kernel", algo, scan_ms, ceiling, prof,
                        "corpus bytes (every row read once for all 16 queries of its request) / the scan kernel's HIP-event time",
                        {"algorithmic_bytes_per_launch": algo, "whole_call_rate": algo / (ms * 1e-3) / 1e9})
    rec = {"metric": "flat_requests_per_s" + ("_f16" if half else ""), "value": R / (ms * 1e-3), "unit": "requests/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": args.flat_format, "data": "synthetic",
           "config": {"workload": f"flat: R={R} n={cfg.n} d={cfg.d} nq={cfg.nq} k={cfg.k}", "scale": args.scale},
           "roofline": roof, "stage_ms": {"scan": scan_ms, "merge": merge_ms},
           "cpu_baseline": cpu}
    print(json.dumps(rec), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 10; 100 for the flat workload, whose step is ~1 ms)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="hyper", choices=["hyper", "mid", "tiny", "iter", "flat"])
    ap.add_argument("--scale", type=float, default=1.0, help="shrink n/nlist/components by this factor (development runs)")
    ap.add_argument("--calib-copy-gib", type=float, default=0.0,
                    help="also run the library's plain copy kernel over this many GiB (profiling yardstick)")
    ap.add_argument("--cpu-queries", type=int, default=64, help="queries in the CPU-oracle sample (0 = skip)")
    ap.add_argument("--upper", default="", help="iter workload: also run with an upper level over the lists, 'groups,kept' (e.g. 256,8)")
    ap.add_argument("--iter-batches", default="", help="iter workload: batch sizes to run, e.g. '1' or '1,16' (default 1,4,16; profiling runs)")
    ap.add_argument("--flat-format", default="bf16", choices=["bf16", "f16"], help="flat workload: number format of the embeddings")
    ap.add_argument("--ksub", type=int, default=256, choices=[256, 16],
                    help="codewords per sub-quantiser; 16 = 4-bit codes, two sub-quantisers per code byte")
    ap.add_argument("--m", type=int, default=0, help="sub-quantisers (default: the workload's)")
    ap.add_argument("--no-ceiling", dest="ceiling", action="store_false",
                    help="skip the read-stream ceiling measurement (a 4 GiB buffer read ten times)")
    ap.add_argument("--scan-kernel", default="auto", choices=["auto", "wide", "narrow", "wave"],
                    help="pin one of the library's scan kernels (development runs; the default lets the library choose)")
    ap.add_argument("--metric", default="ip", choices=["ip", "l2"],
                    help="similarity of the IVF-PQ workloads: inner product (the headline) or minus squared Euclidean distance")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = 100 if args.workload == "flat" else 10
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one GPU's shard at real shape); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.workload == "flat":
        run_flat(args)
    else:
        run_ivfpq(args)


if __name__ == "__main__":
    main()
