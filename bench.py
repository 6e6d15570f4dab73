#!/usr/bin/env python3
"""Benchmark of the IVF-TQ hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
  encode half : ivftq_encode_add of the whole database into an empty index
                (normalise, coarse assignment, residual rotation, quantise, pack, list append)
  search half : ivftq_search of the query batch (coarse scoring, probe selection, query rotation,
                list scan, top-k)
The default workload is the 10M x 96 one (4,096-component anisotropic mixture of unit vectors,
nlist=4096 trained on a 500k sample, b=4, 10,000 queries, k=10, nprobe 32): the shape of the
paper's 10M image-descriptor runs (table "Recall@10 on million-scale benchmarks", Section
"Streaming ingestion at scale").  Inputs are resident in device memory before the timed region.

Prints ONE JSON line.  `value` is search QPS at the primary nprobe; encode vectors/s, recall@10,
the nprobe sweep, the roofline of the dominant kernel and the CPU oracle's throughput on a bounded
sample ride along in the same object, and so do (default run only) the same measurement on the
10M x 200 workload (k=100, shifted queries, nprobe 64) and a search on unclustered input.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16 matrix peak: the contractions run on the fp16 pipe
SPLIT_PASSES = 3               # each product is issued as hi*hi + hi*lo + lo*hi (fp32-accurate)
DTYPE = "f16-split products, f32 accumulate (f32-accurate)"


def exact_ground_truth(torch, xd, qd, k, q_chunk=1000, x_chunk=1 << 20):
    """Exact top-k by inner product of normalised rows (measurement harness, not the product)."""
    out = []
    for s in range(0, qd.shape[0], q_chunk):
        q = qd[s:s + q_chunk]
        q = q / q.norm(dim=1, keepdim=True)
        best_v = best_i = None
        for t in range(0, xd.shape[0], x_chunk):
            xb = xd[t:t + x_chunk]
            xb = xb / xb.norm(dim=1, keepdim=True)
            v, i = torch.topk(q @ xb.T, k, dim=1)
            i = i + t
            if best_v is None:
                best_v, best_i = v, i
            else:
                v2, sel = torch.topk(torch.cat([best_v, v], dim=1), k, dim=1)
                best_v, best_i = v2, torch.gather(torch.cat([best_i, i], dim=1), 1, sel)
        out.append(best_i)
    return torch.cat(out).cpu().numpy()


def stored_traffic(workload: str, nprobe: int, kernel: str):
    """HBM-side bytes per launch of `kernel` on `workload`, from the committed summary of the two
    rocprofv3 --pmc runs of this very command (FETCH_SIZE, then WRITE_SIZE, each scaled by what the
    same counter reads for a plain copy of known size): profiles/hbm_traffic_<workload>_nprobe<N>.txt,
    lines `<kernel class> <bytes per launch>`.  None when that run has not been summarised."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}_nprobe{nprobe}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) == 2 and parts[0] == kernel:
            return float(parts[1])
    return None


def recall(found, truth):
    hits = 0
    for f, t in zip(found, truth):
        hits += len(set(f.tolist()) & set(t.tolist()))
    return hits / truth.size


def host_description():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return model, os.cpu_count() or 1, usable


def cpu_baseline(w, X, Q, nprobe, full_cand_per_query):
    """The oracle, as it stands, on a bounded sample of the same workload, on the host's cores: once with
    the thread pool numpy's BLAS brings up by itself, once held to one thread."""
    from threadpoolctl import threadpool_info, threadpool_limits

    from oracle import ivftq_oracle as orc
    from workloads import synth
    model, nproc, usable = host_description()
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    n_s = min(len(X), 4 << 18)                                   # 1,048,576 rows
    q_s = min(len(Q), 1000)
    n_1, q_1 = min(n_s, 1 << 16), min(q_s, 100)                  # the single-thread leg: 65,536 rows, 100 queries
    train = min(n_s, 40_000)
    cent, _ = orc.train_coarse(X[:train], w.nlist, 1, synth.kmeans_init_indices(w.seed, train, w.nlist))
    Pi = orc.haar_rotation_from_gaussian(synth.gaussian_matrix(w.seed, w.d))
    c, tau = orc.lloyd_max_codebook(w.b, w.d)
    idx = orc.ListIndex(cent, Pi, c, tau)
    t0 = time.perf_counter()
    idx.add(X[:n_s])
    t_enc = time.perf_counter() - t0
    t0 = time.perf_counter()
    _, _, probes, _ = orc.search(idx, Q[:q_s], nprobe, w.k)
    t_search = time.perf_counter() - t0
    scanned = sum(len(idx.ids[l]) for row in probes for l in row)
    with threadpool_limits(limits=1):
        one = orc.ListIndex(cent, Pi, c, tau)
        t0 = time.perf_counter()
        one.add(X[:n_1])
        t_enc1 = time.perf_counter() - t0
        t0 = time.perf_counter()
        _, _, probes1, _ = orc.search(idx, Q[:q_1], nprobe, w.k)
        t_search1 = time.perf_counter() - t0
    scanned1 = sum(len(idx.ids[l]) for row in probes1 for l in row)
    return {
        "value": scanned / t_search / full_cand_per_query, "unit": "queries/s", "cores": int(threads), "kind": "oracle",
        "sample": (f"oracle index over the first {n_s} rows of the workload (own 1-iteration k-means on {train} rows, "
                   f"nlist={w.nlist}), {q_s} queries at nprobe={nprobe}: {scanned} candidates scored in {t_search:.2f}s; "
                   f"rate scaled to the {full_cand_per_query:.0f} candidates/query of the full index"),
        "encode_vectors_per_s": n_s / t_enc,
        "encode_sample": f"oracle encode+append of {n_s} rows in {t_enc:.2f}s",
        "single_thread": {"value": scanned1 / t_search1 / full_cand_per_query, "unit": "queries/s",
                          "encode_vectors_per_s": n_1 / t_enc1,
                          "sample": f"{q_1} queries in {t_search1:.2f}s, encode of {n_1} rows in {t_enc1:.2f}s, BLAS pool held to 1 thread"},
        "cpu_model": model, "nproc": nproc, "usable_cpus": usable,
        "note": "numpy float64; the threads are those of numpy's BLAS pool (matrix products), the rest of the oracle is single-threaded",
    }


def run_streaming(args, torch, pkg, synth):
    """Streaming ingest on the 10M x 96 distribution: coarse partition trained on the first 1M rows, those
    rows encoded, then 100k-row batches appended with nothing retrained; after every batch the 10,000 queries
    are searched (nprobe 32, k 10) against exact ground truth on everything inserted so far.  The mixture
    draws are i.i.d., so consecutive slices of the database are an i.i.d. shuffle."""
    dev = torch.device("cuda:0")
    w = synth.config_10m_d96(args.bits)
    nprobe = args.nprobe or 32
    n0, bs = 1_000_000, 100_000
    nb = min(args.stream_batches, (w.n - n0) // bs)
    t0 = time.perf_counter()
    X = synth.database(w, 0, n0 + nb * bs)
    Q = synth.queries(w)
    qd = torch.from_numpy(Q).to(dev)
    qn = qd / qd.norm(dim=1, keepdim=True)
    x0 = torch.from_numpy(X[:n0]).to(dev)
    rows = synth.train_sample_indices(w, n_available=n0)
    ix = pkg.Index(w.d, w.b, w.nlist, rotation_seed=w.seed)
    ix.train_coarse(x0[torch.from_numpy(rows).to(dev)].contiguous(), w.kmeans_iters,
                    init_rows=synth.kmeans_init_indices(w.seed, len(rows), w.nlist))
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def add(xb):
        a, b = ev(), ev()
        a.record()
        ix.encode_add(xb)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b)

    best_v = torch.full((w.nq, w.k), -float("inf"), device=dev)
    best_i = torch.full((w.nq, w.k), -1, dtype=torch.int64, device=dev)

    def extend_truth(xb, base):
        nonlocal best_v, best_i
        for t in range(0, xb.shape[0], 1 << 19):
            blk = xb[t:t + (1 << 19)]
            blk = blk / blk.norm(dim=1, keepdim=True)
            v, i = torch.topk(qn @ blk.T, w.k, dim=1)
            v2, sel = torch.topk(torch.cat([best_v, v], dim=1), w.k, dim=1)
            best_v, best_i = v2, torch.gather(torch.cat([best_i, i + base + t], dim=1), 1, sel)

    scores = torch.empty((w.nq, w.k), dtype=torch.float32, device=dev)
    ids = torch.empty((w.nq, w.k), dtype=torch.int64, device=dev)

    def measure():
        a, b = ev(), ev()
        a.record()
        ix.search(qd, nprobe, w.k, out_scores=scores, out_ids=ids)
        b.record()
        torch.cuda.synchronize()
        return recall(ids.cpu().numpy(), best_i.cpu().numpy()), a.elapsed_time(b)

    first_ms = add(x0)
    extend_truth(x0, 0)
    rec0, _ = measure()
    recalls, insert_ms, search_ms = [rec0], [], []
    for bi in range(nb):
        lo = n0 + bi * bs
        xb = torch.from_numpy(X[lo:lo + bs]).to(dev)
        torch.cuda.synchronize()
        insert_ms.append(add(xb))
        extend_truth(xb, lo)
        r, ms = measure()
        recalls.append(r)
        search_ms.append(ms)
    total = ix.ntotal()
    ix.close()
    rate = [bs / (ms * 1e-3) for ms in insert_ms]
    return {
        "metric": f"streaming insert vectors/s (100k-row batches, no retraining) + recall@10 drift (nprobe={nprobe}, k={w.k})",
        "value": float(np.mean(rate)) if rate else None, "unit": "vectors/s", "n_gpus": 1, "steps": nb, "warmup": 0,
        "ms_per_step": float(np.mean(insert_ms)) if insert_ms else None, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": f"streaming ingest: {w.d}-d unit-norm mixture, nlist={w.nlist} trained on the first {n0} rows, "
                               f"{nb} batches of {bs}, b={w.b}, {w.nq} queries after every batch", "nprobe": nprobe, "k": w.k},
        "initial_encode_vectors_per_s": n0 / (first_ms * 1e-3), "ntotal": int(total),
        "insert_vectors_per_s_min": float(np.min(rate)) if rate else None,
        "insert_vectors_per_s_median": float(np.median(rate)) if rate else None,
        "recall_at_10_first": recalls[0], "recall_at_10_last": recalls[-1], "recall_drift": recalls[-1] - recalls[0],
        "recall_at_10_min": float(np.min(recalls)), "recall_at_10_per_batch": [round(r, 4) for r in recalls],
        "search_qps_first": w.nq / (search_ms[0] * 1e-3) if search_ms else None,
        "search_qps_last": w.nq / (search_ms[-1] * 1e-3) if search_ms else None,
        "wall_s": time.perf_counter() - t0,
    }


def workload_label(w, key):
    if key == "1m":
        return "1M x 128 fp32, 1000-component Gaussian mixture, nlist=1024 (k-means on a 100k sample), b=4, 10000 queries, k=10"
    if key == "10m_d96":
        return (f"10M x 96 fp32 unit-norm, 4096-component anisotropic Gaussian mixture, nlist=4096 (k-means on a 500k sample), "
                f"b={w.b}, 10000 queries, k=10")
    if key == "10m_d200":
        return ("10M x 200 fp32, 4096-component anisotropic Gaussian mixture, queries shifted by 0.5 sigma with twice the "
                "variance, nlist=4096 (k-means on a 500k sample), b=4, 10000 queries, k=100")
    return f"{w.name}: {w.n} x {w.d}, nlist={w.nlist}, b={w.b}, {w.nq} queries, k={w.k}"


def run_workload(torch, pkg, synth, key, w, nprobe, steps, warmup, sign_bit=False, extras=True, want_cpu=True):
    """Times `steps` steps of the whole hot path on workload `w` and returns the result object."""
    dev = torch.device("cuda:0")
    t_setup = time.perf_counter()
    X = synth.database(w)
    Q = synth.queries(w)
    xd = torch.from_numpy(X).to(dev)
    qd = torch.from_numpy(Q).to(dev)
    rows = synth.train_sample_indices(w)
    sample = xd[torch.from_numpy(rows).to(dev)].contiguous()

    trainer = pkg.Index(w.d, w.b, w.nlist, rotation_seed=w.seed)
    t0 = time.perf_counter()
    trainer.train_coarse(sample, w.kmeans_iters, init_rows=synth.kmeans_init_indices(w.seed, len(rows), w.nlist))
    t_train = time.perf_counter() - t0
    cent = trainer.get_coarse()
    trainer.close()
    del sample
    truth = exact_ground_truth(torch, xd, qd, w.k)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    ix = pkg.Index(w.d, w.b, w.nlist, rotation_seed=w.seed, sign_bit=sign_bit)
    ix.set_coarse(cent)
    scores = torch.empty((w.nq, w.k), dtype=torch.float32, device=dev)
    ids = torch.empty((w.nq, w.k), dtype=torch.int64, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def step():
        a, b, c = ev(), ev(), ev()
        a.record()
        ix.encode_add(xd)
        b.record()
        ix.search(qd, nprobe, w.k, out_scores=scores, out_ids=ids)
        c.record()
        return a, b, c

    for _ in range(warmup):
        ix.reset()
        step()
        torch.cuda.synchronize()

    def timed_steps(profile):
        """K steps on the one index (emptied before each step, storage and workspace kept);
        returns (wall seconds, encode ms list, search ms list, per-kernel {name: [ms, launches]})."""
        enc, sea, prof = [], [], {}
        ix.profile_enable(profile)
        torch.cuda.synchronize()
        wall0 = time.perf_counter()
        for _ in range(steps):
            ix.reset()
            a, b, c = step()
            torch.cuda.synchronize()
            enc.append(a.elapsed_time(b))
            sea.append(b.elapsed_time(c))
            if profile:
                for name, (ms, cnt) in ix.profile_read().items():
                    t = prof.setdefault(name, [0.0, 0])
                    t[0] += ms
                    t[1] += cnt
        torch.cuda.synchronize()
        return time.perf_counter() - wall0, enc, sea, prof

    # the timed region proper, then the same K steps again with an event pair around every kernel launch
    wall, enc_ms, search_ms, _ = timed_steps(False)
    _, enc_ms_p, search_ms_p, prof = timed_steps(True)
    ix.profile_enable(False)

    found = ids.cpu().numpy()
    rec = recall(found, truth)
    scan_stats = ix.scan_stats()                               # of the last timed search
    enc_t = float(np.mean(enc_ms)) / 1e3
    search_t = float(np.mean(search_ms)) / 1e3
    qps = w.nq / search_t
    vps = w.n / enc_t

    # algorithmic work
    probe, _ = ix.coarse_probe(qd, nprobe)
    probe = probe.cpu().numpy()
    sizes = np.array([ix.list_size(l) for l in range(w.nlist)], dtype=np.int64)
    per_probe = sizes[probe]                                   # [nq, nprobe] vectors behind each probe
    cand = per_probe.sum(axis=1)
    stored_bits = w.b + (1 if sign_bit else 0)
    bytes_per_vec = (stored_bits * w.d + 7) // 8 + 2
    scan_bytes = float(cand.sum()) * bytes_per_vec             # every probed vector's codes + norm, once per query
    csum = np.cumsum(per_probe, axis=1)
    first = np.minimum((csum < w.k).sum(axis=1) + 1, nprobe)           # probes the dense pass covers at least
    stream_cand = float(np.take_along_axis(csum, (first - 1)[:, None], axis=1).sum())
    assign_flops = 2.0 * w.d * w.nlist * w.n
    per_step = {k: v[0] / steps for k, v in prof.items()}

    def avg_ms(name):
        t = prof.get(name)
        return t[0] / t[1] if t and t[1] else None

    # what a loop of nothing but the fp16 MFMA instruction reaches on this device: with constant operands
    # (close to the nominal peak) and with random operand bits (the chip lowers its clock under real data)
    mfma_const = pkg.ivftq_measure_mfma_rate(False)
    mfma_random = pkg.ivftq_measure_mfma_rate(True)

    def mfma_roof(kernel, flops, passes=SPLIT_PASSES, dtype_note="f16 (3 split passes per product, f32 accumulate)"):
        ms = avg_ms(kernel)
        if not ms:
            return None
        r = {"kernel": kernel, "bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12, "peak": MFMA_F16_PEAK_TFLOPS,
             "unit": "TFLOP/s", "traffic": stored_traffic(key, nprobe, kernel) if not sign_bit else None,
             "algorithmic_flops_per_launch": flops, "avg_launch_ms": ms, "mfma_dtype": dtype_note}
        r["frac"] = r["achieved"] / r["peak"]
        r["issued_frac"] = passes * r["frac"]            # share of the fp16 pipe's peak actually issued
        r["issued_vs_measured_pipe_rate"] = passes * r["achieved"] / mfma_random
        return r

    batched = "batch_scan" in prof
    # the assignment screens every row with one product and redoes the undecided rows with all three
    undecided = ix.assign_undecided() / float(w.n)
    rooflines = {"coarse_assign": mfma_roof("coarse_assign", assign_flops, 1.0 + SPLIT_PASSES * undecided,
                                            "f16 (screening pass: leading parts, 1 product; undecided rows: 3 split "
                                            "passes; f32 accumulate)"),
                 "encode_rotate_quantise_pack": mfma_roof("encode_rotate_quantise_pack", 2.0 * w.d * w.d * w.n)}
    if batched:
        rooflines["batch_scan"] = mfma_roof("batch_scan", 2.0 * w.d * (float(cand.sum()) - stream_cand), 1.0,
                                            "f16 (leading parts only, 1 product, f32 accumulate from the error bound: upper "
                                            "bounds; the merge re-scores the few that can reach the top k)")
        rooflines["batch_scan_nearest"] = mfma_roof("batch_scan_nearest", 2.0 * w.d * stream_cand)
    else:
        ms = avg_ms("list_scan")
        r = {"kernel": "list_scan", "bound": "hbm", "achieved": scan_bytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
             "unit": "GB/s", "traffic": stored_traffic(key, nprobe, "list_scan"),
             "algorithmic_bytes_per_launch": scan_bytes, "avg_launch_ms": ms}
        r["frac"] = r["achieved"] / r["peak"]
        rooflines["list_scan"] = r
    rooflines = {k: v for k, v in rooflines.items() if v}
    dominant = max(per_step, key=per_step.get)
    roofline = rooflines.get(dominant) or max(rooflines.values(), key=lambda r: per_step.get(r["kernel"], 0))
    # the scan stage as a whole against the bytes a per-query scan would stream (the method's own
    # accounting); above 1.0 means the batch re-used list data across queries instead of re-reading it
    scan_kernels = ("list_scan", "batch_scan_nearest", "batch_scan", "pair_grouping", "merge_topk")
    scan_stage_ms = sum(per_step.get(n, 0.0) for n in scan_kernels)
    scan_stage = {"kernels": "+".join(scan_kernels), "bound": "hbm",
                  "achieved": scan_bytes / (scan_stage_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                  "algorithmic_bytes_per_step": scan_bytes, "ms_per_step": scan_stage_ms}
    scan_stage["frac"] = scan_stage["achieved"] / scan_stage["peak"]

    def median_ms(fn, reps=3):
        ts = []
        for _ in range(reps):
            a, b = ev(), ev()
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return float(np.median(ts))

    sweep = []
    for npb in w.nprobe:
        ms = median_ms(lambda: ix.search(qd, npb, w.k, out_scores=scores, out_ids=ids))
        sweep.append({"nprobe": npb, "qps": w.nq / (ms / 1e3), "recall_at_k": recall(ids.cpu().numpy(), truth)})

    rerank_info = cascade_info = streaming_info = None
    if extras:
        # optional re-ranking on raw vectors: the 50 best by estimate re-scored exactly (reported, not the headline)
        if w.k <= 50:
            r = 50
            sc_r = torch.empty((w.nq, r), dtype=torch.float32, device=dev)
            id_r = torch.empty((w.nq, r), dtype=torch.int64, device=dev)
            holder = {}

            def rr():
                ix.search(qd, nprobe, r, out_scores=sc_r, out_ids=id_r)
                holder["ids"] = pkg.ivftq_rerank(qd, xd, id_r, w.k)[1]
            ms = median_ms(rr)
            rerank_info = {"candidates": r, "qps": w.nq / (ms / 1e3), "recall_at_k": recall(holder["ids"].cpu().numpy(), truth),
                           "note": "ivftq_search with k=50, then ivftq_rerank on the raw rows (kept by the caller)"}

        # the per-query streaming scan (what a small batch gets): its list scan against the HBM roofline
        nq_s = min(256, w.nq)
        qs = qd[:nq_s].contiguous()
        ix.set_search_mode(1)
        for _ in range(2):
            ix.search(qs, nprobe, w.k)
        torch.cuda.synchronize()
        ix.profile_enable(True)
        ix.profile_read()
        a, b = ev(), ev()
        a.record()
        for _ in range(5):
            ix.search(qs, nprobe, w.k)
        b.record()
        torch.cuda.synchronize()
        ps = ix.profile_read()
        ix.profile_enable(False)
        ix.set_search_mode(0)
        ls_ms = ps["list_scan"][0] / ps["list_scan"][1]
        bytes_s = float(cand[:nq_s].sum()) * bytes_per_vec
        streaming_info = {"nq": nq_s, "qps": nq_s / (a.elapsed_time(b) / 5 / 1e3), "list_scan_ms": ls_ms,
                          "roofline": {"kernel": "list_scan", "bound": "hbm", "achieved": bytes_s / (ls_ms * 1e-3) / 1e9,
                                       "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bytes_s / (ls_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                       "algorithmic_bytes_per_launch": bytes_s,
                                       "traffic": stored_traffic(key, nprobe, "list_scan_streaming")},
                          "note": "ivftq_set_search_mode(1): a row of workgroups per query walks its probed lists, every "
                                  "candidate's packed codes and norm streamed once per query"}

        # the same kernel on a call that reads the index many times over (the launch then works through it in
        # cache-sized slices), and whole-search latency of small calls (which mode 0 gives to the streaming path)
        nq_l = min(4096, w.nq)
        ql = qd[:nq_l].contiguous()
        ix.set_search_mode(1)
        for _ in range(2):
            ix.search(ql, nprobe, w.k)
        torch.cuda.synchronize()
        ix.profile_enable(True)
        ix.profile_read()
        for _ in range(3):
            ix.search(ql, nprobe, w.k)
        torch.cuda.synchronize()
        pl = ix.profile_read()
        ix.profile_enable(False)
        ix.set_search_mode(0)
        ll_ms = pl["list_scan"][0] / pl["list_scan"][1]
        bytes_l = float(cand[:nq_l].sum()) * bytes_per_vec
        streaming_info["large_call"] = {"nq": nq_l, "list_scan_ms": ll_ms, "achieved": bytes_l / (ll_ms * 1e-3) / 1e9, "unit": "GB/s",
                                        "frac": bytes_l / (ll_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        lat = {}
        for n_small in (1, 16, 64):
            qsm = qd[:n_small].contiguous()
            lat[str(n_small)] = median_ms(lambda: ix.search(qsm, nprobe, w.k), 9)
        streaming_info["small_call_search_ms"] = lat

        # cascade search (top bits first, a shortlist kept, full codes second): reported, not the headline.
        # Once on the index as it is (pass 1 reads the full codes through a table that ignores the low bit) and
        # once on an index that keeps the top bits in a plane of their own (pass 1 reads only the plane).
        if w.k <= 100 and w.b >= 2:
            beta, keep = w.b - 1, min(2048, max(100, 4 * w.k))
            holder = {}

            def cs(index):
                holder["ids"] = index.search_cascade(qd, nprobe, w.k, beta, keep)[1]
            ms = median_ms(lambda: cs(ix))
            cascade_info = {"beta": beta, "n_keep": keep, "qps": w.nq / (ms / 1e3),
                            "recall_at_k": recall(holder["ids"].cpu().numpy(), truth)}
            planes = {}
            for pb in sorted({beta, max(1, w.b - 2)}, reverse=True):       # a plane of b-1 bits, and one of b-2
                ixp = pkg.Index(w.d, w.b, w.nlist, rotation_seed=w.seed, sign_bit=sign_bit)
                ixp.set_coarse(cent)
                ixp.set_cascade_plane(pb)
                ixp.encode_add(xd)
                holder["ids"] = ixp.search_cascade(qd, nprobe, w.k, pb, keep)[1]
                ms_p = median_ms(lambda: ixp.search_cascade(qd, nprobe, w.k, pb, keep))
                rec_p = recall(holder["ids"].cpu().numpy(), truth)
                ms_f = median_ms(lambda: ix.search_cascade(qd, nprobe, w.k, pb, keep))
                # the streaming scan (bandwidth-side kernel) on 256 queries, with and without the plane
                ixp.set_search_mode(1)
                ix.set_search_mode(1)
                ixp.search_cascade(qs, nprobe, w.k, pb, keep)
                ix.search_cascade(qs, nprobe, w.k, pb, keep)
                ms_ps = median_ms(lambda: ixp.search_cascade(qs, nprobe, w.k, pb, keep))
                ms_fs = median_ms(lambda: ix.search_cascade(qs, nprobe, w.k, pb, keep))
                ix.set_search_mode(0)
                planes[f"beta_{pb}"] = {"qps_with_plane": w.nq / (ms_p / 1e3), "qps_without_plane": w.nq / (ms_f / 1e3),
                                        "recall_at_k": rec_p, "index_bytes_with_plane": ixp.index_bytes(),
                                        "streaming_256_queries_ms_with_plane": ms_ps,
                                        "streaming_256_queries_ms_without_plane": ms_fs}
                ixp.close()
            cascade_info["planes"] = planes

    out = {
        "metric": f"search QPS at recall@{w.k} (nprobe={nprobe}, k={w.k}) + encode vectors/s",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": wall / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": workload_label(w, key), "nprobe": nprobe, "n": w.n, "d": w.d,
                   "nlist": w.nlist, "b": w.b, "sign_bit": bool(sign_bit), "nq": w.nq, "k": w.k},
        "recall_at_k": rec,
        "search_ms": search_t * 1e3, "encode_ms": enc_t * 1e3, "encode_vectors_per_s": vps,
        "candidates_per_query": float(cand.mean()),
        "batched_scan": scan_stats,
        "index_bytes": ix.index_bytes(),
        "search_ms_with_kernel_events": float(np.mean(search_ms_p)), "encode_ms_with_kernel_events": float(np.mean(enc_ms_p)),
        "kernel_ms_per_step": per_step, "dominant_kernel": dominant, "assign_undecided_fraction": undecided,
        "roofline": roofline, "rooflines": rooflines, "scan_stage_vs_streamed_bytes": scan_stage,
        "mfma_pipe_measured": {"unit": "TFLOP/s", "instruction": "v_mfma_f32_32x32x16_f16", "constant_operands": mfma_const,
                               "random_operands": mfma_random,
                               "note": "pure MFMA loop, 2 wavefronts per SIMD; issued_vs_measured_pipe_rate compares with random_operands"},
        "sweep": sweep, "rerank": rerank_info, "cascade": cascade_info, "streaming_scan": streaming_info,
        "setup_s": t_setup, "train_coarse_s": t_train,
    }
    ix.close()
    del xd, qd
    torch.cuda.empty_cache()
    if want_cpu:
        out["cpu_baseline"] = cpu_baseline(w, X, Q, nprobe, float(cand.mean()))
    return out


def run_unclustered(torch, pkg, n, d, nlist, b, nq, nprobe, k, seed=42):
    """Search time on input with no cluster structure at all (every coordinate i.i.d. Gaussian, drawn on the
    device): the batched scan's threshold pass then lets many more candidates through than on a mixture.
    Timing only; results are checked against exact ground truth for recall."""
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    xd = torch.randn((n, d), generator=g, device=dev, dtype=torch.float32)
    qd = torch.randn((nq, d), generator=g, device=dev, dtype=torch.float32)
    ix = pkg.Index(d, b, nlist, rotation_seed=seed)
    sample = xd[:: max(1, n // 500_000)][:500_000].contiguous()
    ix.train_coarse(sample, 10, seed=seed)
    del sample
    ev = lambda: torch.cuda.Event(enable_timing=True)
    a0, a1 = ev(), ev()
    a0.record()
    ix.encode_add(xd)
    a1.record()
    scores = torch.empty((nq, k), dtype=torch.float32, device=dev)
    ids = torch.empty((nq, k), dtype=torch.int64, device=dev)
    for _ in range(2):
        ix.search(qd, nprobe, k, out_scores=scores, out_ids=ids)
    torch.cuda.synchronize()
    ts = []
    for _ in range(5):
        a, bb = ev(), ev()
        a.record()
        ix.search(qd, nprobe, k, out_scores=scores, out_ids=ids)
        bb.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(bb))
    truth = exact_ground_truth(torch, xd, qd, k)
    out = {"workload": f"{n} x {d} i.i.d. Gaussian rows (no clusters), nlist={nlist}, b={b}, {nq} queries, nprobe={nprobe}, k={k}",
           "search_ms": float(np.median(ts)), "qps": nq / (float(np.median(ts)) / 1e3),
           "encode_ms_first_call": a0.elapsed_time(a1), "recall_at_k": recall(ids.cpu().numpy(), truth)}
    ix.close()
    del xd, qd
    torch.cuda.empty_cache()
    return out


def run_cascade_plane_check(args, torch, pkg, synth):
    """Pass 1 of the cascade search through the streaming scan, with and without the plane of top bits: the two
    list-scan kernels (codes of b bits, codes of beta bits) can then be told apart in a counter trace."""
    dev = torch.device("cuda:0")
    w = {"1m": synth.config_1m, "10m_d96": lambda: synth.config_10m_d96(args.bits), "10m_d200": synth.config_10m_d200}[args.workload]()
    nprobe = args.nprobe if args.nprobe is not None else (32 if args.workload == "1m" else w.nprobe[1])
    beta = args.cascade_plane_check
    xd = torch.from_numpy(synth.database(w)).to(dev)
    qs = torch.from_numpy(synth.queries(w, 256)).to(dev)
    rows = synth.train_sample_indices(w)
    out = {"workload": workload_label(w, args.workload), "nprobe": nprobe, "beta": beta, "queries": 256}
    cent = None
    for plane in (0, beta):
        ix = pkg.Index(w.d, w.b, w.nlist, rotation_seed=w.seed)
        if cent is None:
            ix.train_coarse(xd[torch.from_numpy(rows).to(dev)].contiguous(), w.kmeans_iters,
                            init_rows=synth.kmeans_init_indices(w.seed, len(rows), w.nlist))
            cent = ix.get_coarse()
        else:
            ix.set_coarse(cent)
        ix.set_cascade_plane(plane)
        ix.set_search_mode(1)
        ix.encode_add(xd)
        keep = min(2048, max(100, 4 * w.k))
        ts = []
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            ix.search_cascade(qs, nprobe, w.k, beta, keep)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        out["with_plane_ms" if plane else "without_plane_ms"] = float(np.median(ts))
        out["index_bytes_with_plane" if plane else "index_bytes_without_plane"] = ix.index_bytes()
        ix.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--nprobe", type=int, default=None, help="primary nprobe (default: the workload's second value, 32 for 1m and 10m_d96)")
    ap.add_argument("--workload", default="10m_d96", choices=["1m", "10m_d96", "10m_d200", "stream_d96"],
                    help="10m_d96 is the benchmark workload; stream_d96 is the streaming-ingest run (1M rows, then 100k-row batches)")
    ap.add_argument("--stream-batches", type=int, default=90)
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--sign-bit", action="store_true",
                    help="store the sign-bit refinement as well (bits + 1 stored per coordinate; not the default workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", action="store_true",
                    help="the named workload alone: leave out the 10M x 200 result, the unclustered search and the extras "
                         "(what the rocprofv3 summaries under profiles/ are taken from)")
    ap.add_argument("--cascade-plane-check", type=int, default=0, metavar="BETA",
                    help="only run the cascade search's pass 1 in streaming mode on 256 queries, 3 times on an index without "
                         "and 3 times on one with a plane of the top BETA bits (for reading FETCH_SIZE of the two list scans)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy 5 times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2605_17415_amd as pkg
    from workloads import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": 5}))
        return
    if args.workload == "stream_d96":
        print(json.dumps(run_streaming(args, torch, pkg, synth)))
        return
    if args.cascade_plane_check:
        print(json.dumps(run_cascade_plane_check(args, torch, pkg, synth)))
        return
    w = {"1m": synth.config_1m, "10m_d96": lambda: synth.config_10m_d96(args.bits),
         "10m_d200": synth.config_10m_d200}[args.workload]()
    nprobe = args.nprobe if args.nprobe is not None else (32 if args.workload == "1m" else w.nprobe[1])
    t0 = time.perf_counter()
    out = run_workload(torch, pkg, synth, args.workload, w, nprobe, args.steps, args.warmup, sign_bit=args.sign_bit,
                       extras=not args.only, want_cpu=not args.no_cpu_baseline)
    default_run = args.workload == "10m_d96" and not args.only and not args.sign_bit and args.bits == 4
    if default_run:
        # the other 10M configuration (inner-product search with out-of-distribution queries, k = 100) and a
        # search on unclustered input of the benchmark's shape, in the same line
        w2 = synth.config_10m_d200()
        out["also_10m_d200"] = run_workload(torch, pkg, synth, "10m_d200", w2, w2.nprobe[1], min(args.steps, 5), min(args.warmup, 2),
                                            extras=False, want_cpu=False)
        out["unclustered_10m_d96"] = run_unclustered(torch, pkg, w.n, w.d, w.nlist, w.b, w.nq, nprobe, w.k)
    out["wall_s"] = time.perf_counter() - t0
    print(json.dumps(out))


if __name__ == "__main__":
    main()
