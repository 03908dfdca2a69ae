#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: one
insertion batch on the data stream (assignment, slot reservation, block
opening, fill, publication) and, concurrently, one search batch on a pooled
search stream (coarse scores, probe selection, list scan, top-k).  The
workload is the SIFT-shaped configuration (byte-valued L2, d=128, 1M base
vectors, nlist=1024, nprobe=32, k=100, block of 128 vectors, inserts in batches
of 64), with every input resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is queries per second over the timed steps;
`roofline` is for the list scan (bytes of the union of the probed lists per
launch over the launch's mean duration, measured with HIP events on the
caller's stream, against 8 TB/s; `alu_issue` is the arithmetic side of the
same launches); `cpu_baseline` is the CPU oracle on the host cores.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
VALU_ISSUE_PEAK_T = 256 * 4 * 16 * 2.4e9 / 1e12  # fp32 vector instructions per lane and second, all CUs (no packed math)


def percentile(xs, p):
    return float(np.percentile(np.asarray(xs, dtype=np.float64), p)) if len(xs) else float("nan")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=256, help="queries per search batch")
    ap.add_argument("--scale", type=float, default=1.0, help="shrinks base/query/insert counts")
    ap.add_argument("--search-streams", type=int, default=4)
    ap.add_argument("--latency-iters", type=int, default=2000)
    ap.add_argument("--cpu-queries", type=int, default=1024, help="queries of the oracle sample; 0 skips it")
    ap.add_argument("--no-extras", action="store_true", help="only the timed steps (for profiler runs)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only the plain copy kernel on 1 GiB (yardstick for the traffic counters)")
    ap.add_argument("--pq-m", type=int, default=0,
                    help="with --study pq: only this number of sub-spaces, and only the --batch query batch")
    ap.add_argument("--shape", type=int, default=0, help="with --study shapes: only this configuration (3, 4 or 5)")
    ap.add_argument("--study", choices=["rearrange", "blocksize", "pq", "storage", "shapes", "mixed", "growth"],
                    help="run one of the side studies instead of the benchmark (one JSON line each)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (lists would be sharded by owner GPU)",
              file=sys.stderr)
        return 2

    import torch
    from paper_2408_02937_amd import rtams, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            rtams.copy_plain(dst, src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_per_launch": 1 << 30, "launches": 5}))
        return 0
    if args.study:
        from paper_2408_02937_amd import studies
        fn = {"rearrange": studies.rearrangement_study, "blocksize": studies.block_size_sweep,
              "pq": studies.pq_study, "storage": studies.storage_study, "shapes": studies.shape_study,
              "mixed": studies.mixed_load_study, "growth": studies.growth_study}[args.study]
        if args.study == "pq" and args.pq_m:
            print(json.dumps(fn(scale=args.scale, iters=args.latency_iters, ms=(args.pq_m,), batches=(args.batch,))))
            return 0
        if args.study == "shapes" and args.shape:
            print(json.dumps(fn(scale=args.scale, iters=args.latency_iters, which=(args.shape,))))
            return 0
        print(json.dumps(fn(scale=args.scale, iters=args.latency_iters)))
        return 0
    t_gen = time.perf_counter()
    w = synth.config(2, scale=args.scale)
    t_gen = time.perf_counter() - t_gen
    B, k, nprobe, ib = args.batch, w.k, w.nprobe, w.insert_batch
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    base, cents, queries, inserts = map(to_dev, (w.base, w.centroids, w.queries, w.inserts))
    n_all = len(w.base) + len(w.inserts) * 2
    pool_blocks = n_all // w.block_vecs + 2 * w.nlist + 64
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=pool_blocks, n_resources=8,
                    max_batch=max(B, 256), max_k=128, max_nprobe=64, max_add_batch=65536,
                    candidates_per_query=65536)
    data_stream = torch.cuda.Stream(dev)
    search_streams = [torch.cuda.Stream(dev) for _ in range(args.search_streams)]
    g.set_centroids(cents, stream=data_stream)

    # ---- bulk load of the base set through add (one format for offline and online data)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g.add(base, stream=data_stream)
    torch.cuda.synchronize()
    bulk_s = time.perf_counter() - t0

    nq_batches = len(w.queries) // B
    q_batches = [queries[i * B:(i + 1) * B] for i in range(nq_batches)]
    n_ins_batches = len(w.inserts) // ib
    ins_batches = [inserts[i * ib:(i + 1) * ib] for i in range(n_ins_batches)]
    outs = [(torch.empty((B, k), dtype=torch.float32, device=dev),
             torch.empty((B, k), dtype=torch.int64, device=dev)) for _ in search_streams]
    ins_cursor = [0]

    def next_insert():
        b = ins_batches[ins_cursor[0] % n_ins_batches]
        ins_cursor[0] += 1
        return b

    def submit_search(i, q):
        s = i % len(search_streams)
        while True:
            try:
                g.search(q, k, nprobe, outs[s][0], outs[s][1], stream=search_streams[s])
                return
            except rtams.RtamsError as e:
                if e.code != rtams.EBUSY:
                    raise
                search_streams[(s + 1) % len(search_streams)].synchronize()

    def step(i):
        g.add(next_insert(), stream=data_stream)
        submit_search(i, q_batches[i % nq_batches])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    g.scan_time(reset=True)
    g.set_param("profile_scan", 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    g.set_param("profile_scan", 0)
    scan_ms, scan_n = g.scan_time(reset=True)
    assert g.poll_error() == 0, "a kernel raised an error during the timed steps"
    qps = args.steps * B / elapsed

    # ---- algorithmic bytes of the scan kernel per launch (what the method must read)
    sizes = g.list_sizes()
    pair_bytes, union_bytes = [], []
    for i in range(min(args.steps, nq_batches)):
        pl = g.probe(q_batches[(args.warmup + i) % nq_batches], nprobe).cpu().numpy()
        ln = sizes[pl]
        per_list = lambda l: l * w.d * 4 + ((l + w.block_vecs - 1) // w.block_vecs) * 4
        pair_bytes.append(int(per_list(ln).sum()))
        union_bytes.append(int(per_list(sizes[np.unique(pl)]).sum()))
    pair_b, union_b = float(np.mean(pair_bytes)), float(np.mean(union_bytes))
    # Arithmetic of the same launch: every (query, candidate) pair costs d subtract + d fused
    # multiply-add instructions per lane for L2 (d multiply-adds for IP); the yardstick is the rate at
    # which 256 CUs x 4 SIMDs x 16 lanes issue one fp32 instruction per lane and clock at 2.4 GHz.
    pair_vecs = pair_b / (w.d * 4 + 4.0 / w.block_vecs)
    lane_ops = pair_vecs * w.d * (2 if w.metric == "l2" else 1)
    scan_avg_ms = scan_ms / max(scan_n, 1)
    # The scan reads a list once for all the queries of the batch that probe it, so
    # the bytes it must move are those of the UNION of the probed lists; bytes
    # counted once per (query, list) pair are reported beside it, never credited.
    achieved = union_b / (scan_avg_ms * 1e-3) / 1e9 if scan_n else float("nan")
    traffic = measured_traffic(w.name, B)

    result = {
        "metric": "search QPS under concurrent insertion",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n_base": len(w.base), "d": w.d, "nlist": w.nlist,
                   "block_vecs": w.block_vecs, "metric": w.metric, "query_batch": B, "nprobe": nprobe,
                   "k": k, "insert_batch": ib, "search_streams": args.search_streams, "seed": w.seed,
                   # what was measured on: the first MiB of the base set, and the hardware queues asked for
                   "base_sha256_first_mib": hashlib.sha256(w.base.tobytes()[:1 << 20]).hexdigest()[:16],
                   "numpy": np.__version__,
                   "gpu_max_hw_queues": os.environ.get("GPU_MAX_HW_QUEUES", "runtime default (4)")},
        "roofline": {"bound": "hbm", "kernel": "k_scan", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "bytes_per_launch": union_b, "pair_bytes_per_launch": pair_b,
                     "avg_launch_ms": scan_avg_ms, "launches_timed": scan_n,
                     "alu_issue": {"lane_instructions_per_launch": lane_ops,
                                   "achieved_T_per_s": lane_ops / (scan_avg_ms * 1e-3) / 1e12 if scan_n else None,
                                   "peak_T_per_s": VALU_ISSUE_PEAK_T,
                                   "frac": lane_ops / (scan_avg_ms * 1e-3) / 1e12 / VALU_ISSUE_PEAK_T if scan_n else None}},
        "inserts_per_s_in_step": args.steps * ib / elapsed,
        "bulk_load_vectors_per_s": len(w.base) / bulk_s,
    }

    if not args.no_extras:
        result.update(extras(args, g, w, torch, rtams, q_batches, queries, ins_batches, data_stream,
                             search_streams, dev))
        if args.cpu_queries > 0:
            result["cpu_baseline"] = cpu_baseline(args, w)
    print(json.dumps(result))
    g.close()
    return 0


def measured_traffic(workload: str, batch: int):
    """HBM bytes per scan launch from the committed profiler summary of this
    workload (FETCH_SIZE + WRITE_SIZE, scaled by the copy-kernel yardstick), or None."""
    path = os.path.join(ROOT, "profiles", f"k_scan_{workload}_batch{batch}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def extras(args, g, w, torch, rtams, q_batches, queries, ins_batches, data_stream, search_streams, dev):
    """Latency of one search request (closed loop, one in flight) with and
    without the insertion stream running at the configured rate; saturated
    insertion rate."""
    k, nprobe, ib = w.k, w.nprobe, w.insert_batch
    s = search_streams[0]
    out = {}

    def latencies(bs, iters, timed_scan=False):
        od = torch.empty((bs, k), dtype=torch.float32, device=dev)
        oi = torch.empty((bs, k), dtype=torch.int64, device=dev)
        lat = []
        nb = len(queries) // bs
        if timed_scan:
            g.scan_time(reset=True)
            g.set_param("profile_scan", 1)
        for i in range(iters + 10):
            q = queries[(i % nb) * bs:(i % nb + 1) * bs]
            t0 = time.perf_counter()
            g.search(q, k, nprobe, od, oi, stream=s)
            s.synchronize()
            if i >= 10:
                lat.append((time.perf_counter() - t0) * 1e3)
        if timed_scan:
            g.set_param("profile_scan", 0)
            ms, cnt = g.scan_time(reset=True)
            return lat, ms / max(cnt, 1)
        return lat

    def union_bytes(bs, batches):
        sizes = g.list_sizes()
        nb = len(queries) // bs
        tot = []
        for i in range(batches):
            pl = g.probe(queries[(i % nb) * bs:(i % nb + 1) * bs], nprobe).cpu().numpy()
            ln = sizes[np.unique(pl)]
            tot.append(int((ln * w.d * 4 + ((ln + w.block_vecs - 1) // w.block_vecs) * 4).sum()))
        return float(np.mean(tot))

    rate = 10_000.0  # vectors per second of the configured insertion stream
    stop = threading.Event()
    sent = [0]

    def inserter():
        period = ib / rate
        nxt = time.perf_counter()
        i = 0
        while not stop.is_set():
            g.add(ins_batches[i % len(ins_batches)], stream=data_stream)
            i += 1
            sent[0] += ib
            nxt += period
            dt = nxt - time.perf_counter()
            if dt > 0:
                time.sleep(dt)

    per_batch = {}
    for bs in (1, 32, 256):
        iters = args.latency_iters
        alone = latencies(bs, iters)
        _, scan_ms = latencies(bs, max(iters // 3, 20), timed_scan=True)  # the timing events cost a few microseconds
        ub = union_bytes(bs, min(iters, 64))
        stop.clear()
        sent[0] = 0
        th = threading.Thread(target=inserter)
        t0 = time.perf_counter()
        th.start()
        loaded = latencies(bs, iters)
        stop.set()
        th.join()
        data_stream.synchronize()
        dt = time.perf_counter() - t0
        per_batch[str(bs)] = {
            "search_only": {"qps": bs / (np.mean(alone) * 1e-3), "p50_ms": percentile(alone, 50),
                            "p99_ms": percentile(alone, 99)},
            "with_inserts": {"qps": bs / (np.mean(loaded) * 1e-3), "p50_ms": percentile(loaded, 50),
                             "p99_ms": percentile(loaded, 99), "inserts_per_s": sent[0] / dt},
            "p99_ratio": percentile(loaded, 99) / percentile(alone, 99),
            # list scan of one request running alone: union bytes of the probed lists over its duration
            "scan": {"avg_launch_ms": scan_ms, "bytes_per_launch": ub,
                     "achieved_GBps": ub / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else None,
                     "frac_of_hbm_peak": ub / (scan_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if scan_ms > 0 else None},
        }
    out["latency_by_query_batch"] = per_batch

    # the configuration's own mix: closed-loop searches of the benchmark's batch on all search streams while
    # the insertion thread keeps its 10,000 vectors/s (the timed steps insert 64 vectors per search batch,
    # about 40 times that rate)
    B = args.batch
    nb = len(queries) // B
    outs = [(torch.empty((B, k), dtype=torch.float32, device=dev), torch.empty((B, k), dtype=torch.int64, device=dev))
            for _ in search_streams]
    stop.clear()
    sent[0] = 0
    th = threading.Thread(target=inserter)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    th.start()
    n_req = 4000
    for i in range(n_req):
        si = i % len(search_streams)
        while True:
            try:
                g.search(queries[(i % nb) * B:(i % nb + 1) * B], k, nprobe, outs[si][0], outs[si][1],
                         stream=search_streams[si])
                break
            except rtams.RtamsError as e:
                if e.code != rtams.EBUSY:
                    raise
                search_streams[(si + 1) % len(search_streams)].synchronize()
    for st_ in search_streams:
        st_.synchronize()
    dt = time.perf_counter() - t0
    stop.set()
    th.join()
    data_stream.synchronize()
    out["at_configured_insert_rate"] = {"qps": n_req * B / dt, "query_batch": B, "search_streams": len(search_streams),
                                        "inserts_per_s": sent[0] / dt}

    # practical ceiling of a streaming read on this chip: the library's plain read kernel over 1 GiB
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).zero_()
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    for _ in range(3):
        rtams.read_plain(src, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        rtams.read_plain(src, sink)
    e1.record()
    torch.cuda.synchronize()
    out["plain_read_GBps"] = 10 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src

    # saturated insertion: batches back to back on the data stream
    torch.cuda.synchronize()
    n = 300
    t0 = time.perf_counter()
    for i in range(n):
        g.add(ins_batches[i % len(ins_batches)], stream=data_stream)
    data_stream.synchronize()
    out["inserts_per_s_saturated"] = n * ib / (time.perf_counter() - t0)
    st = g.pool_stats()
    out["pool"] = {"blocks_in_use": st.blocks_in_use, "blocks_total": st.blocks_total,
                   "utilisation": st.utilisation, "ntotal": st.ntotal}
    return out


def cpu_baseline(args, w):
    """The CPU oracle, as it stands, on the host cores of this machine: the same
    index (built by the oracle itself) and a bounded sample of the queries."""
    from oracle import oracle as orc
    o = orc.OracleIndex(w.d, w.nlist, w.metric, w.block_vecs,
                        pool_blocks=len(w.base) // w.block_vecs + 2 * w.nlist + 64)
    o.set_centroids(w.centroids)
    t0 = time.perf_counter()
    o.add(w.base)
    t_add = time.perf_counter() - t0
    n = min(args.cpu_queries, len(w.queries))
    t0 = time.perf_counter()
    o.search(w.queries[:n], w.k, w.nprobe)
    t_search = time.perf_counter() - t0
    return {"value": n / t_search, "unit": "queries/s", "cores": orc.threads(), "kind": "oracle",
            "sample": f"first {n} queries of the workload against the full {len(w.base)}-vector index, "
                      f"nprobe {w.nprobe}, k {w.k}; search only ({t_search:.1f} s)",
            "bulk_load_vectors_per_s": len(w.base) / t_add}


if __name__ == "__main__":
    sys.exit(main())
