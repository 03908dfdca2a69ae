#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: one
insertion batch on the data stream (assignment, slot reservation, block
opening, fill, publication, and the rearrangement rounds Exceed() asks for)
and, concurrently, one search batch on a pooled search stream (coarse scores,
probe selection, list scan, top-k).  Every input is resident in HBM before the
timed region starts.

The default workload is the largest configuration: skewed growth (L2, d = 256,
20 M base vectors whose lists follow a Zipf(1.1) law over 16,384 lists, blocks
of 256 vectors, nprobe 64, k 50, query batch 256, inserts in batches of 1024
with the rearrangement threshold armed, 7 search streams and the data stream).
`--config 3`, `--config 4` and `--config 2` run the inner-product and the
byte-valued configurations the same way; the default run also carries a short block for
configuration 2.

Prints ONE JSON line on stdout (progress lines go to stderr).  `value` is
queries per second over the timed steps; `roofline` is for the list scan (bytes
of the union of the probed lists per launch over the launch's mean duration,
measured with HIP events on the caller's stream, against 8 TB/s; `alu_issue` is
the arithmetic side of the same launches); `cpu_baseline` is the CPU oracle on
the host cores.
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

# What each configuration prescribes beyond the data: query batch, search streams beside the data
# stream, rate of the insert stream in vectors per second, rearrangement threshold (the smallest of
# the paper's rearrangement table for the skewed configuration), batch sizes of the latency table.
PROTOCOL = {
    2: {"batch": 256, "search_streams": 4, "insert_rate": 10_000.0, "threshold": 0, "latency_batches": (1, 32, 256)},
    3: {"batch": 128, "search_streams": 4, "insert_rate": 50_000.0, "threshold": 0, "latency_batches": (1, 128)},
    # (the configuration's own protocol, open-loop mixed load, is `--study mixed`; here its largest query batch in
    # closed loop beside 30 % of its highest offered rate of 50,000 operations/s as inserts)
    4: {"batch": 64, "search_streams": 7, "insert_rate": 15_000.0, "threshold": 0, "latency_batches": (1, 64)},
    5: {"batch": 256, "search_streams": 7, "insert_rate": 100_000.0, "threshold": 10_000, "latency_batches": (1, 256)},
}
T_START = time.perf_counter()


def note(msg: str) -> None:
    print(f"[bench +{time.perf_counter() - T_START:6.1f}s] {msg}", file=sys.stderr, flush=True)


# queries the CPU oracle answers for `cpu_baseline`: 5-15 s of work on the box's 16 cores (measured: 1,900
# queries/s on configuration 2, 50 on configuration 5)
CPU_SAMPLE_QUERIES = {2: 8192, 3: 512, 4: 512, 5: 768}


def percentile(xs, p):
    return float(np.percentile(np.asarray(xs, dtype=np.float64), p)) if len(xs) else float("nan")


class Bench:
    """One configuration loaded into an index, with the streams its protocol names."""

    def __init__(self, torch, rtams, synth, idx: int, scale: float, batch: int, search_streams: int):
        self.torch, self.rtams, self.idx = torch, rtams, idx
        self.dev = dev = torch.device("cuda:0")
        proto = PROTOCOL[idx]
        note(f"configuration {idx}: drawing the set on the host")
        t0 = time.perf_counter()
        self.w = w = synth.config(idx, scale=scale)
        self.host_generation_s = time.perf_counter() - t0
        self.B = batch or proto["batch"]
        self.k, self.nprobe, self.ib = w.k, w.nprobe, w.insert_batch
        self.rate = proto["insert_rate"]
        n_streams = search_streams or proto["search_streams"]
        to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        cents, self.queries, inserts = map(to_dev, (w.centroids, w.queries, w.inserts))
        # room for the base set, the insert stream of every phase below, and spare blocks for rearrangement
        n_all = len(w.base) + 4 * len(w.inserts) + 2_000_000
        pool_blocks = n_all // w.block_vecs + 3 * w.nlist + 8192
        # candidates a query may have: a few times the average; under the Zipf law a quarter of everything
        # (most queries of a batch may probe the longest list, which holds a seventh of the vectors)
        cand = max(65536, 4 * w.nprobe * (len(w.base) // w.nlist + w.block_vecs))
        if idx == 5:
            cand = max(cand, len(w.base) // 4)
        if idx == 2:
            cand = 65536
        self.g = g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=pool_blocks,
                                 rearrange_threshold=proto["threshold"], n_resources=max(8, n_streams + 1),
                                 max_batch=max(self.B, 256), max_k=128, max_nprobe=64, max_add_batch=65536,
                                 candidates_per_query=cand)
        self.data_stream = torch.cuda.Stream(dev)
        self.search_streams = [torch.cuda.Stream(dev) for _ in range(n_streams)]
        g.set_centroids(cents, stream=self.data_stream)
        note(f"configuration {idx}: bulk load of {len(w.base)} vectors through add")
        # bulk load of the base set through add (one format for offline and online data), in pieces so
        # that the set need not sit in HBM twice; only the add calls are timed
        bulk_s = 0.0
        for lo in range(0, len(w.base), 1 << 22):
            part = to_dev(w.base[lo:lo + (1 << 22)])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g.add(part, stream=self.data_stream)
            torch.cuda.synchronize()
            bulk_s += time.perf_counter() - t0
            del part
        self.bulk_s = bulk_s
        self.rearrange_after_load_s = None
        if proto["threshold"] > 0:
            # the offline segment of the paper is contiguous: every list the bulk load left exceeding is
            # rearranged before the online phase, which then rearranges what ITS inserts make exceed
            note(f"configuration {idx}: rearranging the lists the bulk load left exceeding")
            t0 = time.perf_counter()
            g.rearrange(-1, stream=self.data_stream)
            self.data_stream.synchronize()
            self.rearrange_after_load_s = time.perf_counter() - t0
        B, ib = self.B, self.ib
        self.nq_batches = len(w.queries) // B
        self.q_batches = [self.queries[i * B:(i + 1) * B] for i in range(self.nq_batches)]
        self.n_ins_batches = len(w.inserts) // ib
        self.ins_batches = [inserts[i * ib:(i + 1) * ib] for i in range(self.n_ins_batches)]
        self.outs = [(torch.empty((B, self.k), dtype=torch.float32, device=dev),
                      torch.empty((B, self.k), dtype=torch.int64, device=dev)) for _ in self.search_streams]
        self.ins_cursor = 0

    def next_insert(self):
        b = self.ins_batches[self.ins_cursor % self.n_ins_batches]
        self.ins_cursor += 1
        return b

    def submit_search(self, i, q, outs=None):
        outs = outs or self.outs
        s = i % len(self.search_streams)
        while True:
            try:
                self.g.search(q, self.k, self.nprobe, outs[s][0], outs[s][1], stream=self.search_streams[s])
                return
            except self.rtams.RtamsError as e:
                if e.code != self.rtams.EBUSY:
                    raise
                self.search_streams[(s + 1) % len(self.search_streams)].synchronize()

    def step(self, i):
        self.g.add(self.next_insert(), stream=self.data_stream)
        self.submit_search(i, self.q_batches[i % self.nq_batches])

    def timed_steps(self, steps, warmup):
        torch, g = self.torch, self.g
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        g.scan_time(reset=True)
        g.scan_kernels(reset=True)
        g.set_param("profile_scan", 1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(warmup + i)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        g.set_param("profile_scan", 0)
        scan_ms, scan_n = g.scan_time(reset=True)
        by_kernel = g.scan_kernels(reset=True)  # which scan kernel the library chose for these requests
        self.scan_kernel = max(by_kernel, key=by_kernel.get)
        assert g.poll_error() == 0, "a kernel raised an error during the timed steps"
        return elapsed, scan_ms, scan_n

    def scan_scheduling(self, steps, warmup, union_b):
        """The same timed steps with the scans of different requests made to run one after the other,
        and left to overlap: the library queues them up only when they are long, and a scan that
        shares the chip with another one takes longer without being any less efficient, so the
        per-launch duration (and with it `roofline.frac`) reads differently in the two modes."""
        g, out = self.g, {}
        for name, (pairs, nbytes) in (("one_at_a_time", (1, 1)), ("overlapping", (0, 1))):
            g.set_param("scan_exclusive_pairs", pairs)
            g.set_param("scan_exclusive_bytes", nbytes)
            e, ms, n = self.timed_steps(steps, warmup)
            avg = ms / max(n, 1)
            out[name] = {"qps": steps * self.B / e, "ms_per_step": e / steps * 1e3, "scan_avg_launch_ms": avg,
                         "scan_frac_of_hbm_peak": union_b / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS if n else None}
        g.set_param("scan_exclusive_pairs", 4096)  # the library's defaults
        g.set_param("scan_exclusive_bytes", 16 << 30)
        return out

    def scan_bytes(self, batches, bs=None, first=0):
        """Algorithmic bytes of the scan per launch: what the method must read.  The scan reads a list
        once for all the queries of the batch that probe it, so these are the bytes of the UNION of
        the probed lists; bytes counted once per (query, list) pair are reported beside them, never
        credited."""
        w, g = self.w, self.g
        bs = bs or self.B
        nb = max(len(self.queries) // bs, 1)
        sizes = g.list_sizes()
        per_list = lambda l: l * w.d * 4 + ((l + w.block_vecs - 1) // w.block_vecs) * 4
        pair_bytes, union_bytes = [], []
        for i in range(batches):
            b = (first + i) % nb
            pl = g.probe(self.queries[b * bs:(b + 1) * bs], self.nprobe).cpu().numpy()
            pair_bytes.append(int(per_list(sizes[pl]).sum()))
            union_bytes.append(int(per_list(sizes[np.unique(pl)]).sum()))
        return float(np.mean(pair_bytes)), float(np.mean(union_bytes))

    def roofline(self, scan_ms, scan_n, pair_b, union_b, traffic):
        """Arithmetic of the same launch: every (query, candidate) pair costs d subtract + d fused
        multiply-add instructions per lane for L2 (d multiply-adds for IP); the yardstick is the rate at
        which 256 CUs x 4 SIMDs x 16 lanes issue one fp32 instruction per lane and clock at 2.4 GHz."""
        w = self.w
        pair_vecs = pair_b / (w.d * 4 + 4.0 / w.block_vecs)
        lane_ops = pair_vecs * w.d * (2 if w.metric == "l2" else 1)
        scan_avg_ms = scan_ms / max(scan_n, 1)
        achieved = union_b / (scan_avg_ms * 1e-3) / 1e9 if scan_n else float("nan")
        return {"bound": "hbm", "kernel": self.scan_kernel, "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "bytes_per_launch": union_b, "pair_bytes_per_launch": pair_b,
                "avg_launch_ms": scan_avg_ms, "launches_timed": scan_n,
                # what the direct form of the same launch costs on the vector unit (the matrix-core scan does not pay it)
                "alu_issue": {"lane_instructions_per_launch": lane_ops,
                              "achieved_T_per_s": lane_ops / (scan_avg_ms * 1e-3) / 1e12 if scan_n else None,
                              "peak_T_per_s": VALU_ISSUE_PEAK_T,
                              "frac": lane_ops / (scan_avg_ms * 1e-3) / 1e12 / VALU_ISSUE_PEAK_T if scan_n else None}}

    def config_block(self):
        w = self.w
        return {"workload": w.name, "n_base": len(w.base), "d": w.d, "nlist": w.nlist,
                "block_vecs": w.block_vecs, "metric": w.metric, "query_batch": self.B, "nprobe": self.nprobe,
                "k": self.k, "insert_batch": self.ib, "search_streams": len(self.search_streams),
                "configured_insert_rate": self.rate, "rearrange_threshold": PROTOCOL[self.idx]["threshold"],
                "seed": w.seed,
                # what was measured on: the first MiB of the base set, and the hardware queues asked for
                "base_sha256_first_mib": hashlib.sha256(w.base[:max(1, (1 << 20) // (4 * w.d))].tobytes()).hexdigest()[:16],
                "numpy": np.__version__,
                "gpu_max_hw_queues": os.environ.get("GPU_MAX_HW_QUEUES", "runtime default (4)")}

    # ---- latency of one request, alone and beside the insert stream at the configured rate
    def latencies(self, bs, iters, stream, timed_scan=False):
        torch, g = self.torch, self.g
        od = torch.empty((bs, self.k), dtype=torch.float32, device=self.dev)
        oi = torch.empty((bs, self.k), dtype=torch.int64, device=self.dev)
        lat = []
        nb = max(len(self.queries) // bs, 1)
        if timed_scan:
            g.scan_time(reset=True)
            g.set_param("profile_scan", 1)
        for i in range(iters + 10):
            q = self.queries[(i % nb) * bs:(i % nb + 1) * bs]
            t0 = time.perf_counter()
            g.search(q, self.k, self.nprobe, od, oi, stream=stream)
            stream.synchronize()
            if i >= 10:
                lat.append((time.perf_counter() - t0) * 1e3)
        if timed_scan:
            g.set_param("profile_scan", 0)
            ms, cnt = g.scan_time(reset=True)
            return lat, ms / max(cnt, 1)
        return lat

    def inserter(self, stop, sent):
        """Paces insertion batches on the data stream at the configured rate until told to stop."""
        period = self.ib / self.rate
        nxt = time.perf_counter()
        while not stop.is_set():
            self.g.add(self.next_insert(), stream=self.data_stream)
            sent[0] += self.ib
            nxt += period
            dt = nxt - time.perf_counter()
            if dt > 0:
                time.sleep(dt)

    def latency_table(self, iters, batches):
        s = self.search_streams[0]
        per_batch = {}
        for bs in batches:
            note(f"configuration {self.idx}: latency of one request at batch {bs}, alone and beside the insert stream")
            alone = self.latencies(bs, iters, s)
            _, scan_ms = self.latencies(bs, max(iters // 3, 20), s, timed_scan=True)  # the timing events cost a few microseconds
            _, ub = self.scan_bytes(min(iters, 32), bs=bs)
            stop, sent = threading.Event(), [0]
            th = threading.Thread(target=self.inserter, args=(stop, sent))
            t0 = time.perf_counter()
            th.start()
            loaded = self.latencies(bs, iters, s)
            stop.set()
            th.join()
            self.data_stream.synchronize()
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
        return per_batch

    def at_configured_rate(self, n_req):
        """The configuration's own mix: closed-loop searches of the benchmark's batch on all search
        streams while the insertion thread keeps the configured rate."""
        torch = self.torch
        stop, sent = threading.Event(), [0]
        th = threading.Thread(target=self.inserter, args=(stop, sent))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        th.start()
        for i in range(n_req):
            self.submit_search(i, self.q_batches[i % self.nq_batches])
        for st_ in self.search_streams:
            st_.synchronize()
        dt = time.perf_counter() - t0
        stop.set()
        th.join()
        self.data_stream.synchronize()
        return {"qps": n_req * self.B / dt, "query_batch": self.B, "search_streams": len(self.search_streams),
                "inserts_per_s": sent[0] / dt, "requests": n_req}

    def saturated_inserts(self, n):
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            self.g.add(self.next_insert(), stream=self.data_stream)
        self.data_stream.synchronize()
        return n * self.ib / (time.perf_counter() - t0)

    def close(self):
        self.g.close()


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


def plain_read_rate(torch, rtams, dev):
    """Practical ceiling of a streaming read on this chip: the library's plain read kernel over 1 GiB."""
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
    return 10 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9


def cpu_baseline(b: Bench, n_queries: int):
    """The CPU oracle, as it stands, on the host cores of this machine: the same index (built by the oracle
    itself; for the skewed configuration from the list every vector was drawn for, which is its
    nearest centroid by construction and saves the oracle's assignment pass of an hour) and a bounded
    sample of the queries."""
    from oracle import oracle as orc
    w = b.w
    o = orc.OracleIndex(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=len(w.base) // w.block_vecs + 2 * w.nlist + 64)
    o.set_centroids(w.centroids)
    assign = w.extra["base_component"].astype(np.int32) if "base_component" in w.extra else None
    if assign is None and len(w.base) * w.nlist * w.d > 2e12:
        return {"value": None, "unit": "queries/s", "cores": orc.threads(), "kind": "oracle",
                "sample": "skipped: the oracle's assignment pass over this base set takes more than ten minutes"}
    note(f"configuration {b.idx}: the oracle builds the index on {orc.threads()} host threads")
    t0 = time.perf_counter()
    o.add(w.base, assign=assign)
    t_add = time.perf_counter() - t0
    n = min(n_queries, len(w.queries))
    note(f"configuration {b.idx}: the oracle answers {n} queries")
    t0 = time.perf_counter()
    o.search(w.queries[:n], w.k, w.nprobe)
    t_search = time.perf_counter() - t0
    out = {"value": n / t_search, "unit": "queries/s", "cores": orc.threads(), "kind": "oracle",
           "sample": f"first {n} queries of the workload against the full {len(w.base)}-vector index, "
                     f"nprobe {w.nprobe}, k {w.k}; search only ({t_search:.1f} s)"}
    if assign is None:
        out["bulk_load_vectors_per_s"] = len(w.base) / t_add
    else:
        out["index_build_s_with_given_lists"] = t_add
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, choices=sorted(PROTOCOL),
                    help="benchmark configuration: 5 skewed growth (default), 4 wide inner product, 3 inner product, 2 byte-valued")
    ap.add_argument("--batch", type=int, default=0, help="queries per search batch (default: the configuration's)")
    ap.add_argument("--scale", type=float, default=1.0, help="shrinks base/query/insert counts")
    ap.add_argument("--search-streams", type=int, default=0, help="default: the configuration's")
    ap.add_argument("--latency-iters", type=int, default=0, help="requests per latency figure (default 300, 2000 for configuration 2)")
    ap.add_argument("--cpu-queries", type=int, default=0, help="queries of the oracle sample (default: 768 for configuration 5, 512 for 3, 8192 for 2); -1 skips it")
    ap.add_argument("--no-extras", action="store_true", help="only the timed steps (for profiler runs)")
    ap.add_argument("--set", action="append", default=[], metavar="KEY=VALUE",
                    help="a launch-shape parameter of the library (rtams_set_param), e.g. scan_mfma=0; may be repeated")
    ap.add_argument("--no-config2", action="store_true", help="leave out the short block for configuration 2")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only the plain copy kernel on 1 GiB (yardstick for the traffic counters)")
    ap.add_argument("--pq-m", type=int, default=0,
                    help="with --study pq: only this number of sub-spaces, and only the --batch query batch")
    ap.add_argument("--shape", type=int, default=0, help="with --study shapes: only this configuration (3, 4 or 5)")
    ap.add_argument("--study", choices=["rearrange", "rearrange5", "blocksize", "pq", "storage", "shapes", "mixed", "growth", "online"],
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
              "mixed": studies.mixed_load_study, "growth": studies.growth_study,
              "rearrange5": studies.hot_list_rearrangement_study, "online": studies.online_latency_study}[args.study]
        iters = args.latency_iters or 2000
        if args.study == "pq":
            params = {k: int(v) for k, v in (kv.split("=") for kv in args.set)}
            if args.pq_m:
                print(json.dumps(fn(scale=args.scale, iters=iters, ms=(args.pq_m,), batches=(args.batch or 256,), params=params)))
            else:
                print(json.dumps(fn(scale=args.scale, iters=iters, params=params)))
            return 0
        if args.study == "shapes" and args.shape:
            print(json.dumps(fn(scale=args.scale, iters=iters, which=(args.shape,))))
            return 0
        print(json.dumps(fn(scale=args.scale, iters=iters)))
        return 0

    b = Bench(torch, rtams, synth, args.config, args.scale, args.batch, args.search_streams)
    w = b.w
    params = {k: int(v) for k, v in (kv.split("=") for kv in args.set)}
    for key, value in params.items():
        b.g.set_param(key, value)
    note(f"configuration {args.config}: {args.warmup} warm-up and {args.steps} timed steps")
    elapsed, scan_ms, scan_n = b.timed_steps(args.steps, args.warmup)
    qps = args.steps * b.B / elapsed
    pair_b, union_b = b.scan_bytes(min(args.steps, b.nq_batches, 32), first=args.warmup)
    result = {
        "metric": "search QPS under concurrent insertion",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": b.config_block(),
        "roofline": b.roofline(scan_ms, scan_n, pair_b, union_b, measured_traffic(w.name, b.B)),
        "inserts_per_s_in_step": args.steps * b.ib / elapsed,
        "bulk_load_vectors_per_s": len(w.base) / b.bulk_s,
        "host_generation_s": b.host_generation_s,
        "rearrange_after_bulk_load_s": b.rearrange_after_load_s,
    }
    if params:
        result["config"]["library_parameters"] = params
    if not args.no_extras:
        big = args.config != 2
        iters = args.latency_iters or (300 if big else 2000)
        if not params:
            result["scan_scheduling"] = b.scan_scheduling(args.steps, args.warmup, union_b)
        result["latency_by_query_batch"] = b.latency_table(iters, PROTOCOL[args.config]["latency_batches"])
        note(f"configuration {args.config}: closed-loop searches on every stream beside the insert stream")
        result["at_configured_insert_rate"] = b.at_configured_rate(400 if big else 4000)
        result["plain_read_GBps"] = plain_read_rate(torch, rtams, dev)
        result["inserts_per_s_saturated"] = b.saturated_inserts(100 if big else 300)
        b.g.rearrange(-1, stream=b.data_stream)  # the rounds the last batches asked for
        b.data_stream.synchronize()
        b.g.validate()
        st = b.g.pool_stats()
        result["pool"] = {"blocks_in_use": st.blocks_in_use, "blocks_total": st.blocks_total,
                          "utilisation": st.utilisation, "ntotal": st.ntotal, "lists_exceeding": st.lists_exceeding,
                          "add_waits": st.add_waits}
        assert b.g.poll_error() == 0, "a kernel raised an error"
    b.close()
    if not args.no_extras and args.cpu_queries >= 0:
        result["cpu_baseline"] = cpu_baseline(b, args.cpu_queries or CPU_SAMPLE_QUERIES[args.config])
    del b
    torch.cuda.empty_cache()

    if args.config != 2 and not args.no_extras and not args.no_config2:
        # the byte-valued configuration (1 M x 128, half of it fits the last-level cache), kept beside the headline
        b2 = Bench(torch, rtams, synth, 2, args.scale, 0, 0)
        note("configuration 2: timed steps")
        e2, ms2, n2 = b2.timed_steps(200, 20)
        p2, u2 = b2.scan_bytes(32, first=20)
        block = {"config": b2.config_block(), "value": 200 * b2.B / e2, "unit": "queries/s",
                 "ms_per_step": e2 / 200 * 1e3,
                 "roofline": b2.roofline(ms2, n2, p2, u2, measured_traffic(b2.w.name, b2.B)),
                 "scan_scheduling": b2.scan_scheduling(200, 20, u2),
                 "latency_by_query_batch": b2.latency_table(args.latency_iters or 1000, PROTOCOL[2]["latency_batches"]),
                 "at_configured_insert_rate": b2.at_configured_rate(2000),
                 "inserts_per_s_saturated": b2.saturated_inserts(300),
                 "bulk_load_vectors_per_s": len(b2.w.base) / b2.bulk_s}
        b2.close()
        if args.cpu_queries >= 0:
            block["cpu_baseline"] = cpu_baseline(b2, CPU_SAMPLE_QUERIES[2])
        result["configuration_2"] = block
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
