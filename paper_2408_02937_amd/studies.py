"""Two measured studies on one GPU, run through `bench.py --study ...`.

* `rearrangement_study`: the analogue of the paper's rearrangement table
  (Memory Rearrangement, "Experiments on memory rearrangement"): every online
  vector goes to one list until it holds T_m' of them; search latency before,
  the cost of rearranging that list, search latency after, and what searches
  see while the rearrangement runs.
* `hot_list_rearrangement_study`: the same table on the skewed configuration's
  hottest list (millions of vectors), grown by 10,000 / 50,000 / 100,000 online
  vectors.
* `block_size_sweep`: the analogue of the paper's block-size figure ("Effects
  of memory block size"): latency, scan rate and pad memory as T_m grows.

* `pq_study`: product-quantised lists (the IVF-PQ kind of list the paper names
  beside IVF-Flat) in the same blocks: load rate, bytes per vector, latency
  and scan time per query batch, insertion latency, and how many of the flat
  index's top-k the coded index returns.

* `shape_study`: configurations 3, 4 and 5 (other dimensions, metrics, list
  counts, block sizes and batch sizes) at a fraction of their base sets: load
  rate, latency per request at the configuration's batch, scan time and bytes.

* `mixed_load_study`: configuration 4's protocol: an open-loop stream of
  operations (70 % queries, 30 % inserted vectors) offered at fixed rates, 7
  search streams and the data stream; latency from arrival to completion.

* `growth_study`: configuration 5's protocol: Zipf-distributed inserts at a
  fixed rate with Exceed() armed, so rearrangement rounds run between the
  insertion batches while searches run beside them; latency second by second.

The first three use configuration 2's synthetic data (byte-valued, d = 128, 1 M vectors,
1024 lists) and go through the same C ABI as everything else.
"""
from __future__ import annotations

import threading
import time

import numpy as np
import torch

from . import rtams, synth


LDS_LOOKUPS_PEAK_G = 256 * 128 / 4 * 2.4  # 4-byte LDS reads per nanosecond of the whole chip, conflict-free
VALU_ISSUE_PEAK_T = 256 * 64 * 2.4e9 / 1e12  # unpacked fp32 lane instructions per second, all CUs


def _p(xs, q):
    return float(np.percentile(np.asarray(xs, dtype=np.float64), q)) if len(xs) else float("nan")


def _to_dev(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def _search_latencies(g, queries, bs, k, nprobe, iters, stream, dev):
    od = torch.empty((bs, k), dtype=torch.float32, device=dev)
    oi = torch.empty((bs, k), dtype=torch.int64, device=dev)
    nb = max(len(queries) // bs, 1)
    lat = []
    for i in range(iters + 10):
        q = queries[(i % nb) * bs:(i % nb) * bs + bs]
        t0 = time.perf_counter()
        g.search(q, k, nprobe, od, oi, stream=stream)
        stream.synchronize()
        if i >= 10:
            lat.append((time.perf_counter() - t0) * 1e3)
    return lat


def rearrangement_study(scale: float = 1.0, thresholds=(10_000, 50_000, 100_000), iters: int = 200) -> dict:
    dev = torch.device("cuda:0")
    w = synth.config(2, scale=scale)
    rng = np.random.Generator(np.random.PCG64([w.seed, 77]))
    base, cents, inserts = (_to_dev(a, dev) for a in (w.base, w.centroids, w.inserts))
    hot = 17 % w.nlist
    rows = []
    for thr in thresholds:
        n_hot = thr + 1  # Exceed() is strict: T_m' vectors do not trigger, one more does
        # vectors of the hot list: its centroid plus small integer noise (kept byte-valued)
        hv = np.clip(np.rint(w.centroids[hot][None, :] + 2.0 * rng.standard_normal((n_hot, w.d))), 0, 255)
        hv = _to_dev(hv.astype(np.float32), dev)
        n_all = len(w.base) + n_hot + len(w.inserts)
        spare = 2 * (n_hot // w.block_vecs + 2)
        g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs,
                        pool_blocks=n_all // w.block_vecs + 2 * w.nlist + spare + 64, n_resources=8,
                        max_batch=256, max_k=128, max_nprobe=64, max_add_batch=65536, candidates_per_query=262144)
        ds, ss, s2 = torch.cuda.Stream(dev), torch.cuda.Stream(dev), torch.cuda.Stream(dev)
        g.set_centroids(cents, stream=ds)
        g.add(base, stream=ds)
        ds.synchronize()
        assigned = g.assign(hv[:4096]).cpu().numpy()
        on_hot = float((assigned == hot).mean())
        # online phase: a batch into the hot list, a batch of ordinary traffic, in turn
        ib = w.insert_batch
        t0 = time.perf_counter()
        j = 0
        for o in range(0, n_hot, ib):
            g.add(hv[o:o + ib], stream=ds)
            g.add(inserts[(j % (len(inserts) // ib)) * ib:(j % (len(inserts) // ib)) * ib + ib], stream=ds)
            j += 1
        ds.synchronize()
        t_online = time.perf_counter() - t0
        blocks, runs_before, online = g.list_info(hot)
        qh = hv[:2000]
        before = {bs: _search_latencies(g, qh, bs, w.k, w.nprobe, iters, ss, dev) for bs in (1, 10)}

        # searches that run while the list is rearranged
        during, stop = [], threading.Event()

        def searcher():
            od = torch.empty((10, w.k), dtype=torch.float32, device=dev)
            oi = torch.empty((10, w.k), dtype=torch.int64, device=dev)
            i = 0
            while not stop.is_set():
                t = time.perf_counter()
                g.search(qh[(i % 100) * 10:(i % 100) * 10 + 10], w.k, w.nprobe, od, oi, stream=s2)
                s2.synchronize()
                during.append((t, (time.perf_counter() - t) * 1e3))
                i += 1

        g.rearrange((hot + 1) % w.nlist, stream=ds)  # one-time set-up cost of the first call stays out of the timing
        ds.synchronize()
        th = threading.Thread(target=searcher)
        th.start()
        time.sleep(0.05)
        t0 = time.perf_counter()
        g.rearrange(hot, stream=ds)
        ds.synchronize()
        t1 = time.perf_counter()
        time.sleep(0.02)
        stop.set()
        th.join()
        cost_ms = (t1 - t0) * 1e3
        overl = [l for (t, l) in during if t + l * 1e-3 >= t0 and t <= t1]
        quiet = [l for (t, l) in during if t + l * 1e-3 < t0]
        _, runs_after, _ = g.list_info(hot)
        after = {bs: _search_latencies(g, qh, bs, w.k, w.nprobe, iters, ss, dev) for bs in (1, 10)}
        g.validate()
        assert g.poll_error() == 0
        rows.append({
            "threshold": thr, "hot_list": hot, "hot_list_len": int(g.list_sizes()[hot]), "blocks": int(blocks),
            "share_of_online_vectors_on_hot_list": on_hot, "online_phase_s": t_online,
            "runs_before": int(runs_before), "runs_after": int(runs_after),
            "rearrange_cost_ms": cost_ms,
            "latency_ms": {str(bs): {"before_p50": _p(before[bs], 50), "before_p99": _p(before[bs], 99),
                                     "after_p50": _p(after[bs], 50), "after_p99": _p(after[bs], 99)}
                           for bs in (1, 10)},
            "searches_during_rearrangement": {"count": len(overl), "max_ms": max(overl) if overl else None,
                                              "quiet_p50_ms": _p(quiet, 50), "quiet_max_ms": max(quiet) if quiet else None},
        })
        g.close()
    return {"study": "rearrangement", "workload": w.name, "block_vecs": w.block_vecs, "rows": rows}


def hot_list_rearrangement_study(scale: float = 1.0, thresholds=(10_000, 50_000, 100_000), iters: int = 100) -> dict:
    """The paper's rearrangement table on the skewed configuration (20 M x 256 under a Zipf(1.1) law): T_m' + 1
    online vectors all go to the HOTTEST list (millions of vectors, thousands of blocks, made contiguous
    after the bulk load), in batches of 1024 that alternate with batches of ordinary traffic so that the
    list's new blocks interleave with other lists'.  Search latency (queries that probe the hot list;
    batches of 1, 10 and 256) before, the wall time of rearranging the list while a searcher runs beside
    it, latency after.  One index for all thresholds: the hot list keeps growing."""
    dev = torch.device("cuda:0")
    w = synth.config(5, scale=scale)
    rng = np.random.Generator(np.random.PCG64([w.seed, 78]))
    cents, inserts = (_to_dev(a, dev) for a in (w.centroids, w.inserts))
    n_online = sum(t + 1 for t in thresholds)
    n_all = len(w.base) + 2 * n_online + 64 * w.insert_batch
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=n_all // w.block_vecs + 3 * w.nlist + 8192,
                    n_resources=8, max_batch=256, max_k=64, max_nprobe=64, max_add_batch=65536,
                    candidates_per_query=max(65536, (len(w.base) + 2 * n_online) // 4))
    ds, ss, s2 = torch.cuda.Stream(dev), torch.cuda.Stream(dev), torch.cuda.Stream(dev)
    g.set_centroids(cents, stream=ds)
    for lo in range(0, len(w.base), 1 << 22):
        part = _to_dev(w.base[lo:lo + (1 << 22)], dev)
        g.add(part, stream=ds)
        ds.synchronize()
        del part
    sizes = g.list_sizes()
    hot = int(sizes.argmax())
    t0 = time.perf_counter()
    g.rearrange(hot, stream=ds)  # the offline segment is contiguous
    ds.synchronize()
    first_ms = (time.perf_counter() - t0) * 1e3
    blocks0, runs0, _ = g.list_info(hot)
    rows = []
    ib = w.insert_batch
    j = 0
    for thr in thresholds:
        n_hot = thr + 1
        hv = _to_dev((w.centroids[hot][None, :] + 0.1 * rng.standard_normal((n_hot, w.d))).astype(np.float32), dev)
        on_hot = float((g.assign(hv[:4096]).cpu().numpy() == hot).mean())
        for o in range(0, n_hot, ib):  # a batch into the hot list, a batch of ordinary traffic, in turn
            g.add(hv[o:o + ib], stream=ds)
            g.add(inserts[(j % (len(inserts) // ib)) * ib:(j % (len(inserts) // ib)) * ib + ib], stream=ds)
            j += 1
        ds.synchronize()
        blocks, runs_before, _ = g.list_info(hot)
        qh = hv[:2560]
        batches = (1, 10, 256)
        before = {bs: _search_latencies(g, qh, bs, w.k, w.nprobe, iters, ss, dev) for bs in batches}
        during, stop = [], threading.Event()

        def searcher():
            od = torch.empty((10, w.k), dtype=torch.float32, device=dev)
            oi = torch.empty((10, w.k), dtype=torch.int64, device=dev)
            i = 0
            while not stop.is_set():
                t = time.perf_counter()
                g.search(qh[(i % 100) * 10:(i % 100) * 10 + 10], w.k, w.nprobe, od, oi, stream=s2)
                s2.synchronize()
                during.append((t, (time.perf_counter() - t) * 1e3))
                i += 1

        th = threading.Thread(target=searcher)
        th.start()
        time.sleep(0.05)
        t0 = time.perf_counter()
        g.rearrange(hot, stream=ds)
        ds.synchronize()
        t1 = time.perf_counter()
        time.sleep(0.02)
        stop.set()
        th.join()
        overl = [l for (t, l) in during if t + l * 1e-3 >= t0 and t <= t1]
        quiet = [l for (t, l) in during if t + l * 1e-3 < t0]
        _, runs_after, _ = g.list_info(hot)
        after = {bs: _search_latencies(g, qh, bs, w.k, w.nprobe, iters, ss, dev) for bs in batches}
        assert g.poll_error() == 0
        rows.append({
            "threshold": thr, "hot_list_len": int(g.list_sizes()[hot]), "blocks": int(blocks),
            "share_of_online_vectors_on_hot_list": on_hot,
            "runs_before": int(runs_before), "runs_after": int(runs_after),
            "rearrange_cost_ms": (t1 - t0) * 1e3,
            "latency_ms": {str(bs): {"before_p50": _p(before[bs], 50), "before_p99": _p(before[bs], 99),
                                     "after_p50": _p(after[bs], 50), "after_p99": _p(after[bs], 99)}
                           for bs in batches},
            "searches_during_rearrangement": {"count": len(overl), "max_ms": max(overl) if overl else None,
                                              "quiet_p50_ms": _p(quiet, 50), "quiet_max_ms": max(quiet) if quiet else None},
        })
    g.validate()
    st = g.pool_stats()
    out = {"study": "hot_list_rearrangement", "workload": w.name, "n_base": len(w.base), "block_vecs": w.block_vecs,
           "hot_list": hot, "hot_list_len_after_bulk_load": int(sizes[hot]), "hot_list_blocks_after_bulk_load": int(blocks0),
           "first_rearrangement_ms": first_ms, "runs_after_first_rearrangement": int(runs0),
           "blocks_in_use": st.blocks_in_use, "rows": rows}
    g.close()
    return out


def block_size_sweep(scale: float = 1.0, sizes=(64, 128, 256, 512, 1024, 2048), iters: int = 200) -> dict:
    dev = torch.device("cuda:0")
    w = synth.config(2, scale=scale)
    base, cents, queries, inserts = (_to_dev(a, dev) for a in (w.base, w.centroids, w.queries, w.inserts))
    rows = []
    for T in sizes:
        n_all = len(w.base) + 2 * len(w.inserts)
        g = rtams.Index(w.d, w.nlist, w.metric, T, pool_blocks=n_all // T + 2 * w.nlist + 64, n_resources=8,
                        max_batch=256, max_k=128, max_nprobe=64, max_add_batch=65536, candidates_per_query=65536)
        ds, ss = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
        g.set_centroids(cents, stream=ds)
        t0 = time.perf_counter()
        g.add(base, stream=ds)
        ds.synchronize()
        bulk_s = time.perf_counter() - t0
        st = g.pool_stats()
        row = {"block_vecs": T, "blocks_in_use": st.blocks_in_use,
               "pad_bytes": int((st.blocks_in_use * T - st.ntotal) * (w.d * 4 + 8)),
               "pool_bytes": int(st.pool_bytes),
               "bulk_load_vectors_per_s": len(w.base) / bulk_s, "search": {}}
        sizes_now = g.list_sizes()
        for bs in (1, 10, 32, 256):
            g.scan_time(reset=True)
            g.set_param("profile_scan", 1)
            lat = _search_latencies(g, queries, bs, w.k, w.nprobe, iters, ss, dev)
            g.set_param("profile_scan", 0)
            ms, cnt = g.scan_time(reset=True)
            nb = len(queries) // bs
            ub = []
            for i in range(min(32, nb)):
                pl = g.probe(queries[i * bs:(i + 1) * bs], w.nprobe).cpu().numpy()
                ub.append(int((sizes_now[np.unique(pl)] * w.d * 4).sum()))
            scan_ms = ms / max(cnt, 1)
            row["search"][str(bs)] = {"p50_ms": _p(lat, 50), "p99_ms": _p(lat, 99), "scan_ms": scan_ms,
                                      "scan_GBps": float(np.mean(ub)) / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else None}
        ib = w.insert_batch
        lat = []
        for i in range(iters + 10):
            t0 = time.perf_counter()
            g.add(inserts[(i % (len(inserts) // ib)) * ib:(i % (len(inserts) // ib)) * ib + ib], stream=ds)
            ds.synchronize()
            if i >= 10:
                lat.append((time.perf_counter() - t0) * 1e3)
        row["insert_batch64_p50_ms"] = _p(lat, 50)
        row["insert_batch64_p99_ms"] = _p(lat, 99)
        assert g.poll_error() == 0
        rows.append(row)
        g.close()
    return {"study": "block_size", "workload": w.name, "rows": rows}


def pq_study(scale: float = 1.0, ms=(16, 32), iters: int = 200, batches=(1, 10, 32, 256), params=None) -> dict:
    dev = torch.device("cuda:0")
    w = synth.config(2, scale=scale)
    base, cents, queries, inserts = (_to_dev(a, dev) for a in (w.base, w.centroids, w.queries, w.inserts))
    n_all = len(w.base) + 2 * len(w.inserts)
    blocks = n_all // w.block_vecs + 2 * w.nlist + 64
    kw = dict(pool_blocks=blocks, n_resources=8, max_batch=256, max_k=128, max_nprobe=64, max_add_batch=65536,
              candidates_per_query=65536)
    ds, ss = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
    flat = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, **kw)
    flat.set_centroids(cents, stream=ds)
    flat.add(base, stream=ds)
    ds.synchronize()
    nq_recall = min(1024, len(w.queries))

    def ids_of(index, o):
        ids = index.search(queries[o:min(o + 256, nq_recall)], w.k, w.nprobe, stream=ss)[1]
        ss.synchronize()
        return ids.cpu().numpy()

    exact = np.concatenate([ids_of(flat, o) for o in range(0, nq_recall, 256)])
    flat_bytes = int(flat.pool_stats().pool_bytes)
    flat.close()
    rows = []
    for M in ms:
        cb = _to_dev(synth.codebooks_from_rows(w.seed, w.base, M), dev)
        g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pq_m=M, **kw)
        g.set_centroids(cents, stream=ds)
        g.set_codebooks(cb, stream=ds)
        for key, value in (params or {}).items():  # launch-shape parameters of the library, e.g. pq_by_list
            g.set_param(key, value)
        t0 = time.perf_counter()
        g.add(base, stream=ds)
        ds.synchronize()
        bulk_s = time.perf_counter() - t0
        st = g.pool_stats()
        row = {"pq_m": M, "bytes_per_vector_in_lists": M + 8, "pool_bytes": int(st.pool_bytes),
               "flat_pool_bytes": flat_bytes, "bulk_load_vectors_per_s": len(w.base) / bulk_s, "search": {}}
        sizes_now = g.list_sizes()
        hit = 0
        for o in range(0, nq_recall, 256):
            got = ids_of(g, o)
            hit += sum(len(np.intersect1d(got[i], exact[o + i])) for i in range(len(got)))
        row["share_of_flat_topk_returned"] = hit / (nq_recall * w.k)
        for bs in batches:
            g.scan_time(reset=True)
            g.set_param("profile_scan", 1)
            lat = _search_latencies(g, queries, bs, w.k, w.nprobe, iters, ss, dev)
            g.set_param("profile_scan", 0)
            ms_, cnt = g.scan_time(reset=True)
            # table look-ups of one scan launch: one per (query, candidate, sub-space); the yardstick is what
            # the LDS of 256 CUs delivers without bank conflicts (128 bytes per clock each, 2.4 GHz, 4-byte entries)
            nb = max(len(queries) // bs, 1)
            looks = []
            for i in range(min(16, nb)):
                pl = g.probe(queries[i * bs:(i + 1) * bs], w.nprobe).cpu().numpy()
                looks.append(float(sizes_now[pl].sum()) * M)
            scan_ms = ms_ / max(cnt, 1)
            rate = float(np.mean(looks)) / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else None
            row["search"][str(bs)] = {"p50_ms": _p(lat, 50), "p99_ms": _p(lat, 99), "qps": bs / (np.mean(lat) * 1e-3),
                                      "scan_ms": scan_ms,
                                      "roofline": {"bound": "lds", "achieved": rate, "peak": LDS_LOOKUPS_PEAK_G,
                                                   "unit": "G look-ups/s", "frac": rate / LDS_LOOKUPS_PEAK_G if rate else None,
                                                   "lookups_per_launch": float(np.mean(looks))}}
        ib = w.insert_batch
        lat = []
        for i in range(iters + 10):
            t0 = time.perf_counter()
            g.add(inserts[(i % (len(inserts) // ib)) * ib:(i % (len(inserts) // ib)) * ib + ib], stream=ds)
            ds.synchronize()
            if i >= 10:
                lat.append((time.perf_counter() - t0) * 1e3)
        row["insert_batch64_p50_ms"] = _p(lat, 50)
        row["insert_batch64_p99_ms"] = _p(lat, 99)
        g.validate()
        assert g.poll_error() == 0
        rows.append(row)
        g.close()
    return {"study": "product_quantised_lists", "workload": w.name, "k": w.k, "nprobe": w.nprobe,
            "codebooks": "256 sampled sub-vectors per sub-space (untrained)", "rows": rows}


def storage_study(scale: float = 1.0, iters: int = 200, batches=(1, 10, 32, 256)) -> dict:
    """Flat lists that keep floats, halves or bytes: memory, insertion rate, search latency and the scan's
    rate in bytes of what the lists hold.  Two data sets: configuration 2 (byte-valued, so all three kinds
    return the same answers) and a fifth of configuration 3 (unit vectors, inner products; floats and halves)."""
    dev = torch.device("cuda:0")
    elem = {"f32": 4, "f16": 2, "u8": 1}
    out = []
    for idx, frac, kinds in ((2, 1.0, ("f32", "f16", "u8")), (3, 0.2, ("f32", "f16"))):
        w = synth.config(idx, scale=frac * scale)
        base, cents, queries, inserts = (_to_dev(a, dev) for a in (w.base, w.centroids, w.queries, w.inserts))
        n_all = len(w.base) + 2 * len(w.inserts)
        blocks = n_all // w.block_vecs + 2 * w.nlist + 64
        cand = max(65536, 4 * w.nprobe * (len(w.base) // w.nlist + w.block_vecs))
        ds, ss = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
        nq_recall = min(1024, len(w.queries))
        exact = None
        rows = []
        for kind in kinds:
            g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=blocks, n_resources=8, max_batch=256,
                            max_k=128, max_nprobe=64, max_add_batch=65536, candidates_per_query=cand, storage=kind)
            g.set_centroids(cents, stream=ds)
            t0 = time.perf_counter()
            g.add(base, stream=ds)
            ds.synchronize()
            bulk_s = time.perf_counter() - t0
            st = g.pool_stats()
            got = []
            for o in range(0, nq_recall, 256):
                ids = g.search(queries[o:min(o + 256, nq_recall)], w.k, w.nprobe, stream=ss)[1]
                ss.synchronize()
                got.append(ids.cpu().numpy())
            got = np.concatenate(got)
            if exact is None:
                exact = got
            share = sum(len(np.intersect1d(got[i], exact[i])) for i in range(len(got))) / (len(got) * w.k)
            row = {"storage": kind, "bytes_per_vector_in_lists": w.d * elem[kind] + 8,
                   "block_bytes": int(st.block_bytes), "blocks_in_use": int(st.blocks_in_use),
                   "list_bytes": int(st.block_bytes) * int(st.blocks_in_use),
                   "bulk_load_vectors_per_s": len(w.base) / bulk_s, "share_of_f32_topk_returned": share,
                   "search": {}}
            sizes_now = g.list_sizes()
            for bs in batches:
                g.scan_time(reset=True)
                g.set_param("profile_scan", 1)
                lat = _search_latencies(g, queries, bs, w.k, w.nprobe, iters, ss, dev)
                g.set_param("profile_scan", 0)
                ms_, cnt = g.scan_time(reset=True)
                nb = max(len(queries) // bs, 1)
                union = []  # bytes of the union of the probed lists, as stored
                for i in range(min(16, nb)):
                    pl = np.unique(g.probe(queries[i * bs:(i + 1) * bs], w.nprobe).cpu().numpy())
                    union.append(float(sizes_now[pl].sum()) * w.d * elem[kind])
                scan_ms = ms_ / max(cnt, 1)
                gbps = float(np.mean(union)) / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else None
                row["search"][str(bs)] = {"p50_ms": _p(lat, 50), "p99_ms": _p(lat, 99),
                                          "qps": bs / (np.mean(lat) * 1e-3), "scan_ms": scan_ms,
                                          "scan_bytes_per_launch": float(np.mean(union)), "scan_GBps": gbps,
                                          "frac_of_hbm_peak": gbps / 8000.0 if gbps else None}
            ib = w.insert_batch
            lat = []
            for i in range(iters + 10):
                t0 = time.perf_counter()
                g.add(inserts[(i % (len(inserts) // ib)) * ib:(i % (len(inserts) // ib)) * ib + ib], stream=ds)
                ds.synchronize()
                if i >= 10:
                    lat.append((time.perf_counter() - t0) * 1e3)
            row["insert_batch_p50_ms"] = _p(lat, 50)
            g.validate()
            assert g.poll_error() == 0
            rows.append(row)
            g.close()
        out.append({"workload": w.name, "metric": w.metric, "d": w.d, "n_base": len(w.base), "k": w.k,
                    "nprobe": w.nprobe, "insert_batch": w.insert_batch, "rows": rows})
    return {"study": "storage_of_flat_lists", "sets": out}


def shape_study(scale: float = 1.0, iters: int = 100, which=(3, 4, 5)) -> dict:
    """scale 1.0 stands for a fifth of configuration 3's and 4's base sets (2 M x 96, 1 M x 768) and a
    tenth of configuration 5's (2 M x 256): the host has to draw them."""
    dev = torch.device("cuda:0")
    frac = {3: 0.2, 4: 0.2, 5: 0.1}
    batches = {3: (128,), 4: (1, 64), 5: (256,)}
    rows = []
    for idx in which:
        t0 = time.perf_counter()
        w = synth.config(idx, scale=frac[idx] * scale)
        t_gen = time.perf_counter() - t0
        base, cents, queries, inserts = (_to_dev(a, dev) for a in (w.base, w.centroids, w.queries, w.inserts))
        n_all = len(w.base) + 2 * len(w.inserts)
        # room for the candidates: a few times the average, and for the skewed set a quarter of everything
        # (most queries of a batch may probe the hottest list, which holds a seventh of the vectors)
        cand = max(65536, 4 * w.nprobe * (len(w.base) // w.nlist + w.block_vecs))
        if idx == 5:
            cand = max(cand, len(w.base) // 4)
        g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=n_all // w.block_vecs + 2 * w.nlist + 64,
                        n_resources=4, max_batch=256, max_k=128, max_nprobe=64, max_add_batch=65536,
                        candidates_per_query=cand)
        ds, ss = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
        g.set_centroids(cents, stream=ds)
        t0 = time.perf_counter()
        g.add(base, stream=ds)
        ds.synchronize()
        bulk_s = time.perf_counter() - t0
        sizes_now = g.list_sizes()
        st = g.pool_stats()
        row = {"workload": w.name, "n_base": len(w.base), "d": w.d, "nlist": w.nlist, "metric": w.metric,
               "block_vecs": w.block_vecs, "nprobe": w.nprobe, "k": w.k, "host_generation_s": t_gen,
               "bulk_load_vectors_per_s": len(w.base) / bulk_s, "blocks_in_use": st.blocks_in_use,
               "longest_list": int(sizes_now.max()), "search": {}}
        for bs in batches[idx]:
            g.scan_time(reset=True)
            g.set_param("profile_scan", 1)
            lat = _search_latencies(g, queries, bs, w.k, w.nprobe, iters, ss, dev)
            g.set_param("profile_scan", 0)
            ms, cnt = g.scan_time(reset=True)
            nb = max(len(queries) // bs, 1)
            ub, pairs = [], []
            for i in range(min(16, nb)):
                pl = g.probe(queries[i * bs:(i + 1) * bs], w.nprobe).cpu().numpy()
                ub.append(int((sizes_now[np.unique(pl)] * w.d * 4).sum()))
                pairs.append(int(sizes_now[pl].sum()))
            scan_ms = ms / max(cnt, 1)
            gbps = float(np.mean(ub)) / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else None
            # arithmetic of the same launch: d subtract + d multiply-add lane instructions per (query, candidate)
            # pair for L2, d multiply-adds for IP, against 256 CUs x 64 lanes x 2.4 GHz unpacked fp32 issue
            lane_ops = float(np.mean(pairs)) * w.d * (2 if w.metric == "l2" else 1)
            t_ops = lane_ops / (scan_ms * 1e-3) / 1e12 if scan_ms > 0 else None
            row["search"][str(bs)] = {"p50_ms": _p(lat, 50), "p99_ms": _p(lat, 99), "qps": bs / (np.mean(lat) * 1e-3),
                                      "scan_ms": scan_ms, "scan_bytes": float(np.mean(ub)), "scan_GBps": gbps,
                                      "frac_of_hbm_peak": gbps / 8000.0 if gbps else None,
                                      "pairs": float(np.mean(pairs)), "alu_T_lane_instructions_per_s": t_ops,
                                      "frac_of_alu_issue_peak": t_ops / VALU_ISSUE_PEAK_T if t_ops else None}
        ib = w.insert_batch
        n_ib = max(len(inserts) // ib, 1)
        lat = []
        for i in range(iters + 10):
            t0 = time.perf_counter()
            g.add(inserts[(i % n_ib) * ib:(i % n_ib) * ib + ib], stream=ds)
            ds.synchronize()
            if i >= 10:
                lat.append((time.perf_counter() - t0) * 1e3)
        row["insert_batch"] = ib
        row["insert_p50_ms"] = _p(lat, 50)
        row["inserts_per_s_one_batch_in_flight"] = ib / (np.mean(lat) * 1e-3)
        assert g.poll_error() == 0
        rows.append(row)
        g.close()
        del base, cents, queries, inserts, w
        torch.cuda.empty_cache()
    return {"study": "shapes", "rows": rows}


def mixed_load_study(scale: float = 1.0, rates=(1_000, 5_000, 20_000, 50_000, 200_000), seconds: float = 2.0,
                     iters: int = 0) -> dict:
    """Open loop: operations arrive as a Poisson process at the offered rate whatever the index does; an
    operation is one query (70 %) or one inserted vector (30 %).  Queries are sent in batches whose size is
    drawn from {1, 2, 4, ..., 64} (a batch leaves when that many have arrived), inserted vectors in batches
    of 64.  Latency of an operation = completion of its batch minus its own arrival (it includes the wait
    for the batch to fill, which dominates at low rates); service time = completion minus submission of the
    batch.  `iters` is unused."""
    dev = torch.device("cuda:0")
    w = synth.config(4, scale=0.2 * scale)
    rng = np.random.Generator(np.random.PCG64([w.seed, 99]))
    base, cents, queries, inserts = (_to_dev(a, dev) for a in (w.base, w.centroids, w.queries, w.inserts))
    n_all = len(w.base) + 4 * len(w.inserts) + 200_000
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=n_all // w.block_vecs + 2 * w.nlist + 64,
                    n_resources=16, max_batch=64, max_k=16, max_nprobe=w.nprobe, max_add_batch=65536,
                    candidates_per_query=65536)
    data = torch.cuda.Stream(dev)
    sstreams = [torch.cuda.Stream(dev) for _ in range(7)]
    g.set_centroids(cents, stream=data)
    g.add(base, stream=data)
    data.synchronize()
    od = [torch.empty((64, w.k), dtype=torch.float32, device=dev) for _ in range(64)]
    oi = [torch.empty((64, w.k), dtype=torch.int64, device=dev) for _ in range(64)]
    for s_ in sstreams:  # warm up every stream
        g.search(queries[:64], w.k, w.nprobe, od[0], oi[0], stream=s_)
        s_.synchronize()
    rows = []
    nq, ni = len(queries), len(inserts)
    for rate in rates:
        n_ops = int(rate * seconds)
        gaps = rng.exponential(1.0 / rate, size=n_ops)
        arrivals = np.cumsum(gaps)
        is_query = rng.random(n_ops) < 0.7
        pend_q, pend_i = [], []          # arrival times of operations waiting for their batch
        want = int(2 ** rng.integers(0, 7))
        in_flight = []                   # (event, arrival times, kind)
        q_lat, i_lat, q_svc, i_svc = [], [], [], []
        busy = 0
        qpos = ipos = slot = 0
        free_events = [torch.cuda.Event() for _ in range(256)]

        def reap(block=False):
            keep = []
            for ev, arr, kind, t_sub in in_flight:
                if block:
                    ev.synchronize()
                if block or ev.query():
                    t = time.perf_counter() - t_start
                    (q_lat if kind == "q" else i_lat).extend((t - a) * 1e3 for a in arr)
                    (q_svc if kind == "q" else i_svc).append((t - t_sub) * 1e3)
                    free_events.append(ev)
                else:
                    keep.append((ev, arr, kind, t_sub))
            in_flight[:] = keep

        t_start = time.perf_counter()
        for op in range(n_ops):
            while time.perf_counter() - t_start < arrivals[op]:
                reap()
            if is_query[op]:
                pend_q.append(arrivals[op])
                if len(pend_q) >= want:
                    bs = len(pend_q)
                    st = sstreams[slot % len(sstreams)]
                    t_sub = time.perf_counter() - t_start
                    while True:
                        try:
                            g.search(queries[qpos:qpos + bs], w.k, w.nprobe, od[slot % 64][:bs], oi[slot % 64][:bs], stream=st)
                            break
                        except rtams.RtamsError as e:
                            if e.code != rtams.EBUSY:
                                raise
                            busy += 1
                            reap()
                    ev = free_events.pop() if free_events else torch.cuda.Event()
                    ev.record(st)
                    in_flight.append((ev, pend_q, "q", t_sub))
                    pend_q = []
                    qpos = (qpos + bs) % (nq - 64)
                    slot += 1
                    want = int(2 ** rng.integers(0, 7))
            else:
                pend_i.append(arrivals[op])
                if len(pend_i) >= 64:
                    t_sub = time.perf_counter() - t_start
                    g.add(inserts[ipos:ipos + 64], stream=data)
                    ev = free_events.pop() if free_events else torch.cuda.Event()
                    ev.record(data)
                    in_flight.append((ev, pend_i, "i", t_sub))
                    pend_i = []
                    ipos = (ipos + 64) % (ni - 64)
        t_sent = time.perf_counter() - t_start
        reap(block=True)
        t_done = time.perf_counter() - t_start
        assert g.poll_error() == 0
        rows.append({"offered_ops_per_s": rate, "operations": n_ops, "achieved_ops_per_s": (len(q_lat) + len(i_lat)) / t_done,
                     "generator_lag_ms": (t_sent - float(arrivals[-1])) * 1e3,
                     "query_latency_ms": {"p50": _p(q_lat, 50), "p99": _p(q_lat, 99), "n": len(q_lat)},
                     "insert_latency_ms": {"p50": _p(i_lat, 50), "p99": _p(i_lat, 99), "n": len(i_lat)},
                     "search_service_ms": {"p50": _p(q_svc, 50), "p99": _p(q_svc, 99), "requests": len(q_svc)},
                     "insert_service_ms": {"p50": _p(i_svc, 50), "p99": _p(i_svc, 99), "requests": len(i_svc)},
                     "requests_refused_busy": busy})
    g.validate()
    g.close()
    return {"study": "mixed_load", "workload": w.name, "n_base": len(w.base), "nprobe": w.nprobe, "k": w.k,
            "search_streams": len(sstreams), "seconds_per_rate": seconds, "rows": rows}


def online_latency_study(scale: float = 1.0, search_rates=(1_000, 5_000, 10_000),
                         insert_rates=(0, 100, 1_000, 2_000, 5_000, 10_000, 50_000), seconds: float = 3.0,
                         iters: int = 0) -> dict:
    """The shape of the paper's online experiment (its figure of average latency against the insert rate
    at fixed search rates; section "Comparing to state-of-the-art methods") on configuration 2's data:
    single queries arrive as a Poisson process at QPS_search and are sent one request each (nprobe 32, k
    100); single vectors arrive at QPS_insert and leave in batches of up to 64 (a batch leaves when it is
    full, or 10 ms after its first vector arrived); 7 search streams and the data stream.  Reported per
    point, as the paper does: the average latency of a search request plus the average latency of an
    insertion request (submission to completion), their p99s, and the time an operation waited for its
    batch.  `iters` is unused."""
    dev = torch.device("cuda:0")
    w = synth.config(2, scale=scale)
    rng = np.random.Generator(np.random.PCG64([w.seed, 77]))
    base, cents, queries, inserts = (_to_dev(a, dev) for a in (w.base, w.centroids, w.queries, w.inserts))
    n_all = len(w.base) + 3_000_000
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=n_all // w.block_vecs + 2 * w.nlist + 64,
                    n_resources=16, max_batch=64, max_k=128, max_nprobe=w.nprobe, max_add_batch=65536,
                    candidates_per_query=65536)
    data = torch.cuda.Stream(dev)
    sstreams = [torch.cuda.Stream(dev) for _ in range(7)]
    g.set_centroids(cents, stream=data)
    g.add(base, stream=data)
    data.synchronize()
    od = [torch.empty((1, w.k), dtype=torch.float32, device=dev) for _ in range(64)]
    oi = [torch.empty((1, w.k), dtype=torch.int64, device=dev) for _ in range(64)]
    for s_ in sstreams:
        g.search(queries[:1], w.k, w.nprobe, od[0], oi[0], stream=s_)
        s_.synchronize()
    nq, ni = len(queries), len(inserts)
    flush_s = 0.010
    rows = []
    for qs in search_rates:
        for qi in insert_rates:
            n_q = int(qs * seconds)
            tq = np.cumsum(rng.exponential(1.0 / qs, size=n_q))
            ti = np.cumsum(rng.exponential(1.0 / qi, size=int(qi * seconds))) if qi > 0 else np.zeros(0)
            times = np.concatenate([tq, ti])
            kinds = np.concatenate([np.ones(len(tq), bool), np.zeros(len(ti), bool)])
            order = np.argsort(times, kind="stable")
            times, kinds = times[order], kinds[order]
            in_flight, q_lat, i_lat, i_wait = [], [], [], []
            pend_i = []
            busy = 0
            qpos = ipos = slot = 0
            free_events = [torch.cuda.Event() for _ in range(256)]

            def reap(block=False):
                keep = []
                for ev, arr, kind, t_sub in in_flight:
                    if block:
                        ev.synchronize()
                    if block or ev.query():
                        t = time.perf_counter() - t_start
                        if kind == "q":
                            q_lat.append((t - t_sub) * 1e3)
                        else:
                            i_lat.append((t - t_sub) * 1e3)
                            i_wait.extend((t_sub - a) * 1e3 for a in arr)
                        free_events.append(ev)
                    else:
                        keep.append((ev, arr, kind, t_sub))
                in_flight[:] = keep

            def flush_inserts():
                nonlocal pend_i, ipos
                t_sub = time.perf_counter() - t_start
                n = len(pend_i)
                g.add(inserts[ipos:ipos + n], stream=data)
                ev = free_events.pop() if free_events else torch.cuda.Event()
                ev.record(data)
                in_flight.append((ev, pend_i, "i", t_sub))
                pend_i = []
                ipos = (ipos + n) % (ni - 64)

            t_start = time.perf_counter()
            for op in range(len(times)):
                while True:
                    now = time.perf_counter() - t_start
                    if pend_i and now - pend_i[0] >= flush_s:
                        flush_inserts()
                    if now >= times[op]:
                        break
                    reap()
                if kinds[op]:
                    st = sstreams[slot % len(sstreams)]
                    t_sub = time.perf_counter() - t_start
                    while True:
                        try:
                            g.search(queries[qpos:qpos + 1], w.k, w.nprobe, od[slot % 64], oi[slot % 64], stream=st)
                            break
                        except rtams.RtamsError as e:
                            if e.code != rtams.EBUSY:
                                raise
                            busy += 1
                            reap()
                    ev = free_events.pop() if free_events else torch.cuda.Event()
                    ev.record(st)
                    in_flight.append((ev, None, "q", t_sub))
                    qpos = (qpos + 1) % (nq - 1)
                    slot += 1
                else:
                    pend_i.append(times[op])
                    if len(pend_i) >= 64:
                        flush_inserts()
            if pend_i:
                flush_inserts()
            t_sent = time.perf_counter() - t_start
            reap(block=True)
            assert g.poll_error() == 0
            sa = float(np.mean(q_lat)) if q_lat else 0.0
            ia = float(np.mean(i_lat)) if i_lat else 0.0
            rows.append({"qps_search": qs, "qps_insert": qi, "search_requests": len(q_lat), "insert_requests": len(i_lat),
                         "latency_avg_ms": sa + ia, "search_avg_ms": sa, "search_p99_ms": _p(q_lat, 99) if q_lat else None,
                         "insert_avg_ms": ia if i_lat else None, "insert_p99_ms": _p(i_lat, 99) if i_lat else None,
                         "insert_wait_for_batch_avg_ms": float(np.mean(i_wait)) if i_wait else None,
                         "generator_lag_ms": (t_sent - float(times[-1])) * 1e3, "requests_refused_busy": busy})
    g.validate()
    g.close()
    return {"study": "online_latency", "workload": w.name, "n_base": len(w.base), "nprobe": w.nprobe, "k": w.k,
            "search_streams": len(sstreams), "seconds_per_point": seconds, "insert_batch": 64, "insert_flush_ms": flush_s * 1e3,
            "rows": rows}


def growth_study(scale: float = 1.0, seconds: float = 6.0, rate: float = 100_000.0, threshold: int = 10_000,
                 iters: int = 0) -> dict:
    """Skewed growth under load: a tenth of configuration 5's base set, then `seconds` of inserts at `rate`
    vectors/s (batches of 1024, list popularity Zipf(1.1)) on the data stream with the rearrangement
    threshold armed, and closed-loop searches (batch 256, nprobe 64, k 50) on a search stream.  Reports the
    search latency per second of the run and the state of the hottest lists.  `iters` is unused."""
    dev = torch.device("cuda:0")
    w = synth.config(5, scale=0.1 * scale)
    base, cents, queries, inserts = (_to_dev(a, dev) for a in (w.base, w.centroids, w.queries, w.inserts))
    ib = w.insert_batch
    n_new = int(rate * seconds) + 4 * ib
    n_all = len(w.base) + n_new
    g = rtams.Index(w.d, w.nlist, w.metric, w.block_vecs, pool_blocks=n_all // w.block_vecs + 3 * w.nlist + 4096,
                    rearrange_threshold=threshold, n_resources=8, max_batch=256, max_k=64, max_nprobe=64,
                    max_add_batch=65536,
                    candidates_per_query=max(65536, 4 * w.nprobe * (n_all // w.nlist + w.block_vecs)))
    data, ss = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
    g.set_centroids(cents, stream=data)
    g.add(base, stream=data)
    data.synchronize()
    sizes0 = g.list_sizes()
    hot = [int(i) for i in np.argsort(-sizes0)[:4]]
    runs0 = {h: g.list_info(h)[1] for h in hot}
    st0 = g.pool_stats()
    bs = 256
    od = torch.empty((bs, w.k), dtype=torch.float32, device=dev)
    oi = torch.empty((bs, w.k), dtype=torch.int64, device=dev)
    nb = max(len(queries) // bs, 1)

    def search_for(duration, sink):
        i = 0
        t_end = time.perf_counter() + duration
        while time.perf_counter() < t_end:
            t = time.perf_counter()
            g.search(queries[(i % nb) * bs:(i % nb) * bs + bs], w.k, w.nprobe, od, oi, stream=ss)
            ss.synchronize()
            sink.append((t, (time.perf_counter() - t) * 1e3))
            i += 1

    quiet = []
    search_for(0.5, quiet)
    stop = threading.Event()
    sent = [0]
    n_ib = len(inserts) // ib

    def inserter():
        period = ib / rate
        nxt = time.perf_counter()
        i = 0
        while not stop.is_set():
            g.add(inserts[(i % n_ib) * ib:(i % n_ib) * ib + ib], stream=data)
            sent[0] += ib
            i += 1
            nxt += period
            dt = nxt - time.perf_counter()
            if dt > 0:
                time.sleep(dt)

    lat = []
    th = threading.Thread(target=inserter)
    t0 = time.perf_counter()
    th.start()
    search_for(seconds, lat)
    stop.set()
    th.join()
    data.synchronize()
    t_run = time.perf_counter() - t0
    g.rearrange(-1, stream=data)  # the rounds the last batches asked for
    data.synchronize()
    after = []
    search_for(0.5, after)
    assert g.poll_error() == 0
    g.validate()
    sizes1 = g.list_sizes()
    st1 = g.pool_stats()
    per_second = []
    for sec in range(int(seconds)):
        xs = [l for (t, l) in lat if sec <= t - t0 < sec + 1]
        per_second.append({"second": sec, "requests": len(xs), "p50_ms": _p(xs, 50), "p99_ms": _p(xs, 99)})
    out = {"study": "skewed_growth", "workload": w.name, "n_base": len(w.base), "rearrange_threshold": threshold,
           "insert_rate_offered": rate, "insert_rate_achieved": sent[0] / t_run, "vectors_inserted": sent[0],
           "search": {"before": {"p50_ms": _p([l for _, l in quiet], 50), "p99_ms": _p([l for _, l in quiet], 99)},
                      "during": {"p50_ms": _p([l for _, l in lat], 50), "p99_ms": _p([l for _, l in lat], 99),
                                 "requests": len(lat), "per_second": per_second},
                      "after": {"p50_ms": _p([l for _, l in after], 50), "p99_ms": _p([l for _, l in after], 99)}},
           "hot_lists": [{"list": h, "vectors_before": int(sizes0[h]), "vectors_after": int(sizes1[h]),
                          "blocks_after": int(g.list_info(h)[0]), "runs_before": int(runs0[h]),
                          "runs_after": int(g.list_info(h)[1])} for h in hot],
           "pool": {"blocks_in_use_before": st0.blocks_in_use, "blocks_in_use_after": st1.blocks_in_use,
                    "blocks_free_after": st1.blocks_free, "lists_exceeding_after": st1.lists_exceeding,
                    "utilisation_after": st1.utilisation}}
    g.close()
    return out
