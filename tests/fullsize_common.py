"""What the parity tests at the configurations' full sizes share: progress lines that get past
pytest's capture (a multi-gigabyte set takes a minute to draw, load and check, and a run that prints
nothing looks hung), and the list of every base vector for the oracle without its one-chain-at-a-time
assignment pass, which takes minutes for ten million vectors: either the list is known from how the
set was drawn, or a double-precision matrix product names the few centroids that can win and the
oracle's own arithmetic decides among them.  Either shortcut is checked against the oracle's
assignment on a large random sample before it is used.  Nothing here touches the HIP library."""
from __future__ import annotations

import os
import time

import numpy as np
from concurrent.futures import ThreadPoolExecutor
from threadpoolctl import threadpool_limits

_T0 = time.time()


def say(request, msg: str) -> None:
    line = f"[fullsize +{time.time() - _T0:6.1f}s] {msg}"
    capman = request.config.pluginmanager.getplugin("capturemanager")
    if capman is not None:
        with capman.global_and_fixture_disabled():
            print(line, flush=True)
    else:
        print(line, flush=True)


def filtered_assignment(o, metric: str, X: np.ndarray, C: np.ndarray, rows_per_step: int = 4096,
                        margin: float = 1e-9) -> np.ndarray:
    """Nearest centroid of every row of X (ties to the lowest index).  A double-precision matrix
    product gives every (row, centroid) score to about 1e-13; the centroids within `margin`
    (relative to the scores' magnitude) of a row's best are the only ones that can win, and where
    there is more than one the oracle's coarse scores of that row decide."""
    C64 = C.astype(np.float64)
    cn = np.einsum("ij,ij->i", C64, C64)
    out = np.empty(len(X), dtype=np.int32)

    def step(lo: int) -> None:
        x = X[lo:lo + rows_per_step].astype(np.float64)
        s = x @ C64.T
        if metric == "l2":  # |x|^2 is the same for every centroid of a row
            s *= -2.0
            s += cn
            xn = np.einsum("ij,ij->i", x, x)
            best = s.min(axis=1)
            scale = np.abs(best) + xn + 1.0
            near = s <= (best + margin * scale)[:, None]
        else:
            best = s.max(axis=1)
            scale = np.abs(best) + 1.0
            near = s >= (best - margin * scale)[:, None]
        out[lo:lo + len(x)] = near.argmax(axis=1)
        for r in np.nonzero(near.sum(axis=1) > 1)[0]:
            exact = o.coarse_scores(X[lo + r])
            cand = np.nonzero(near[r])[0]
            e = exact[cand]
            out[lo + r] = cand[np.argmin(e) if metric == "l2" else np.argmax(e)]  # first of the best: lowest index

    # row steps side by side on threads (numpy releases the interpreter lock), one BLAS thread each
    with threadpool_limits(limits=1, user_api="blas"):
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
            list(pool.map(step, range(0, len(X), rows_per_step)))
    return out


def check_assignment_on_sample(o, X: np.ndarray, assign: np.ndarray, n_sample: int, seed: int) -> int:
    """The oracle's own assignment of a random sample must be the shortcut's."""
    rng = np.random.default_rng(seed)
    rows = np.sort(rng.choice(len(X), size=min(n_sample, len(X)), replace=False))
    ref = o.assign(X[rows])
    bad = np.nonzero(ref != assign[rows])[0]
    assert len(bad) == 0, f"shortcut assignment differs from the oracle's on {len(bad)} of {len(rows)} sampled vectors"
    return len(rows)


def compare_lists(g, o, lists, what: str) -> None:
    """ids and vector bits of the given lists, as sets (sorted by id)."""
    for k in lists:
        gi, gx = g.list_export(int(k))
        gi, gx = gi.cpu().numpy(), gx.cpu().numpy()
        oi, ox = o.list_export(int(k))
        a, b = np.argsort(gi, kind="stable"), np.argsort(oi, kind="stable")
        assert np.array_equal(gi[a], oi[b]), f"{what}: list {k}: ids differ"
        assert np.array_equal(gx[a].view(np.uint32), ox[b].view(np.uint32)), f"{what}: list {k}: vector bits differ"
        del gi, gx, oi, ox
