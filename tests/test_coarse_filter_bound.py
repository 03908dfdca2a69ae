"""The error bound the matrix-core coarse filter relies on, checked on the CPU against an emulation of
what the matrix instruction is fed: operands split into two bf16 halves (round to nearest even),
the three products hi*hi + hi*lo + lo*hi, accumulation in fp32.  The GPU path decides nothing from
these scores; it only assumes |approx - exact| <= E when it picks the centroids to rescore exactly,
with E = (4 (d + 4) 2^-24 + 4 * 2^-16) (|y|^2 + max |c|^2).  Nothing here touches the HIP library."""
import numpy as np
import pytest


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32."""
    b = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) >> 16 << 16
    return b.astype(np.uint32).view(np.float32)


def split(x):
    hi = bf16_round(x)
    lo = bf16_round((x - hi).astype(np.float32))  # the difference is exact in fp32
    return hi, lo


def approx_scores(y, C, metric, order):
    """What the filter computes for one vector against all centroids, with the products added in fp32
    in the given order of the coordinates (the matrix cores' own order is not documented)."""
    yh, yl = split(y)
    Ch, Cl = split(C)
    # every product of two bf16 values is exact in fp32
    terms = np.stack([Cl * yh, Ch * yl, Ch * yh], axis=2).astype(np.float32)  # [nlist][d][3]
    terms = terms[:, order, :].reshape(len(C), -1)
    acc = np.zeros(len(C), np.float32)
    for j in range(terms.shape[1]):
        acc = (acc + terms[:, j]).astype(np.float32)
    if metric == "ip":
        return -acc
    cn = (C.astype(np.float64) ** 2).sum(axis=1).astype(np.float32)
    return (cn - np.float32(2) * acc).astype(np.float32)


def exact_scores(y, C, metric):
    y64, C64 = y.astype(np.float64), C.astype(np.float64)
    if metric == "ip":
        return -(C64 @ y64)
    return (C64 ** 2).sum(axis=1) - 2.0 * (C64 @ y64)  # |y|^2 is the same for every centroid


def bound(y, C, d):
    norms = float((y.astype(np.float64) ** 2).sum() + (C.astype(np.float64) ** 2).sum(axis=1).max())
    return (4.0 * (d + 4) * 2.0 ** -24 + 4.0 * 2.0 ** -16) * norms


@pytest.mark.parametrize("metric", ["l2", "ip"])
@pytest.mark.parametrize("d", [4, 36, 128, 260])
@pytest.mark.parametrize("kind", ["gauss", "offset", "mixed-scales", "all-positive"])
def test_split_contraction_stays_inside_the_band(metric, d, kind):
    rng = np.random.default_rng(d * 7 + len(kind))
    nlist = 64
    if kind == "gauss":
        C = rng.standard_normal((nlist, d))
        y = C[3] + 0.01 * rng.standard_normal(d)
    elif kind == "offset":  # data far from the origin: the norms dwarf the distances
        C = 100.0 + rng.standard_normal((nlist, d))
        y = C[5] + 0.001 * rng.standard_normal(d)
    elif kind == "mixed-scales":
        scale = 10.0 ** rng.integers(-3, 4, size=d)
        C = rng.standard_normal((nlist, d)) * scale
        y = rng.standard_normal(d) * scale
    else:  # no cancellation between the products: the rounding errors add up with one sign
        C = rng.random((nlist, d)) + 0.5
        y = rng.random(d) + 0.5
    C, y = C.astype(np.float32), y.astype(np.float32)
    E = bound(y, C, d)
    exact = exact_scores(y, C, metric)
    for order in (np.arange(d), np.arange(d)[::-1], rng.permutation(d)):
        err = np.abs(approx_scores(y, C, metric, order).astype(np.float64) - exact).max()
        assert err <= E, f"{kind} d={d} {metric}: error {err:.3e} above the bound {E:.3e}"


def test_the_split_leaves_at_most_two_to_the_minus_16():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(200000) * 10.0 ** rng.integers(-20, 20, 200000)).astype(np.float32)
    hi, lo = split(x)
    r = x.astype(np.float64) - hi.astype(np.float64) - lo.astype(np.float64)
    assert np.all(np.abs(r) <= 2.0 ** -16 * np.abs(x.astype(np.float64)))
    assert np.all(np.abs(lo.astype(np.float64)) <= 2.0 ** -8 * np.abs(x.astype(np.float64)) * (1 + 2.0 ** -7))
