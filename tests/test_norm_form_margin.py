"""The margin the matrix-core scan relies on when it scores squared distances in the norm form
|x|^2 + |q|^2 - 2 <x, q>: |norm form - direct form| <= slack (2 v + 3 |q|^2) with slack = 1.01 (4 d + 8)
2^-24, for v either of the two values.  Checked on the CPU against fp32 emulations of both forms (the
norm form with its inner product added in several orders, the direct form as one chain in the order
of the coordinates).  The GPU loosens every limit by this margin before it compares across the two
forms; nothing here touches the HIP library."""
import numpy as np
import pytest

F = np.float32


def direct_form(x, q):
    acc = F(0)
    for a, b in zip(x, q):
        t = F(a - b)
        acc = F(acc + F(t * t))  # (the GPU fuses multiply and add: one rounding fewer, inside the same margin)
    return acc


def norm_form(x, q, order):
    xn = F(0)
    for a in x:
        xn = F(xn + F(a * a))
    qn = F(np.sum(q.astype(np.float64) ** 2))  # |q|^2 is computed in double and rounded once
    dot = F(0)
    for j in order:
        dot = F(dot + F(x[j] * q[j]))
    return F(F(xn + qn) + F(F(-2) * dot)), qn


@pytest.mark.parametrize("d", [4, 32, 128, 260])
@pytest.mark.parametrize("kind", ["near", "far", "offset", "mixed-scales"])
def test_norm_form_stays_within_the_margin_of_the_direct_form(d, kind):
    rng = np.random.default_rng(17 * d + len(kind))
    slack = 1.01 * (4 * d + 8) * 2.0 ** -24
    worst = 0.0
    for _ in range(40):
        if kind == "near":  # neighbours: the distance is a small difference of large norms
            q = rng.standard_normal(d)
            x = q + 0.01 * rng.standard_normal(d)
        elif kind == "far":
            q, x = rng.standard_normal(d), rng.standard_normal(d)
        elif kind == "offset":
            q = 50.0 + rng.standard_normal(d)
            x = q + 0.1 * rng.standard_normal(d)
        else:
            scale = 10.0 ** rng.integers(-2, 3, size=d)
            q, x = rng.standard_normal(d) * scale, rng.standard_normal(d) * scale
        q, x = q.astype(F), x.astype(F)
        dv = float(direct_form(x, q))
        for order in (np.arange(d), np.arange(d)[::-1], rng.permutation(d)):
            nv, qn = norm_form(x, q, order)
            nv, qn = float(nv), float(qn)
            for v in (dv, max(nv, 0.0)):
                margin = slack * (2.0 * v + 3.0 * qn)
                assert abs(nv - dv) <= margin, f"{kind} d={d}: |{nv} - {dv}| above {margin}"
                worst = max(worst, abs(nv - dv) / margin)
    assert worst < 1.0
