"""Host-side check of the error bound behind the brute force's fp32 screen (Sec. 2.1, 5.3.1: the exact
graph is what recall is measured against, so the screen may never lose a true neighbour).

k_brute_mfma rules a pair out when <q,b>, as the fp32 matrix instructions deliver it, lies below
h_q + h_b, which is algebraically "fp32 distance - E > T" with E = (d + 16) 2^-23 (|q|^2 + |b|^2)
(squared L2) or (d + 16) 2^-23 (|q|^2 / 2 + |b|^2 / 2 + 1) (1 - <q,b>) and T a bound on the query's
final k-th distance, padded by 2^-20 of itself.  Whatever order the hardware sums the d products
in, its result differs from the true dot product by at most gamma_d sum |q_i b_i| (gamma_d =
d u / (1 - d u), u = 2^-24).  The tests put the *worst* value that bound allows into the screen's
arithmetic (fp32, with and without the multiply-adds fused) and require that a pair whose exact
distance does not exceed T still passes -- on data far from the origin, near-duplicates, integer
values and unit vectors, for short and long rows.  Halving the bound's d-term and dropping its
constant must fail the same check, so the check can tell.
"""
import numpy as np
import pytest

F = np.float32


def _fma(a, b, c):
    return F(np.float64(a) * np.float64(b) + np.float64(c))      # one rounding (exact in fp64 for fp32 inputs up to the sum)


def _screen_passes(acc, nq, nb, t_bound, d, metric, fused, d_term=1.0, const=16.0):
    """The kernel's arithmetic for one pair, in fp32.  acc: the fp32 <q,b>; nq, nb: fp32 squared norms."""
    epsd = F(F(d_term * d + const) * F(1.1920929e-7))
    t = F(F(t_bound) * F(1.000001))
    half = F(0.5)
    if metric == 0:
        c = F(half * F(F(1.0) - epsd))
        hq = _fma(c, nq, -F(half * t)) if fused else F(F(c * nq) - F(half * t))
        h = _fma(c, nb, hq) if fused else F(hq + F(c * nb))
    else:
        hq0 = F(F(F(1.0) - t) - epsd)
        ce = F(half * epsd)
        hq = _fma(-ce, nq, hq0) if fused else F(hq0 - F(ce * nq))
        h = _fma(-ce, nb, hq) if fused else F(hq - F(ce * nb))
    return not (acc < h)


def _exact_distance(q, b, metric):
    """The ABI's recipe: fp64 chain in index order, fused multiply-add, one rounding to fp32."""
    acc = np.float64(0.0)
    if metric == 0:
        for x, y in zip(q.astype(np.float64), b.astype(np.float64)):
            df = x - y
            acc = df * df + acc          # (numpy has no fused multiply-add: up to 2^-53 relative per step, far below fp32)
        return F(acc)
    for x, y in zip(q.astype(np.float64), b.astype(np.float64)):
        acc = x * y + acc
    r = 1.0 - acc
    return F(r if r > 0.0 else 0.0)


def _pairs(kind, d, rng, count):
    if kind == "far":                       # a tight cloud far from the origin: the screen can rule out nothing
        c = rng.standard_normal(d) * 1000.0
        pts = c + rng.standard_normal((2 * count, d)) * 0.01
    elif kind == "dup":                     # near-duplicates: distances a 1e-8 of the norms
        base = rng.standard_normal((count, d)) * 3.0
        pts = np.concatenate([base, base * (1.0 + 1e-6 * rng.standard_normal((count, 1)))])
    elif kind == "int":                     # integer values as in 8-bit descriptors
        pts = rng.integers(0, 256, (2 * count, d)).astype(np.float64)
    elif kind == "unit":
        pts = rng.standard_normal((2 * count, d))
        pts /= np.linalg.norm(pts, axis=1, keepdims=True)
    else:                                   # ordinary gaussian data
        pts = rng.standard_normal((2 * count, d))
    pts = pts.astype(F)
    return pts[:count], pts[count:]


def _check(kind, d, metric, seed, d_term=1.0, const=16.0, count=24):
    rng = np.random.default_rng(seed)
    qs, bs = _pairs(kind, d, rng, count)
    lost = 0
    u = 2.0 ** -24
    gamma = d * u / (1.0 - d * u)
    for q, b in zip(qs, bs):
        q64, b64 = q.astype(np.float64), b.astype(np.float64)
        nq, nb = F(np.dot(q64, q64)), F(np.dot(b64, b64))        # the pre-pass: an fp64 sum rounded once
        dot = float(np.dot(q64, b64))
        worst = F(dot - gamma * float(np.dot(np.abs(q64), np.abs(b64))))      # the lowest <q,b> any order may give
        dist = _exact_distance(q, b, metric)
        # bounds the pair must survive: its own exact distance, the next fp32 above it, a slack one
        for t_bound in (dist, np.nextafter(dist, F(np.inf)), F(dist * F(1.5)), F(np.inf)):
            for acc in (worst, F(dot)):
                for fused in (False, True):
                    if not _screen_passes(acc, nq, nb, t_bound, d, metric, fused, d_term, const):
                        lost += 1
    return lost


@pytest.mark.parametrize("d", (4, 32, 100, 128, 960))
@pytest.mark.parametrize("kind", ("far", "dup", "int", "gauss"))
def test_screen_never_loses_a_pair_within_the_bound_l2(kind, d):
    assert _check(kind, d, 0, seed=d) == 0


@pytest.mark.parametrize("d", (4, 96, 128, 960))
@pytest.mark.parametrize("kind", ("unit", "dup", "gauss"))
def test_screen_never_loses_a_pair_within_the_bound_ip(kind, d):
    assert _check(kind, d, 1, seed=1000 + d) == 0


def test_a_bound_without_its_margin_does_lose_pairs():
    """The same check with a quarter (a tenth for 1 - <q,b>, whose bound carries a constant 1) of the
    bound's d-term and no constant: the worst-case <q,b> is then ruled out although the pair's exact
    distance equals the bound."""
    lost = sum(_check("far", d, 0, seed=d, d_term=0.25, const=0.0) for d in (128, 960))
    assert lost > 0
    lost_ip = sum(_check("unit", d, 1, seed=d, d_term=0.1, const=0.0) for d in (128, 960))
    assert lost_ip > 0
