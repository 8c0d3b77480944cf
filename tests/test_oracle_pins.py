"""Pins for the CPU oracle: what the paper and the mathematics fix.

None of these re-type the oracle's formula over the same data path: expected
values come from closed forms (trigonometry on angles, hand-worked integer
cases), from limiting cases the paper states (tau = 2 is plain averaging,
Sec. 4.1; a seed that agrees with nothing leaves c = 1, Sec. 3.1), from the
sketch of Fig. 2, from numpy's own mean, and from the statistics of the
synthetic generators.
"""
import math
import os

import numpy as np
import pytest

from conftest import oracle_arrays
from paper_2412_18052_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
f32 = np.float32


def vecs(*rows):
    return [np.array(r, dtype=f32) for r in rows]


# ---------------------------------------------------------------- Eq. 4 -----
def test_identical_negated_orthogonal(oracle):
    rng = np.random.default_rng(1)
    x = rng.standard_normal(1001).astype(f32)
    assert abs(oracle.cosine_distance(x, x)) < 1e-12            # perfectly correlated: 0
    assert abs(oracle.cosine_distance(x, -x) - 2.0) < 1e-12     # opposite: 2
    a = np.zeros(1000, f32); b = np.zeros(1000, f32)
    a[:500] = rng.standard_normal(500); b[500:] = rng.standard_normal(500)
    assert oracle.cosine_distance(a, b) == 1.0                  # disjoint supports: exactly 1


def test_hand_worked_pairs(oracle):
    # 3-4-5 triangle: cos = 24/25
    assert abs(oracle.cosine_distance(*vecs([3, 4], [4, 3])) - (1 - 24 / 25)) < 1e-15
    # 45 degrees and 135 degrees
    assert abs(oracle.cosine_distance(*vecs([1, 0, 0], [1, 1, 0])) - (1 - 1 / math.sqrt(2))) < 1e-15
    assert abs(oracle.cosine_distance(*vecs([1, 0], [-1, 1])) - (1 + 1 / math.sqrt(2))) < 1e-15
    # asymmetric lengths: x.y = 2, |x|^2 = 1, |y|^2 = 4+9+36 = 49  -> cos = 2/7
    assert abs(oracle.cosine_distance(*vecs([1, 0, 0], [2, 3, 6])) - (1 - 2 / 7)) < 1e-15
    # symmetric in its arguments
    x, y = vecs([1, 2, 3, 4], [-2, 0.5, 1, 7])
    assert oracle.cosine_distance(x, y) == oracle.cosine_distance(y, x)


def test_angle_closed_form(oracle):
    # unit-circle vectors: D = 1 - cos(difference of angles)
    for a, b, ra, rb in [(10, 55, 1.0, 3.0), (200, 20, 0.1, 7.0), (0, 90, 2.0, 2.0), (33, 303, 5.0, 0.5)]:
        x = np.array([ra * math.cos(math.radians(a)), ra * math.sin(math.radians(a))], f32)
        y = np.array([rb * math.cos(math.radians(b)), rb * math.sin(math.radians(b))], f32)
        assert abs(oracle.cosine_distance(x, y) - (1 - math.cos(math.radians(a - b)))) < 2e-7


def test_scale_invariance(oracle):
    rng = np.random.default_rng(2)
    g = [rng.standard_normal(4096).astype(f32) for _ in range(5)]
    out, mask, dist, c = oracle.aggregate(g, 1.0)
    for k in (0.125, 4.0, 1024.0):   # powers of two: exact rescaling in binary32
        out2, mask2, dist2, c2 = oracle.aggregate([x * f32(k) for x in g], 1.0)
        assert mask2.tolist() == mask.tolist() and c2 == c
        np.testing.assert_allclose(dist2, dist, rtol=0, atol=1e-14)
        np.testing.assert_allclose(out2, out * k, rtol=1e-15)
    # rescaling one non-seed input alone leaves every distance and the mask alone
    g2 = list(g); g2[2] = g2[2] * f32(8.0)
    _, mask3, dist3, _ = oracle.aggregate(g2, 2.0)
    _, mask0, dist0, _ = oracle.aggregate(g, 2.0)
    assert mask3.tolist() == mask0.tolist()
    assert abs(dist3[2] - dist0[2]) < 1e-14   # (later distances change: the sum changed)


def test_zero_norm_and_nan(oracle):
    z = np.zeros(8, f32); x = np.arange(1, 9, dtype=f32)
    assert oracle.cosine_distance(z, x) == 1.0 and oracle.cosine_distance(x, z) == 1.0
    out, mask, dist, c = oracle.aggregate([x, z, x], 0.5)
    assert mask.tolist() == [1, 0, 1] and c == 2 and dist[1] == 1.0
    bad = x.copy(); bad[3] = np.nan
    out, mask, dist, c = oracle.aggregate([x, bad, x], 2.0)
    assert mask.tolist() == [1, 0, 1] and math.isnan(dist[1]) and c == 2
    np.testing.assert_array_equal(out, x.astype(np.float64))


# ------------------------------------------------------- Algorithm 1 --------
def test_tau_two_is_plain_average(oracle):
    rng = np.random.default_rng(3)
    g = [rng.standard_normal(10007).astype(f32) * f32(s) for s in (1, 3, 0.2, 5, 1, 1, 2)]
    out, mask, dist, c = oracle.aggregate(g, 2.0)
    assert mask.tolist() == [1] * 7 and c == 7
    mean = np.mean(np.stack(g).astype(np.float64), axis=0)     # Eq. 2 by numpy
    np.testing.assert_allclose(out, mean, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(oracle.plain_average(g), mean, rtol=1e-13, atol=1e-15)
    # exactly negated data is a tie at 2 up to rounding: use a threshold just above
    out, mask, dist, c = oracle.aggregate([g[0], -g[0] * f32(0.5)], 2.001)
    assert mask.tolist() == [1, 1] and abs(dist[1] - 2.0) < 1e-12
    np.testing.assert_allclose(out, g[0].astype(np.float64) * 0.25, rtol=1e-15)


def test_negative_tau_keeps_only_seed(oracle):
    rng = np.random.default_rng(4)
    g = [rng.standard_normal(999).astype(f32) for _ in range(6)]
    g[3] = g[0].copy()            # even an identical copy has D = 0 > tau
    out, mask, dist, c = oracle.aggregate(g, -1e-6)
    assert mask.tolist() == [1, 0, 0, 0, 0, 0] and c == 1
    np.testing.assert_array_equal(out, g[0].astype(np.float64))
    assert dist[0] == 0.0 and abs(dist[3]) < 1e-12


def test_seed_orthogonal_to_all_skips_macrobatch(oracle):
    # Sec. 3.1: a seed orthogonal to everything else leaves c = 1
    e = np.eye(6, dtype=f32)
    g = [e[0], e[1] + e[2], e[2] + e[3], e[1] + e[2], e[4]]
    out, mask, dist, c = oracle.aggregate(g, 0.97)
    assert c == 1 and mask.tolist() == [1, 0, 0, 0, 0]
    assert dist[1:].tolist() == [1.0] * 4
    np.testing.assert_array_equal(out, e[0].astype(np.float64))
    # the same set with another seed finds agreement: order dependence
    out, mask, dist, c = oracle.aggregate([g[1], g[0], g[2], g[3], g[4]], 0.97)
    assert mask.tolist() == [1, 0, 1, 1, 0] and c == 3


def test_hand_worked_sequence(oracle):
    # g=(1,0); (0,1): D=1 exactly, accepted at tau=1 (tie counts as accept);
    # sum (1,1); (-1,-1): D=2 rejected; (1,-1): D=1 accepted; sum (2,0); c=3
    g = vecs([1, 0], [0, 1], [-1, -1], [1, -1])
    out, mask, dist, c = oracle.aggregate(g, 1.0)
    assert mask.tolist() == [1, 1, 0, 1] and c == 3
    assert dist[0] == 0.0 and dist[1] == 1.0 and abs(dist[2] - 2.0) < 1e-15 and abs(dist[3] - 1.0) < 1e-15
    np.testing.assert_allclose(out, [2 / 3, 0.0], rtol=1e-15)
    # distance is against the running SUM, not the seed and not the last accepted:
    # seed (1,0), then (1,1) [D=1-1/sqrt2, accept], sum=(2,1);
    # (0,1): vs sum cos = 1/sqrt5 -> D = 0.5528; vs seed it would be 1; vs last 0.2929
    g = vecs([1, 0], [1, 1], [0, 1])
    out, mask, dist, c = oracle.aggregate(g, 0.6)
    assert abs(dist[2] - (1 - 1 / math.sqrt(5))) < 1e-15 and mask.tolist() == [1, 1, 1]
    np.testing.assert_allclose(out, [2 / 3, 2 / 3], rtol=1e-15)
    # a rejected gradient leaves sum and count alone: mean is over the accepted only
    g = vecs([2, 0], [0, 5], [2, 2])
    out, mask, dist, c = oracle.aggregate(g, 0.5)
    assert mask.tolist() == [1, 0, 1] and c == 2
    np.testing.assert_allclose(out, [2.0, 1.0], rtol=1e-15)
    # integer case with unequal norms, P = 4
    g = vecs([1, 2, 2, 0], [2, 4, 4, 0], [0, 0, 0, 3], [-3, -6, -6, 1])
    out, mask, dist, c = oracle.aggregate(g, 0.9)
    # D2 = 0; sum = (3,6,6,0); D3 = 1; D4: dot = -81, |sum| = 9, |g4| = sqrt(82)
    assert abs(dist[1]) < 1e-15 and dist[2] == 1.0
    assert abs(dist[3] - (1 + 81 / (9 * math.sqrt(82)))) < 1e-15
    assert mask.tolist() == [1, 1, 0, 0] and c == 2
    np.testing.assert_allclose(out, [1.5, 3.0, 3.0, 0.0], rtol=1e-15)


def test_order_dependence(oracle):
    # a = 0 deg, b = 80 deg, c = 160 deg, tau = 0.9 (accept iff angle <= ~84.3 deg)
    def v(deg):
        return np.array([math.cos(math.radians(deg)), math.sin(math.radians(deg))], f32)
    a, b, c_ = v(0), v(80), v(160)
    # order a,b,c: b accepted (80), sum at 40 deg, c at 120 from it -> rejected
    _, m1, _, c1 = oracle.aggregate([a, b, c_], 0.9)
    # order b,a,c: a accepted, sum at 40 deg -> c rejected; order b,c,a: c accepted (80),
    # sum at 120 deg, a at 120 from it -> rejected
    _, m2, _, c2 = oracle.aggregate([b, c_, a], 0.9)
    # order a,c,b: c rejected (160), b accepted
    _, m3, _, c3 = oracle.aggregate([a, c_, b], 0.9)
    assert m1.tolist() == [1, 1, 0] and m2.tolist() == [1, 1, 0] and m3.tolist() == [1, 0, 1]
    assert (c1, c2, c3) == (2, 2, 2)


def test_fig2_worked_example(oracle):
    rows, length = {}, None
    with open(os.path.join(HERE, "golden", "fig2_arrows.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].split()
            if not line:
                continue
            if line[0] == "length":
                length = float(line[1])
            else:
                rows[line[0]] = (line[1], [float(x) for x in line[2:]])
    assert length == 2.0 and set(rows) == {"aligned", "misaligned"}

    def arrow(deg):
        return np.array([length * math.cos(math.radians(deg)), length * math.sin(math.radians(deg))], f32)

    def expect(d1, d2):           # trigonometric closed form, independent of Eq. 4's dot-product form
        return 1 - math.cos(math.radians(d1 - d2))

    for name, (claim, angles) in rows.items():
        g = [arrow(a) for a in angles]
        D, _ = oracle.pairwise(g)
        for i in range(3):
            for j in range(3):
                if i != j:
                    assert abs(D[i, j] - expect(angles[i], angles[j])) < 3e-7
                    assert (D[i, j] < 1) if claim == "lt1" else (D[i, j] >= 1)
        out, mask, dist, c = oracle.aggregate(g, f32(0.97))
        if claim == "lt1":
            # both accepted; the third is measured against the sum of two equal-length
            # arrows, which points along their bisector
            bis = 0.5 * (angles[0] + angles[1])
            assert mask.tolist() == [1, 1, 1] and c == 3
            assert abs(dist[1] - expect(angles[1], angles[0])) < 3e-7
            assert abs(dist[2] - expect(angles[2], bis)) < 3e-7
            mean = np.mean(np.stack(g).astype(np.float64), axis=0)
            np.testing.assert_allclose(out, mean, rtol=1e-14)
        else:
            assert mask.tolist() == [1, 0, 0] and c == 1
            assert abs(dist[1] - expect(angles[1], angles[0])) < 3e-7
            assert abs(dist[2] - expect(angles[2], angles[0])) < 3e-7   # sum is still the seed
            np.testing.assert_array_equal(out, g[0].astype(np.float64))


def test_step_matches_aggregate(oracle):
    w, grads = wl.generate("streaming", 5, P=50_021)
    a = oracle_arrays(grads)
    out, mask, dist, c = oracle.aggregate(a, f32(w.tau))
    s = np.full(w.P, np.nan)       # contents before the seed must not matter
    cnt = 0
    for i, g in enumerate(a):
        d, acc, cnt = oracle.step(s, cnt, g, f32(w.tau))
        assert acc == mask[i] and abs(d - dist[i]) < 1e-13   # OpenMP combines thread sums in any order
    assert cnt == c
    np.testing.assert_allclose(s / cnt, out, rtol=1e-15)


# ------------------------------------------------------- pairwise -----------
def test_pairwise_properties_and_gram_consistency(oracle):
    w, grads = wl.generate("diagnostic", 1, P=20_011, N=24)
    a = oracle_arrays(grads)
    D, G = oracle.pairwise(a)
    assert np.array_equal(D, D.T) and np.all(np.diag(D) == 0.0)
    assert D.min() >= 0.0 and D.max() <= 2.0
    X = np.stack(a).astype(np.float64)
    # BLAS contraction. Two summation orders of an inner product differ by a multiple of
    # eps |x|.|y| (not of the result, which cancellation can make small): bound by |x| |y|.
    nrm = np.sqrt(np.diag(G))
    assert np.all(np.abs(G - X @ X.T) <= 1e-13 * np.outer(nrm, nrm))
    out, mask, dist, c = oracle.aggregate(a, f32(w.tau))
    # the sequential distances follow from G alone: with A the accepted set so far,
    # g_i . sum = sum_{j in A} G_ij, |sum|^2 = sum_{j,k in A} G_jk, |g_i|^2 = G_ii
    A = [0]
    for i in range(1, len(a)):
        dot = G[i, A].sum(); nn = G[np.ix_(A, A)].sum()
        d = 1 - dot / math.sqrt(nn * G[i, i])
        assert abs(d - dist[i]) < 1e-12
        if mask[i]:
            A.append(i)
    assert len(A) == c
    # until something besides the seed is accepted, the sequential distance is D[0, j]
    first = int(np.argmax(mask[1:])) + 1
    np.testing.assert_allclose(dist[1:first + 1], D[0, 1:first + 1], rtol=0, atol=1e-14)


# ------------------------------------------- generator statistics -----------
def _expected_cos(w, accepted, i):
    """E cos(g_i, sum_{j in A} g_j) under g = a (s sqrt(rho) c + sqrt(1-rho) z)."""
    S = sum(w.scale[j] * w.sign[j] * math.sqrt(w.rho[j]) for j in accepted)
    var = sum(w.scale[j] ** 2 * (1 - w.rho[j]) for j in accepted)
    return w.sign[i] * math.sqrt(w.rho[i]) * S / math.sqrt(var + S * S)


@pytest.mark.parametrize("name,P", [("tiny", None), ("resnet18", 400_000), ("streaming", 400_000)])
def test_generator_closed_form(oracle, name, P):
    w, grads = wl.generate(name, 0, P=P)
    out, mask, dist, c = oracle.aggregate(oracle_arrays(grads), f32(w.tau))
    tol = 5 / math.sqrt(w.P)
    A = [0]
    for i in range(1, w.N):
        assert abs((1 - dist[i]) - _expected_cos(w, A, i)) < tol, (i, dist[i])
        if mask[i]:
            A.append(i)
    if name == "tiny":
        assert mask.tolist() == [1, 1, 0, 1] and c == 3
        np.testing.assert_allclose(dist, [0, 0.700, 1.372, 0.628], atol=4e-3)
    if name == "streaming":
        assert 0.25 * w.N <= c <= 0.75 * w.N and np.all(np.abs(dist[1:] - 1) < 0.06)


def test_large_and_diagnostic_expectations(oracle):
    w, grads = wl.generate("large", 0, P=400_000)
    out, mask, dist, c = oracle.aggregate(oracle_arrays(grads), f32(w.tau))
    # accepted exactly those sharing the seed's sign (rho = 0.1: D ~ 0.9 / 1.1 and beyond)
    assert mask.tolist() == [1 if s == w.sign[0] else 0 for s in w.sign]
    w, grads = wl.generate("diagnostic", 0, P=200_000)
    out, mask, dist, c = oracle.aggregate(oracle_arrays(grads), f32(w.tau))
    assert mask.tolist() == [1 if k == 0 else 0 for k in w.cluster] and c == 16
    # same cluster, m members accepted so far: D = 1 - 0.36 m / sqrt(0.64 m + 0.36 m^2)
    m = 0
    for i in range(1, w.N):
        if w.cluster[i] == 0:
            m += 1
            assert abs(dist[i] - (1 - 0.36 * m / math.sqrt(0.64 * m + 0.36 * m * m))) < 0.012
        elif w.cluster[i] in (1, 3):
            assert abs(dist[i] - 1.0) < 0.012
    assert abs(dist[2] - (1 + 0.36 / math.sqrt(1.25))) < 0.012   # anti-aligned cluster vs the seed


def test_bf16_widening_is_exact(oracle):
    import torch
    t = torch.randn(4099, generator=torch.Generator().manual_seed(7)).to(torch.bfloat16)
    u = wl.to_host_array(t)
    assert u.dtype == np.uint16
    ref = t.to(torch.float64).numpy()
    out, mask, dist, c = oracle.aggregate([u], 1.0)
    np.testing.assert_array_equal(out, ref)
    v = wl.to_host_array((t * 3).to(torch.bfloat16))
    x, y = ref, (t * 3).to(torch.bfloat16).to(torch.float64).numpy()
    d = 1 - (x @ y) / (np.linalg.norm(x) * np.linalg.norm(y))
    assert abs(oracle.cosine_distance(u, v) - d) < 1e-13


# ------------------------------ exact rational arithmetic on tiny inputs -----
# Algorithm 1 decided without any rounding: small integer vectors, every inner
# product an integer, and "1 - a/sqrt(b) <= tau" settled by comparing squares of
# rationals (no square root is ever taken). The mean is an exact fraction.
def _exact_accepts(a, b, tau):
    """Is 1 - a / sqrt(b) <= tau, for integers a, b >= 0 and a Fraction tau? (b = 0: the
    zero-norm reading, D = 1.) Returns None when the two sides are exactly equal."""
    from fractions import Fraction
    if b == 0:
        return Fraction(1) <= tau
    t = 1 - tau                       # accept iff t * sqrt(b) <= a
    if a == 0 and t == 0:
        return True                   # D is exactly 1 = tau in any arithmetic: the tie accepts
    lhs2, rhs2 = t * t * b, Fraction(a * a)
    if lhs2 == rhs2 and (t >= 0) == (a >= 0):
        return None
    if t >= 0:
        return a >= 0 and lhs2 <= rhs2
    return a >= 0 or lhs2 >= rhs2


def _exact_filter(rows, tau, order):
    from fractions import Fraction
    seed = order[0]
    total = list(rows[seed])
    accepted = [seed]
    for i in order[1:]:
        a = sum(x * y for x, y in zip(total, rows[i]))
        b = sum(x * x for x in total) * sum(y * y for y in rows[i])
        ok = _exact_accepts(a, b, tau)
        if ok is None:
            return None               # an exact tie: not a case for a floating-point comparison
        if ok:
            accepted.append(i)
            total = [x + y for x, y in zip(total, rows[i])]
    return accepted, [Fraction(x, len(accepted)) for x in total]


def test_exact_rational_brute_force(oracle):
    from fractions import Fraction
    rng = np.random.default_rng(77)
    checked = rejected_some = accepted_some = 0
    for trial in range(400):
        N, P = int(rng.integers(2, 7)), int(rng.integers(1, 7))
        rows = rng.integers(-4, 5, size=(N, P)).tolist()
        tau32 = f32(rng.choice([0.5, 0.9, 0.97, 1.0, 1.03, 1.3, 1.9]))
        tau = Fraction(float(tau32))                      # the binary32 value, exactly
        exact = _exact_filter(rows, tau, list(range(N)))
        if exact is None:
            continue
        accepted, mean = exact
        out, mask, dist, c = oracle.aggregate([np.array(r, dtype=f32) for r in rows], tau32)
        # skip the rare case where a distance is within rounding of tau without being 1 = tau exactly
        near = np.abs(dist[1:] - float(tau32)) < 1e-12
        if np.any(near & ~((dist[1:] == 1.0) & (float(tau32) == 1.0))):
            continue
        assert [i for i in range(N) if mask[i]] == accepted, (rows, float(tau32))
        assert c == len(accepted)
        np.testing.assert_allclose(out, [float(m) for m in mean], rtol=1e-15, atol=1e-300)
        checked += 1
        rejected_some += c < N
        accepted_some += c > 1
    assert checked > 300 and rejected_some > 50 and accepted_some > 50
