"""Pins for the oracle's versions of the paper's follow-on items: the
order-indifferent seed choice (Sec. 3.1, last paragraph), the GAF-SGD step with
skip (Algorithm 1, Eq. 6, Sec. 4.1's optimizer) and bucketed filtering
(future research). Expected values: hand-worked cases, limiting cases that
reduce to the plain filter or to plain SGD, and brute force through the
already pinned plain filter."""
import math

import numpy as np

from conftest import oracle_arrays
from paper_2412_18052_amd import workloads as wl

f32 = np.float32


def v2(deg, r=1.0):
    return np.array([r * math.cos(math.radians(deg)), r * math.sin(math.radians(deg))], f32)


# ------------------------------------------------------------ best seed -----
def test_best_seed_rescues_orthogonal_seed(oracle):
    # the paper's degenerate example: the first gradient is orthogonal to all others, so the
    # plain filter keeps only the seed; with every gradient taking a turn as seed the three
    # agreeing ones win
    e = np.eye(5, dtype=f32)
    g = [e[0], e[1] + e[2], e[1] + e[2] + f32(0.1) * e[3], e[1] + e[2] - f32(0.1) * e[3]]
    _, mask0, _, c0 = oracle.aggregate(g, 0.5)
    assert c0 == 1 and mask0.tolist() == [1, 0, 0, 0]
    out, mask, dist, c, seed, counts = oracle.best_seed(g, 0.5)
    assert counts.tolist() == [1, 3, 3, 3]          # seeds 1..3 each collect the other two
    assert seed == 1 and c == 3 and mask.tolist() == [0, 1, 1, 1]   # tie -> lowest seed index
    mean = (g[1].astype(np.float64) + g[2] + g[3]) / 3
    np.testing.assert_allclose(out, mean, rtol=1e-15)
    assert dist[1] == 0.0 and dist[0] == 1.0        # g_0 is visited last, orthogonal to the sum


def test_best_seed_ring_order_by_hand(oracle):
    # angles 0, 80, 160, 200 deg, tau = 0.9 (accept iff angle to the running sum <= 84.26 deg)
    # seed 0:   80 ok (sum 40), 160 (120) no, 200 (160) no              -> c = 2
    # seed 80:  160 ok (sum 120), 200 (80) ok (sum: three unit vectors at 80,160,200 -> angle 150),
    #           0 (150) no                                               -> c = 3
    # seed 160: 200 ok (sum 180), 0 (180) no, 80 (100) no               -> c = 2
    # seed 200: 0 (160) no, 80 (120) no, 160 (40) ok                    -> c = 2
    g = [v2(0), v2(80), v2(160), v2(200)]
    out, mask, dist, c, seed, counts = oracle.best_seed(g, 0.9)
    assert counts.tolist() == [2, 3, 2, 2] and seed == 1 and c == 3
    assert mask.tolist() == [0, 1, 1, 1]
    assert abs(dist[2] - (1 - math.cos(math.radians(80)))) < 3e-7
    assert abs(dist[3] - (1 - math.cos(math.radians(80)))) < 3e-7     # 200 deg against the sum at 120 deg
    np.testing.assert_allclose(out, (g[1].astype(np.float64) + g[2] + g[3]) / 3, rtol=1e-15)


def test_best_seed_equals_plain_filter_on_the_winning_rotation(oracle):
    w, grads = wl.generate("streaming", 3, P=30_011, N=9)
    a = oracle_arrays(grads)
    out, mask, dist, c, seed, counts = oracle.best_seed(a, f32(w.tau))
    for s in range(w.N):                             # brute force through the pinned plain filter
        ring = [a[(s + k) % w.N] for k in range(w.N)]
        o, m, d, cc = oracle.aggregate(ring, f32(w.tau))
        assert cc == counts[s]
        if s == seed:
            np.testing.assert_allclose(out, o, rtol=1e-13)
            assert [m[(i - s) % w.N] for i in range(w.N)] == mask.tolist()
            np.testing.assert_allclose([d[(i - s) % w.N] for i in range(w.N)], dist, atol=1e-13)
    assert c == counts.max() and seed == int(np.argmax(counts))
    # everything admitted: every seed ties at N, seed 0 wins, result is the plain mean
    out, mask, dist, c, seed, counts = oracle.best_seed(a, 2.0)
    assert seed == 0 and c == w.N and counts.tolist() == [w.N] * w.N
    np.testing.assert_allclose(out, np.mean(np.stack(a).astype(np.float64), axis=0), rtol=1e-12, atol=1e-15)


# -------------------------------------------------------------- GAF-SGD -----
def test_sgd_step_by_hand_and_skip(oracle):
    theta = np.array([1.0, -2.0, 0.5]); v = np.zeros(3); g = np.array([0.5, 0.25, -1.0])
    # plain gradient step when mu = wd = 0 (Eq. 6)
    oracle.sgd_step(theta, v, g, 2, 0.1, 0.0, 0.0)
    np.testing.assert_allclose(theta, [0.95, -2.025, 0.6], rtol=1e-15)
    np.testing.assert_allclose(v, g, rtol=0)
    # second step with momentum 0.9 and weight decay 0.01, worked by hand:
    # d = g + 0.01 theta; v = 0.9 v + d; theta -= 0.1 v
    t0 = theta.copy(); v0 = v.copy()
    oracle.sgd_step(theta, v, g, 3, 0.1, 0.9, 0.01)
    d = g + 0.01 * t0; v1 = 0.9 * v0 + d
    np.testing.assert_allclose(v, v1, rtol=1e-15)
    np.testing.assert_allclose(theta, t0 - 0.1 * v1, rtol=1e-15)
    assert abs(v[0] - (0.9 * 0.5 + 0.5 + 0.0095)) < 1e-15
    # c == 1: no consensus, nothing moves (Algorithm 1's skip)
    t1 = theta.copy(); v2_ = v.copy()
    oracle.sgd_step(theta, v, g, 1, 0.1, 0.9, 0.01)
    assert np.array_equal(theta, t1) and np.array_equal(v, v2_)


# ------------------------------------------------------------- bucketed -----
def test_bucketed_by_hand(oracle):
    # two buckets of 2 coordinates; in bucket 0 the second gradient agrees with the seed, in
    # bucket 1 it opposes it
    g = [np.array([1, 0, 1, 0], f32), np.array([1, 1, -1, 0], f32), np.array([0, 1, 1, 1], f32)]
    out, mask, dist, count = oracle.bucketed(g, 0.5, [0, 2, 4])
    # bucket 0: (1,0); (1,1): D = 1 - 1/sqrt2 = .2929 ok, sum (2,1); (0,1): cos = 1/sqrt5, D = .5528 no
    # bucket 1: (1,0); (-1,0): D = 2 no; (1,1): D = .2929 ok
    assert mask.tolist() == [[1, 1, 0], [1, 0, 1]] and count.tolist() == [2, 2]
    assert abs(dist[0, 2] - (1 - 1 / math.sqrt(5))) < 1e-15 and abs(dist[1, 1] - 2.0) < 1e-15
    np.testing.assert_allclose(out, [1.0, 0.5, 1.0, 0.5], rtol=1e-15)


def test_bucketed_reduces_to_plain_and_to_slices(oracle):
    w, grads = wl.generate("resnet18", 2, P=40_009)
    a = oracle_arrays(grads)
    o0, m0, d0, c0 = oracle.aggregate(a, f32(w.tau))
    out, mask, dist, count = oracle.bucketed(a, f32(w.tau), [0, w.P])       # one bucket = the plain filter
    np.testing.assert_allclose(out, o0, rtol=1e-13)
    assert mask[0].tolist() == m0.tolist() and count[0] == c0
    offs = [0, 8, 1000, 17_016, w.P]
    out, mask, dist, count = oracle.bucketed(a, f32(w.tau), offs)
    for b in range(4):                                # each bucket = the plain filter on the slices
        o, m, d, c = oracle.aggregate([x[offs[b]:offs[b + 1]] for x in a], f32(w.tau))
        np.testing.assert_allclose(out[offs[b]:offs[b + 1]], o, rtol=1e-13)
        assert mask[b].tolist() == m.tolist() and count[b] == c
        np.testing.assert_allclose(dist[b], d, atol=1e-13)


def test_best_seed_and_buckets_against_exact_rational_filter(oracle):
    """The two variants against the rounding-free filter of test_oracle_pins (integer vectors,
    comparisons on squares of rationals): every ring rotation, every bucket."""
    from fractions import Fraction
    from test_oracle_pins import _exact_filter
    rng = np.random.default_rng(78)
    checked = 0
    for trial in range(200):
        N, P = int(rng.integers(2, 6)), int(rng.integers(2, 9))
        rows = rng.integers(-4, 5, size=(N, P)).tolist()
        tau32 = np.float32(rng.choice([0.9, 0.97, 1.0, 1.03, 1.3]))
        tau = Fraction(float(tau32))
        arrs = [np.array(r, dtype=np.float32) for r in rows]
        # order-indifferent: all N rotations, largest count, lowest seed on ties
        runs = [_exact_filter(rows, tau, [(s + k) % N for k in range(N)]) for s in range(N)]
        out, mask, dist, c, seed, counts = oracle.best_seed(arrs, tau32)
        d_all = np.array([oracle.aggregate([arrs[(s + k) % N] for k in range(N)], tau32)[2][1:] for s in range(N)])
        near = np.any((np.abs(d_all - float(tau32)) < 1e-12) & ~((d_all == 1.0) & (float(tau32) == 1.0)))
        if all(r is not None for r in runs) and not near:
            best = max(range(N), key=lambda s: (len(runs[s][0]), -s))
            assert counts.tolist() == [len(r[0]) for r in runs]
            assert seed == best and c == len(runs[best][0])
            assert sorted(i for i in range(N) if mask[i]) == sorted(runs[best][0])
            np.testing.assert_allclose(out, [float(m) for m in runs[best][1]], rtol=1e-15, atol=1e-300)
            checked += 1
        # buckets: a cut at a random interior point, each side filtered on its own
        cut = int(rng.integers(1, P))
        parts = [_exact_filter([r[:cut] for r in rows], tau, list(range(N))),
                 _exact_filter([r[cut:] for r in rows], tau, list(range(N)))]
        bout, bmask, bdist, bcount = oracle.bucketed(arrs, tau32, [0, cut, P])
        bnear = (np.abs(bdist[:, 1:] - float(tau32)) < 1e-12) & ~((bdist[:, 1:] == 1.0) & (float(tau32) == 1.0))
        if all(p is not None for p in parts) and not np.any(bnear):
            for b, (acc, mean) in enumerate(parts):
                assert [i for i in range(N) if bmask[b, i]] == acc and bcount[b] == len(acc)
            np.testing.assert_allclose(bout, [float(m) for p in parts for m in p[1]], rtol=1e-15, atol=1e-300)
            checked += 1
    assert checked > 250
