"""Property tests of the CPU oracle on random small inputs (hypothesis): statements that hold
for every input by the definitions in the paper (Eq. 2, Eq. 4, Eq. 5, Algorithm 1), checked
without re-typing the oracle's arithmetic. Comparisons between two oracle results allow 1e-14:
its OpenMP reductions do not fix the order in which the threads' partial sums are combined."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st
from hypothesis.extra import numpy as hnp

f32 = np.float32
finite = st.floats(min_value=-8.0, max_value=8.0, allow_nan=False, allow_infinity=False, width=32)


def batches(min_n=1, max_n=6, min_p=1, max_p=9):
    return st.integers(min_n, max_n).flatmap(
        lambda n: st.integers(min_p, max_p).flatmap(
            lambda p: hnp.arrays(np.float32, (n, p), elements=finite)))


@pytest.fixture(scope="module")
def orc(oracle):
    return oracle


@settings(max_examples=150, deadline=None, derandomize=True)
@given(b=batches(min_n=2, max_n=2))
def test_distance_range_symmetry_negation_scaling(orc, b):
    x, y = b[0], b[1]
    d = orc.cosine_distance(x, y)
    if not np.any(x) or not np.any(y):
        assert d == 1.0                                  # zero norm: defined as exactly 1
        return
    assert -1e-12 <= d <= 2.0 + 1e-12                    # Sec. 1: the range of the cosine distance
    assert abs(d - orc.cosine_distance(y, x)) < 1e-14
    assert abs(orc.cosine_distance(x, -y) - (2.0 - d)) < 1e-12
    assert abs(orc.cosine_distance(f32(4.0) * x, f32(2.0) * y) - d) < 1e-14   # exact rescaling (upwards: no underflow)
    assert abs(orc.cosine_distance(x, x)) < 1e-12


@settings(max_examples=150, deadline=None, derandomize=True)
@given(b=batches(), tau=st.sampled_from([0.3, 0.9, 0.97, 1.0, 1.05, 1.5]))
def test_aggregate_invariants(orc, b, tau):
    grads = [np.ascontiguousarray(r) for r in b]
    out, mask, dist, c = orc.aggregate(grads, f32(tau))
    assert mask[0] == 1 and dist[0] == 0.0               # the seed
    assert c == int(mask.sum()) and 1 <= c <= len(grads)
    # Eq. 5: the result is the plain mean (Eq. 2) of exactly the accepted gradients
    acc = [g for g, m in zip(grads, mask) if m]
    np.testing.assert_allclose(out, orc.plain_average(acc), rtol=1e-14, atol=1e-300)
    np.testing.assert_allclose(out, np.mean(np.stack(acc).astype(np.float64), axis=0), rtol=1e-13, atol=1e-300)
    # Algorithm 1: every decision is "distance <= tau" for the reported distance (NaN rejects)
    for i in range(1, len(grads)):
        assert bool(mask[i]) == bool(dist[i] <= float(f32(tau)))
    # the distance of the first visited gradient is the pairwise one to the seed
    if len(grads) > 1:
        assert abs(dist[1] - orc.cosine_distance(grads[1], grads[0])) < 1e-14
    # a rejected gradient leaves no trace: dropping it changes nothing for the others
    keep = [i for i in range(len(grads)) if mask[i]]
    out2, mask2, dist2, c2 = orc.aggregate([grads[i] for i in keep], f32(tau))
    assert c2 == c and np.all(mask2 == 1)
    np.testing.assert_allclose(out2, out, rtol=1e-14, atol=1e-300)
    np.testing.assert_allclose(dist2, dist[keep], rtol=0, atol=1e-14)


@settings(max_examples=100, deadline=None, derandomize=True)
@given(b=batches(min_n=2))
def test_threshold_limits(orc, b):
    grads = [np.ascontiguousarray(r) for r in b]
    # tau above 2 admits everything: plain averaging (Sec. 4.1); tau below 0 admits nothing but the seed
    out, mask, _, c = orc.aggregate(grads, f32(2.001))
    if all(np.any(g) for g in grads):
        assert c == len(grads)
        np.testing.assert_allclose(out, np.mean(b.astype(np.float64), axis=0), rtol=1e-13, atol=1e-300)
    out, mask, _, c = orc.aggregate(grads, f32(-0.001))
    assert c == 1 and np.array_equal(out, grads[0].astype(np.float64))


@settings(max_examples=100, deadline=None, derandomize=True)
@given(b=batches(min_n=2, max_n=5, min_p=2))
def test_pairwise_matches_pairs_and_best_seed_matches_rotations(orc, b):
    grads = [np.ascontiguousarray(r) for r in b]
    N = len(grads)
    D, G = orc.pairwise(grads)
    for i in range(N):
        for j in range(N):
            if i != j:
                assert abs(D[i, j] - orc.cosine_distance(grads[i], grads[j])) < 1e-14
    np.testing.assert_allclose(G, b.astype(np.float64) @ b.astype(np.float64).T, rtol=0,
                               atol=1e-13 * max(1.0, float(np.abs(G).max())))
    tau = f32(0.97)
    out, mask, dist, c, seed, counts = orc.best_seed(grads, tau)
    runs = [orc.aggregate([grads[(s + k) % N] for k in range(N)], tau) for s in range(N)]
    assert counts.tolist() == [r[3] for r in runs]
    best = max(range(N), key=lambda s: (runs[s][3], -s))
    assert seed == best and c == runs[best][3]
    np.testing.assert_allclose(out, runs[best][0], rtol=1e-14, atol=1e-300)
    assert [int(mask[(best + k) % N]) for k in range(N)] == runs[best][1].tolist()
