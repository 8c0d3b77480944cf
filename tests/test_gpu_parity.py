"""Parity of the HIP library (through its C ABI) against the CPU oracle.

Bars: accept masks and counts bit-exact; cosine distances within 1e-6
absolute; macro-gradient within 1e-5 relative L2 (binary32 inputs) or 2e-3
(bfloat16 inputs). Every generated case keeps each distance at least 1e-3 away
from tau, so the decisions cannot flip on rounding.
"""
import ctypes
import math

import numpy as np
import pytest
import torch

from conftest import MARGIN, oracle_arrays, workload_with_margin
from paper_2412_18052_amd import gaf
from paper_2412_18052_amd import workloads as wl

pytestmark = pytest.mark.gpu

DIST_ATOL = 1e-6
OUT_RTOL = {"f32": 1e-5, "bf16": 2e-3}
TILE = 256 * 4 * 4          # elements one workgroup handles per tile


# Every test runs under both schedules of gaf_aggregate: "sequential" (one fused
# streaming pass per gradient) and "auto" (Gram-first for N <= 64, the default).
@pytest.fixture(scope="module", params=["sequential", "auto"])
def ctx(request):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = gaf.gaf_create(max_P=1 << 31, max_N=256)
    gaf.gaf_set_schedule(c, request.param)
    c.schedule_name = request.param
    yield c
    torch.cuda.synchronize()
    gaf.gaf_destroy(c)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a - b)


def check_against_oracle(res_gpu, res_oracle, dtype):
    out, mask, dist, count = res_gpu
    torch.cuda.synchronize()
    o_out, o_mask, o_dist, o_count = res_oracle
    assert mask.cpu().numpy().tolist() == o_mask.tolist()
    assert int(count.item()) == o_count
    d = dist.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(d - o_dist)) <= DIST_ATOL, (d, o_dist)
    out_h = out.cpu().numpy()
    assert rel_l2(out_h, o_out) <= OUT_RTOL[dtype]
    # Element by element as well (a relative L2 norm would not notice a few wrong elements or one
    # wrong tile among thousands). Both the running mean and the masked mean add c <= N values in
    # binary32: each element is off by at most about (c + 2) 2^-24 of the largest partial sum,
    # which is of the size of the largest output; a wrong element is off by the size of an input.
    bound = 8.0 * (len(o_mask) + 2) * 2.0 ** -24 * np.max(np.abs(o_out))
    worst = np.max(np.abs(out_h.astype(np.float64) - o_out)) if out_h.size else 0.0
    assert worst <= bound, (worst, bound)


def run_aggregate(ctx, oracle, grads_host, tau, dtype="f32"):
    dev = [g.cuda() for g in grads_host]
    res = gaf.gaf_aggregate(ctx, dev, tau)
    ref = oracle.aggregate(oracle_arrays(grads_host), np.float32(tau))
    check_against_oracle(res, ref, dtype)
    return res, ref


# ------------------------------------------------------------ named configs --
def test_tiny_full(ctx, oracle):
    w, grads, ref = workload_with_margin("tiny")
    res = gaf.gaf_aggregate(ctx, [g.cuda() for g in grads], w.tau)
    check_against_oracle(res, ref, w.dtype)
    assert ref[1].tolist() == [1, 1, 0, 1]


def test_resnet18_full(ctx, oracle):
    w, grads, ref = workload_with_margin("resnet18")
    assert w.P == 11_220_132 and w.N == 8
    res = gaf.gaf_aggregate(ctx, [g.cuda() for g in grads], w.tau)
    check_against_oracle(res, ref, w.dtype)


def test_streaming_full(ctx, oracle):
    w, grads, ref = workload_with_margin("streaming")
    assert w.P == 11_220_132 and w.N == 32
    accum = torch.full((w.P,), float("nan"), device="cuda")   # contents before the seed are ignored
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(w.N, device="cuda"); mask = torch.empty(w.N, dtype=torch.uint8, device="cuda")
    for i, g in enumerate(grads):
        gaf.gaf_step(ctx, accum, count, g.cuda(), w.tau, dist[i:i + 1], mask[i:i + 1])
    check_against_oracle((accum, mask, dist, count), ref, w.dtype)
    assert 0.25 * w.N <= ref[3] <= 0.75 * w.N


def test_large_scaled_bf16(ctx, oracle):
    w, grads, ref = workload_with_margin("large", P=5 * TILE * 7 + 1234 + 3)
    res = gaf.gaf_aggregate(ctx, [g.cuda() for g in grads], w.tau)
    check_against_oracle(res, ref, w.dtype)
    # the streaming entry point on the same bf16 data
    accum = torch.empty(w.P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(w.N, device="cuda"); mask = torch.empty(w.N, dtype=torch.uint8, device="cuda")
    for i, g in enumerate(grads):
        gaf.gaf_step(ctx, accum, count, g.cuda(), w.tau, dist[i:i + 1], mask[i:i + 1])
    check_against_oracle((accum, mask, dist, count), ref, w.dtype)


def test_diagnostic_scaled(ctx, oracle):
    w, grads, ref = workload_with_margin("diagnostic", P=1_500_007)
    dev = [g.cuda() for g in grads]
    res = gaf.gaf_aggregate(ctx, dev, w.tau)
    check_against_oracle(res, ref, w.dtype)
    gram = torch.empty((w.N, w.N), dtype=torch.float64, device="cuda")
    D = gaf.gaf_pairwise(ctx, dev, gram=gram)
    torch.cuda.synchronize()
    oD, oG = oracle.pairwise(oracle_arrays(grads))
    Dh = D.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(Dh - oD)) <= DIST_ATOL
    assert np.array_equal(Dh, Dh.T) and np.all(np.diag(Dh) == 0)
    np.testing.assert_allclose(gram.cpu().numpy(), oG, rtol=0, atol=2e-7 * w.P)
    # first row of the matrix = sequential distances until the first acceptance
    first = int(np.argmax(ref[1][1:])) + 1
    assert np.max(np.abs(Dh[0, 1:first + 1] - ref[2][1:first + 1])) <= DIST_ATOL
    # the filter replayed on the matrix gaf_pairwise has just written
    res2 = gaf.gaf_aggregate_with_gram(ctx, dev, w.tau, gram)
    check_against_oracle(res2, ref, w.dtype)
    # matrix and filter from one call
    gram3 = torch.empty_like(gram)
    res3 = gaf.gaf_aggregate_with_matrix(ctx, dev, w.tau, gram=gram3)
    check_against_oracle(res3[:4], ref, w.dtype)
    assert torch.equal(res3[4], D) and torch.equal(gram3, gram)


# ------------------------------------------------------------ shapes / tails --
@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 7, 63, 64, 255, 1023, 1025, TILE - 1, TILE, TILE + 1,
                               3 * TILE + 5, 2049 * TILE + 9])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_sizes(ctx, oracle, P, dtype):
    g = torch.Generator().manual_seed(P)
    base = torch.randn(P, generator=g)
    grads = []
    for s, r in [(1, 0.0), (1, 0.5), (-1, 0.5), (1, 0.3), (1, 0.0)]:
        v = s * math.sqrt(r) * base + math.sqrt(1 - r) * torch.randn(P, generator=g)
        if r == 0.0 and len(grads) == 0:
            v = base.clone()
        grads.append(v.to(torch.bfloat16) if dtype == "bf16" else v)
    tau = 0.9
    arr = oracle_arrays(grads)
    ref = oracle.aggregate(arr, np.float32(tau))
    if np.any(np.abs(ref[2][1:] - np.float32(tau)) < MARGIN):
        tau = 0.9 + 4 * MARGIN if np.all(np.abs(ref[2][1:] - np.float32(0.9 + 4 * MARGIN)) >= MARGIN) else 1.5
        ref = oracle.aggregate(arr, np.float32(tau))
        assert np.all(np.abs(ref[2][1:] - np.float32(tau)) >= MARGIN)
    res = gaf.gaf_aggregate(ctx, [x.cuda() for x in grads], tau)
    check_against_oracle(res, ref, dtype)
    # streaming on the same data
    accum = torch.empty(P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(5, device="cuda"); mask = torch.empty(5, dtype=torch.uint8, device="cuda")
    for i, x in enumerate(grads):
        gaf.gaf_step(ctx, accum, count, x.cuda(), tau, dist[i:i + 1], mask[i:i + 1])
    check_against_oracle((accum, mask, dist, count), ref, dtype)


@pytest.mark.parametrize("N", [1, 2, 3])
def test_small_N(ctx, oracle, N):
    g = torch.Generator().manual_seed(N)
    grads = [torch.randn(70_001, generator=g) for _ in range(N)]
    for tau in (2.0, -0.5):
        run_aggregate(ctx, oracle, grads, tau)


@pytest.mark.parametrize("N", [2, 4, 5, 7, 8, 9, 16, 17, 31, 48, 49, 64])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_batch_sizes(ctx, oracle, N, dtype):
    # every kernel variant of the batch call: vector-ALU Gram (N <= 8), 1..4 row groups of the
    # matrix-core Gram, ragged P
    P = 150_001 + 1000 * N
    name = "large" if dtype == "bf16" else "resnet18"
    w, grads, ref = workload_with_margin(name, P=P, N=N, seed=N)
    dev = [g.cuda() for g in grads]
    res = gaf.gaf_aggregate(ctx, dev, w.tau)
    check_against_oracle(res, ref, dtype)
    gram = torch.empty((N, N), dtype=torch.float64, device="cuda")
    D = gaf.gaf_pairwise(ctx, dev, gram=gram)
    res2 = gaf.gaf_aggregate_with_gram(ctx, dev, w.tau, gram)
    check_against_oracle(res2, ref, dtype)
    oD, oG = oracle.pairwise(oracle_arrays(grads))
    assert np.max(np.abs(D.cpu().numpy().astype(np.float64) - oD)) <= DIST_ATOL


# ------------------------------------------------------- limiting cases -------
def test_tau_limits(ctx, oracle):
    w, grads = wl.generate("resnet18", 3, P=200_003)
    (out, mask, dist, count), ref = run_aggregate(ctx, oracle, grads, 2.0)
    assert mask.cpu().tolist() == [1] * w.N and int(count.item()) == w.N
    mean = oracle.plain_average(oracle_arrays(grads))            # Eq. 2
    assert rel_l2(out.cpu().numpy(), mean) <= 1e-5
    (out, mask, dist, count), ref = run_aggregate(ctx, oracle, grads, -1e-3)
    assert mask.cpu().tolist() == [1] + [0] * (w.N - 1) and int(count.item()) == 1
    assert torch.equal(out.cpu(), grads[0])


def test_identical_negated_orthogonal(ctx, oracle):
    P = 100_000
    x = torch.randn(P, generator=torch.Generator().manual_seed(1))
    a = torch.zeros(P); b = torch.zeros(P); a[: P // 2] = x[: P // 2]; b[P // 2:] = x[P // 2:]
    dev = [x.cuda(), x.clone().cuda(), (-x).cuda(), ]
    out, mask, dist, count = gaf.gaf_aggregate(ctx, dev, 0.5)
    torch.cuda.synchronize()
    d = dist.cpu().numpy()
    assert abs(d[1]) < 1e-7 and abs(d[2] - 2.0) < 1e-7 and mask.cpu().tolist() == [1, 1, 0]
    out, mask, dist, count = gaf.gaf_aggregate(ctx, [a.cuda(), b.cuda()], 0.999)
    torch.cuda.synchronize()
    assert dist.cpu().tolist() == [0.0, 1.0] and mask.cpu().tolist() == [1, 0]   # orthogonal: exactly 1
    out, mask, dist, count = gaf.gaf_aggregate(ctx, [a.cuda(), b.cuda()], 1.0)    # tie accepts
    torch.cuda.synchronize()
    assert mask.cpu().tolist() == [1, 1] and int(count.item()) == 2


def test_seed_orthogonal_to_all(ctx, oracle):
    P = 50_000
    g = torch.Generator().manual_seed(2)
    seed = torch.zeros(P); seed[:1000] = torch.randn(1000, generator=g)
    others = []
    for _ in range(4):
        v = torch.zeros(P); v[1000:] = torch.randn(P - 1000, generator=g) + 0.5
        others.append(v)
    (out, mask, dist, count), ref = run_aggregate(ctx, oracle, [seed] + others, 0.97)
    assert int(count.item()) == 1 and mask.cpu().tolist() == [1, 0, 0, 0, 0]
    assert torch.equal(out.cpu(), seed)


def test_zero_vector_and_nan(ctx, oracle):
    P = 33_333
    g = torch.Generator().manual_seed(3)
    x = torch.randn(P, generator=g); y = x + 0.3 * torch.randn(P, generator=g)
    z = torch.zeros(P)
    (out, mask, dist, count), ref = run_aggregate(ctx, oracle, [x, z, y], 0.5)
    assert dist.cpu().numpy()[1] == 1.0 and mask.cpu().tolist() == [1, 0, 1]
    bad = y.clone(); bad[P // 2] = float("nan")
    inf = y.clone(); inf[7] = float("inf")
    dev = [x.cuda(), bad.cuda(), inf.cuda()]
    out, mask, dist, count = gaf.gaf_aggregate(ctx, dev, 2.0)
    torch.cuda.synchronize()
    assert mask.cpu().tolist() == [1, 0, 0] and int(count.item()) == 1
    assert math.isnan(dist.cpu()[1].item()) and math.isnan(dist.cpu()[2].item())
    assert torch.equal(out.cpu(), x)          # aggregate untouched bit for bit
    # streaming: a rejected NaN gradient leaves accum bitwise alone
    accum = x.cuda().clone(); count = torch.ones(1, dtype=torch.int32, device="cuda")
    d1 = torch.empty(1, device="cuda"); m1 = torch.empty(1, dtype=torch.uint8, device="cuda")
    gaf.gaf_step(ctx, accum, count, bad.cuda(), 2.0, d1, m1)
    torch.cuda.synchronize()
    assert torch.equal(accum.cpu(), x) and int(count.item()) == 1 and m1.item() == 0


@pytest.mark.parametrize("N,dtype", [(20, "f32"), (40, "f32"), (40, "bf16")])
def test_nan_and_inf_in_matrix_core_batches(ctx, oracle, N, dtype):
    # a NaN or Inf in one gradient must poison that gradient's distance only
    name = "large" if dtype == "bf16" else "resnet18"
    w, grads, ref = workload_with_margin(name, P=120_011, N=N, seed=N)
    bad = [g.clone() for g in grads]
    bad[3][77] = float("nan")
    bad[N - 2][5] = float("inf")
    clean = [g for i, g in enumerate(grads) if i not in (3, N - 2)]
    ref2 = oracle.aggregate(oracle_arrays(clean), np.float32(w.tau))
    if not np.all(np.abs(ref2[2][1:] - np.float32(w.tau)) >= MARGIN):
        pytest.skip("margin lost after removing two gradients")
    out, mask, dist, count = gaf.gaf_aggregate(ctx, [g.cuda() for g in bad], w.tau)
    torch.cuda.synchronize()
    m = mask.cpu().numpy(); d = dist.cpu().numpy()
    assert m[3] == 0 and m[N - 2] == 0 and math.isnan(d[3]) and math.isnan(d[N - 2])
    keep = [i for i in range(N) if i not in (3, N - 2)]
    assert m[keep].tolist() == ref2[1].tolist() and int(count.item()) == ref2[3]
    assert np.max(np.abs(d[keep].astype(np.float64) - ref2[2])) <= DIST_ATOL
    assert rel_l2(out.cpu().numpy(), ref2[0]) <= OUT_RTOL[dtype]


def test_order_dependence(ctx, oracle):
    w, grads = wl.generate("large", 4, P=300_017)
    order = list(range(w.N))
    first_minus = next(i for i in range(w.N) if w.sign[i] != w.sign[0])
    order[0], order[first_minus] = order[first_minus], order[0]
    (_, m1, _, _), _ = run_aggregate(ctx, oracle, grads, w.tau, "bf16")
    (_, m2, _, _), _ = run_aggregate(ctx, oracle, [grads[i] for i in order], w.tau, "bf16")
    assert m1.cpu().tolist() != m2.cpu().tolist()


def test_deterministic(ctx):
    w, grads = wl.generate("resnet18", 9, P=3_000_001)
    dev = [g.cuda() for g in grads]
    a = gaf.gaf_aggregate(ctx, dev, w.tau)
    b = gaf.gaf_aggregate(ctx, dev, w.tau)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    D1 = gaf.gaf_pairwise(ctx, dev); D2 = gaf.gaf_pairwise(ctx, dev)
    torch.cuda.synchronize()
    assert torch.equal(D1, D2)


def test_streaming_state_is_resumable(ctx, oracle):
    # (accum, count) is the whole state: copy it out, continue elsewhere
    w, grads, ref = workload_with_margin("streaming", P=400_009, N=12)
    accum = torch.empty(w.P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    for g in grads[:6]:
        gaf.gaf_step(ctx, accum, count, g.cuda(), w.tau)
    accum2 = accum.clone(); count2 = count.clone()
    dist = torch.empty(w.N, device="cuda"); mask = torch.empty(w.N, dtype=torch.uint8, device="cuda")
    for i, g in enumerate(grads[6:], start=6):
        gaf.gaf_step(ctx, accum2, count2, g.cuda(), w.tau, dist[i:i + 1], mask[i:i + 1])
    torch.cuda.synchronize()
    assert mask.cpu().numpy()[6:].tolist() == ref[1][6:].tolist()
    assert np.max(np.abs(dist.cpu().numpy()[6:].astype(np.float64) - ref[2][6:])) <= DIST_ATOL
    assert int(count2.item()) == ref[3] and rel_l2(accum2.cpu().numpy(), ref[0]) <= 1e-5


def test_tiny_integer_batches_against_exact_arithmetic(ctx):
    """Small integer vectors, on which Algorithm 1 can be decided without rounding (comparisons of
    squares of rationals, see test_oracle_pins): the device's mask and count must be the exact
    ones, including the tie D = tau = 1 of orthogonal vectors, and the mean the exact fraction.
    Cases whose distance comes within 1e-6 of tau without being that tie are left out (the
    sequential schedule's running mean is binary32)."""
    from fractions import Fraction
    from test_oracle_pins import _exact_filter
    rng = np.random.default_rng(99)
    checked = ties = 0
    for trial in range(300):
        N, P = int(rng.integers(2, 7)), int(rng.integers(1, 9))
        rows = rng.integers(-4, 5, size=(N, P)).tolist()
        tau32 = np.float32(rng.choice([0.5, 0.9, 0.97, 1.0, 1.03, 1.3]))
        exact = _exact_filter(rows, Fraction(float(tau32)), list(range(N)))
        if exact is None:
            continue
        accepted, mean = exact
        grads = [torch.tensor(r, dtype=torch.float32).cuda() for r in rows]
        out, mask, dist, count = gaf.gaf_aggregate(ctx, grads, float(tau32))
        d = dist.cpu().numpy().astype(np.float64)
        near = np.abs(d[1:] - float(tau32)) < 1e-6
        tie = (d[1:] == 1.0) & (float(tau32) == 1.0)
        if np.any(near & ~tie):
            continue
        assert [i for i in range(N) if mask[i].item()] == accepted, (rows, float(tau32), d)
        assert int(count.item()) == len(accepted)
        np.testing.assert_allclose(out.cpu().numpy(), [float(m) for m in mean], rtol=2e-6, atol=1e-6)
        checked += 1
        ties += int(np.any(tie))
    assert checked > 200 and ties > 5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_streaming_long_vectors(ctx, oracle, dtype):
    """From 2^26 elements on a streaming visit is three launches (reduce, decide, update with one
    workgroup per tile) instead of two; same results, including the seeding first visit."""
    P, N = (1 << 26) + 4099, 6
    gen = torch.Generator(device="cuda").manual_seed(26)
    base = torch.randn(P, generator=gen, device="cuda")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    grads = [(sg * 0.4 * base + 0.9 * torch.randn(P, generator=gen, device="cuda")).to(tdt)
             for sg in (1, 1, -1, 1, -1, 1)]
    del base
    ref = _oracle_sequential_from_device(oracle, grads, 0.95)
    assert np.all(np.abs(ref[2][1:] - np.float32(0.95)) >= MARGIN)
    assert ref[1].tolist() == [1, 1, 0, 1, 0, 1]
    accum = torch.empty(P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(N, device="cuda"); mask = torch.empty(N, dtype=torch.uint8, device="cuda")
    for i, g in enumerate(grads):
        gaf.gaf_step(ctx, accum, count, g, 0.95, dist[i:i + 1], mask[i:i + 1])
    check_against_oracle((accum, mask, dist, count), ref, dtype)


# ------------------------------------------------------------- pairwise -------
@pytest.mark.parametrize("N,P,dtype", [(1, 1000, "f32"), (2, 31, "f32"), (5, 33, "f32"), (32, 4097, "f32"),
                                       (33, 70_001, "f32"), (64, 100_003, "bf16"), (70, 50_021, "f32"),
                                       (130, 20_011, "bf16"), (64, 700_001, "f32")])
def test_pairwise_shapes(ctx, oracle, N, P, dtype):
    g = torch.Generator().manual_seed(N * 7919 + P)
    centre = torch.randn(P, generator=g)
    grads = []
    for i in range(N):
        v = (0.1 * (i % 5) - 0.2) * centre + torch.randn(P, generator=g) * (1 + 0.1 * (i % 3))
        grads.append(v.to(torch.bfloat16) if dtype == "bf16" else v)
    dev = [x.cuda() for x in grads]
    gram = torch.empty((N, N), dtype=torch.float64, device="cuda")
    D = gaf.gaf_pairwise(ctx, dev, gram=gram)
    torch.cuda.synchronize()
    oD, oG = oracle.pairwise(oracle_arrays(grads))
    Dh = D.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(Dh - oD)) <= DIST_ATOL
    assert np.array_equal(Dh, Dh.T) and np.all(np.diag(Dh) == 0)
    scale = np.sqrt(np.outer(np.diag(oG), np.diag(oG)))
    assert np.max(np.abs(gram.cpu().numpy() - oG) / scale) <= 5e-7


# ------------------------------------------------------------ error paths -----
def test_argument_errors(ctx):
    lib = gaf.load()
    P = 4096
    x = torch.randn(P + 8, device="cuda"); out = torch.empty(P + 8, device="cuda")
    mask = torch.empty(80, dtype=torch.uint8, device="cuda"); dist = torch.empty(80, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")

    def agg(ptrs, N, P_, dt, outp):
        table = (ctypes.c_void_p * max(1, len(ptrs)))(*ptrs)
        return lib.gaf_aggregate(ctx.handle, table, N, P_, dt, 1.0, outp, mask.data_ptr(),
                                 dist.data_ptr(), count.data_ptr(), None)
    xp, op = x.data_ptr(), out.data_ptr()
    assert agg([xp, xp], 2, P, 0, op) == gaf.GAF_OK
    assert agg([xp + 4, xp], 2, P, 0, op) == gaf.GAF_EALIGN       # misaligned gradient
    assert agg([xp, xp], 2, P, 0, op + 4) == gaf.GAF_EALIGN       # misaligned out
    assert agg([xp, 0], 2, P, 0, op) == gaf.GAF_EINVAL            # NULL gradient
    assert agg([xp, xp], 0, P, 0, op) == gaf.GAF_EINVAL           # N < 1
    assert agg([xp, xp], 2, 0, 0, op) == gaf.GAF_EINVAL           # P == 0
    assert agg([xp, xp], 2, P, 7, op) == gaf.GAF_EUNSUPPORTED     # unknown dtype
    assert agg([xp, op], 2, P, 0, op) == gaf.GAF_EINVAL           # out aliases an input
    assert agg([xp] * 257, 257, P, 0, op) == gaf.GAF_EINVAL       # beyond the context's max_N
    assert lib.gaf_set_schedule(ctx.handle, 9) == gaf.GAF_EINVAL
    assert lib.gaf_set_schedule(ctx.handle, gaf.GAF_SCHEDULE_GRAM) == gaf.GAF_OK
    assert agg([xp] * 65, 65, P, 0, op) == gaf.GAF_EUNSUPPORTED   # Gram-first handles at most 64
    assert agg([xp], 1, P, 0, op) == gaf.GAF_EUNSUPPORTED
    assert lib.gaf_set_schedule(ctx.handle, gaf.GAF_SCHEDULE_AUTO) == gaf.GAF_OK
    assert agg([xp] * 65, 65, P, 0, op) == gaf.GAF_OK             # auto falls back to sequential
    gaf.gaf_set_schedule(ctx, ctx.schedule_name)
    assert lib.gaf_step(ctx.handle, op, count.data_ptr(), xp + 2, P, 1, 1.0, None, None, None) == gaf.GAF_EALIGN
    assert lib.gaf_step(ctx.handle, op, None, xp, P, 0, 1.0, None, None, None) == gaf.GAF_EINVAL
    assert lib.gaf_pairwise(ctx.handle, (ctypes.c_void_p * 1)(xp), 1, P, 0, None, None, None) == gaf.GAF_EINVAL
    assert lib.gaf_fused_mean_record(ctx.handle, None) == gaf.GAF_EINVAL
    assert lib.gaf_fused_mean_record(None, (ctypes.c_int32 * 4)()) == gaf.GAF_EINVAL
    torch.cuda.synchronize()
    with pytest.raises(gaf.GafError):
        gaf.gaf_aggregate(ctx, [x[1:P + 1], x[1:P + 1]], 1.0)


# ---------------------------------------------- full-size configurations ------
# Generated on the device (the host copy of each gradient is handed to the
# oracle one at a time, so the host never holds the whole batch).
def _oracle_sequential_from_device(oracle, grads, tau):
    P = grads[0].numel()
    g_sum = np.empty(P, dtype=np.float64)
    cnt, mask, dist = 0, [], []
    for g in grads:
        d, a, cnt = oracle.step(g_sum, cnt, wl.to_host_array(g), np.float32(tau))
        mask.append(a); dist.append(d)
    g_sum /= cnt
    return g_sum, np.array(mask, dtype=np.uint8), np.array(dist), cnt


@pytest.mark.timeout(600)
@pytest.mark.parametrize("N,dtype,pattern", [(10, "bf16", "mixed"), (10, "f32", "mixed"), (40, "bf16", "mixed"),
                                             (5, "f32", "mixed"), (5, "bf16", "mixed"),
                                             (10, "bf16", "few"), (10, "f32", "few"), (5, "bf16", "few")])
def test_fused_mean_with_right_and_wrong_guess(ctx, oracle, N, dtype, pattern):
    """Long vectors on the matrix-core path: the accept set is guessed from a sample of 2^22
    elements (256 evenly spaced runs of 2^14, as the header documents) and the Gram pass writes
    the mean of the guess. Here some gradients agree with the seed on the sampled elements and
    oppose it on the rest, so the guess is wrong and the stand-alone mean must take over; a
    second batch is twisted on a prefix instead and a third not at all (guess right). With the "few"
    pattern no gradient agrees with the seed: below a break-even accept count (two at these batch
    sizes) the Gram pass leaves the mean to the stand-alone kernel even when the guess is right."""
    P = (1 << 26) + 12_345
    gen = torch.Generator(device="cuda").manual_seed(100 + N)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    c = torch.randn(P, generator=gen, device="cuda")
    run, stride = 1 << 14, (P // 256) // (1 << 14) * (1 << 14)
    sampled = (torch.arange(256, device="cuda")[:, None] * stride + torch.arange(run, device="cuda")[None, :]).reshape(-1)
    flip = torch.ones(P, device="cuda"); flip[sampled] = -1.0
    flip_prefix = torch.ones(P, device="cuda"); flip_prefix[: 1 << 22] = -1.0
    signs = [1, 1, -1, 1, -1] * (N // 5) if pattern == "mixed" else [1] + [-1] * (N - 1)
    # twist "sample": on the sampled elements; "prefix": on the first 2^22 elements instead (one
    # atypical layer at the front: the spread-out sample must not be misled by it)
    for twist in ("sample", "prefix", None):
        grads = []
        for i in range(N):
            z = torch.randn(P, generator=gen, device="cuda")
            g = signs[i] * 0.4 * c + 0.9 * z
            if twist and i in (1, 2, N - 1):   # (for N = 5: gradients 1, 2 and 4)
                f = flip if twist == "sample" else flip_prefix
                g = g + (f - 1.0) * signs[i] * 0.4 * c      # opposite relation to c on those elements only
            grads.append(g.to(tdt))
            del z, g
        gaf.gaf_set_schedule(ctx, ctx.schedule_name)      # also forgets earlier guesses
        gaf.gaf_profile_begin(ctx)
        res = gaf.gaf_aggregate(ctx, grads, 0.95)
        launches = gaf.gaf_profile_end(ctx)
        torch.cuda.synchronize()
        ref = _oracle_sequential_from_device(oracle, grads, 0.95)
        assert np.all(np.abs(ref[2][1:] - np.float32(0.95)) >= MARGIN)
        check_against_oracle(res, ref, dtype)
        if ctx.schedule_name == "auto":
            # Did the device sample where the header says? With the twist on exactly those elements
            # the guess must be wrong and the stand-alone mean must do its work (>= 150 us at this
            # size); without it, and with enough accepted for the fused write, it returns at once
            # (a few us).
            mean_ms = [ms for name, ms in launches if name == "mean"]
            assert len(mean_ms) == 1 and any(name == "gram_sample" for name, _ in launches)
            rec = gaf.gaf_fused_mean_record(ctx)
            if twist == "sample" or pattern == "few":
                assert mean_ms[0] > 0.05, launches
                assert rec["valid"] == 0
            else:
                assert mean_ms[0] < 0.05, launches
                assert rec == {"write": 1, "valid": 1, "backoff": 0, "penalty": 1}
            if twist == "sample" and pattern == "mixed":
                assert rec == {"write": 1, "valid": 0, "backoff": 1, "penalty": 2}
            # whether the guess was right or wrong, the result equals the two-pass schedule's bit for bit
            gaf.gaf_set_schedule(ctx, "gram")
            two_pass = gaf.gaf_aggregate(ctx, grads, 0.95)
            gaf.gaf_set_schedule(ctx, "auto")
            torch.cuda.synchronize()
            for x, y in zip(res, two_pass):
                assert torch.equal(x, y)
            del two_pass
        if twist == "sample":
            # the sample alone would have decided differently for the twisted gradients
            pre = oracle.aggregate([wl.to_host_array(g[sampled]) for g in grads], np.float32(0.95))
            assert pre[1].tolist() != ref[1].tolist()
        del grads, res


def test_fused_mean_backs_off_after_wrong_guesses(ctx):
    """The context's record of guesses: a written guess that proves wrong stops the writing for
    `penalty` calls and doubles the penalty, a right one halves it. Batch A is built so that the
    sample misleads (see the test above), batch B so that it does not; every call's result must
    equal the two-pass schedule's bit for bit whatever the record says."""
    if ctx.schedule_name != "auto":
        pytest.skip("the fused mean belongs to the AUTO schedule")
    P, N = (1 << 26) + 64, 10
    gen = torch.Generator(device="cuda").manual_seed(7)
    c = torch.randn(P, generator=gen, device="cuda")
    stride = (P // 256) // (1 << 14) * (1 << 14)
    sampled = (torch.arange(256, device="cuda")[:, None] * stride + torch.arange(1 << 14, device="cuda")[None, :]).reshape(-1)
    flip = torch.ones(P, device="cuda"); flip[sampled] = -1.0
    signs = [1, 1, -1, 1, -1] * 2
    batches = {}
    for name in "AB":
        grads = []
        for i in range(N):
            g = signs[i] * 0.4 * c + 0.9 * torch.randn(P, generator=gen, device="cuda")
            if name == "A" and i in (1, 2, N - 1):
                g = g + (flip - 1.0) * signs[i] * 0.4 * c
            grads.append(g.to(torch.bfloat16)); del g
        gaf.gaf_set_schedule(ctx, "gram")
        expect = [t.clone() for t in gaf.gaf_aggregate(ctx, grads, 0.95)]
        batches[name] = (grads, expect)
    gaf.gaf_set_schedule(ctx, "auto")
    assert gaf.gaf_fused_mean_record(ctx) == {"write": 0, "valid": 0, "backoff": 0, "penalty": 1}
    script = [("A", 1, 0, 1, 2), ("B", 0, 0, 0, 2), ("B", 1, 1, 0, 1), ("A", 1, 0, 1, 2), ("A", 0, 0, 0, 2),
              ("A", 1, 0, 2, 4), ("B", 0, 0, 1, 4), ("B", 0, 0, 0, 4), ("B", 1, 1, 0, 2), ("B", 1, 1, 0, 1)]
    for step, (name, write, valid, backoff, penalty) in enumerate(script):
        grads, expect = batches[name]
        res = gaf.gaf_aggregate(ctx, grads, 0.95)
        rec = gaf.gaf_fused_mean_record(ctx)
        assert rec == {"write": write, "valid": valid, "backoff": backoff, "penalty": penalty}, (step, rec)
        for x, y in zip(res, expect):
            assert torch.equal(x, y), step


@pytest.mark.parametrize("N,P,dtype", [(2, (1 << 21) + 7, "f32"), (2, 11_220_132, "bf16"), (5, (1 << 21) + 4097, "f32"),
                                       (12, (1 << 21) + 3, "f32"), (20, 1 << 21, "bf16"), (40, (1 << 21) + 33, "f32")])
def test_carried_guess_on_shorter_vectors(ctx, oracle, N, P, dtype):
    """Below the length where a sample pays, batches of TWO gradients guess the previous call's
    accept set; larger batches do not guess at these lengths. Three batches: X and a second draw X2
    with the same agreement pattern (guess right), Y with another pattern (guess wrong). Every
    result is checked against the oracle, must equal the two-pass schedule's bit for bit, and the
    record must follow the hits and misses (N = 2) or show that nothing was written (N > 2)."""
    if ctx.schedule_name != "auto":
        pytest.skip("the fused mean belongs to the AUTO schedule")
    gen = torch.Generator().manual_seed(1000 + N)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    base = torch.randn(P, generator=gen)
    def batch(signs):
        return [(sg * 0.5 * base + 0.8 * torch.randn(P, generator=gen)).to(tdt) for sg in signs]
    sx = [1 if i % 3 != 2 else -1 for i in range(N)]; sx[0] = 1
    sy = [1 if i % 2 == 0 else -1 for i in range(N)]
    batches = {"X": batch(sx), "X2": batch(sx), "Y": batch(sy)}
    ref, expect, dev = {}, {}, {}
    for k, g in batches.items():
        ref[k] = oracle.aggregate(oracle_arrays(g), np.float32(0.9))
        assert np.all(np.abs(ref[k][2][1:] - np.float32(0.9)) >= MARGIN)
        dev[k] = [t.cuda() for t in g]
        gaf.gaf_set_schedule(ctx, "gram")
        expect[k] = [t.clone() for t in gaf.gaf_aggregate(ctx, dev[k], 0.9)]
    assert ref["X"][1].tolist() == ref["X2"][1].tolist() != ref["Y"][1].tolist()
    gaf.gaf_set_schedule(ctx, "auto")
    if N != 2:
        for step, k in enumerate(("X", "X2", "X", "Y", "Y", "X")):
            res = gaf.gaf_aggregate(ctx, dev[k], 0.9)
            assert gaf.gaf_fused_mean_record(ctx)["write"] == 0, (step, k)
            check_against_oracle(res, ref[k], dtype)
            for x, y in zip(res, expect[k]):
                assert torch.equal(x, y), (step, k)
        return
    # (batch, was a mean written by the Gram pass, was it right, backoff after, penalty after)
    script = [("X", 0, 0, 0, 1),       # nothing to carry yet
              ("X2", 1, 1, 0, 1), ("X", 1, 1, 0, 1),
              ("Y", 1, 0, 1, 2),       # guess X's set, wrong
              ("Y", 0, 0, 0, 2),       # backing off (the guess itself would have been right)
              ("Y", 1, 1, 0, 1), ("X", 1, 0, 1, 2), ("X2", 0, 0, 0, 2), ("X", 1, 1, 0, 1)]
    for step, (k, write, valid, backoff, penalty) in enumerate(script):
        res = gaf.gaf_aggregate(ctx, dev[k], 0.9)
        rec = gaf.gaf_fused_mean_record(ctx)
        assert rec == {"write": write, "valid": valid, "backoff": backoff, "penalty": penalty}, (step, k, rec)
        check_against_oracle(res, ref[k], dtype)
        for x, y in zip(res, expect[k]):
            assert torch.equal(x, y), (step, k)
    # another batch size does not use the guess (three gradients do not guess at this length at all)
    res = [t.clone() for t in gaf.gaf_aggregate(ctx, dev["X"] + dev["Y"][1:], 0.9)]
    gaf.gaf_set_schedule(ctx, "gram")
    for x, y in zip(res, gaf.gaf_aggregate(ctx, dev["X"] + dev["Y"][1:], 0.9)):
        assert torch.equal(x, y)
    gaf.gaf_set_schedule(ctx, "auto")


@pytest.mark.parametrize("N", [3, 9, 33])
def test_near_cancellation_at_tau_two(ctx, oracle, N):
    """g_2 = -g_1 up to noise of 1e-3: the running sum after g_2 nearly cancels. With tau = 2
    everything is accepted and the result is the plain mean (Eq. 2) on every schedule -- the
    running sum's squared norm, carried through the Gram matrix as a difference of large terms,
    must not turn into a negative or random number there."""
    P = 300_000
    gen = torch.Generator().manual_seed(77 + N)
    g1 = torch.randn(P, generator=gen)
    grads = [g1, -g1 + 1e-3 * torch.randn(P, generator=gen)]
    grads += [torch.randn(P, generator=gen) for _ in range(N - 2)]
    res = gaf.gaf_aggregate(ctx, [g.cuda() for g in grads], 2.0)
    ref = oracle.aggregate(oracle_arrays(grads), np.float32(2.0))
    torch.cuda.synchronize()
    assert ref[1].tolist() == [1] * N
    assert res[1].cpu().numpy().tolist() == [1] * N and int(res[3].item()) == N
    mean = oracle.plain_average(oracle_arrays(grads))
    assert rel_l2(res[0].cpu().numpy(), mean) <= 1e-5
    d = np.abs(res[2].cpu().numpy().astype(np.float64) - ref[2])
    # The distance of g_3 is taken against a running sum of relative size 1e-3: binary64 sums
    # (sequential passes, small batches) resolve it; the matrix-core sums do not (their entries
    # carry binary32 rounding of the same size) and report the distance to a zero vector, 1.
    if ctx.schedule_name == "sequential" or N <= 8:
        assert d.max() <= 1e-4, d
    else:
        assert d[2] <= 1e-2 and np.delete(d, 2).max() <= 1e-4, d      # |cos| of unrelated vectors: a few / sqrt(P)


@pytest.mark.parametrize("N,P", [(9, 3000), (33, 2500), (64, 4100), (17, 40_000)])
def test_highly_correlated_rows_on_short_vectors(ctx, oracle, N, P):
    """|cos| near 0.99 between all rows and few columns per workgroup: the matrix-core tiles sum
    in binary32 for up to eight stages before they are added into binary64 totals, and with so few
    columns nothing averages that rounding out -- the distances must still be within 1e-6."""
    gen = torch.Generator().manual_seed(5 * N + P)
    base = torch.randn(P, generator=gen)
    grads = [base + 0.14 * torch.randn(P, generator=gen) for _ in range(N)]
    a = oracle_arrays(grads)
    oD, _ = oracle.pairwise(a)
    assert 0.005 < oD[0, 1] < 0.03
    D = gaf.gaf_pairwise(ctx, [g.cuda() for g in grads])
    torch.cuda.synchronize()
    assert np.max(np.abs(D.cpu().numpy().astype(np.float64) - oD)) <= DIST_ATOL
    for tau in (0.015, 0.5):
        ref = oracle.aggregate(a, np.float32(tau))
        if np.all(np.abs(ref[2][1:] - np.float32(tau)) >= MARGIN):
            check_against_oracle(gaf.gaf_aggregate(ctx, [g.cuda() for g in grads], tau), ref, "f32")


@pytest.mark.timeout(600)
def test_large_full_size(ctx, oracle):
    for seed in range(4):
        w, grads = wl.generate("large", seed, device="cuda")
        assert w.P == 1_000_000_000 and w.N == 16 and grads[0].dtype == torch.bfloat16
        res = gaf.gaf_aggregate(ctx, grads, w.tau)
        torch.cuda.synchronize()
        ref = _oracle_sequential_from_device(oracle, grads, w.tau)
        if np.all(np.abs(ref[2][1:] - np.float32(w.tau)) >= MARGIN):
            break
        del grads, res
    check_against_oracle(res, ref, "bf16")
    # the streaming entry point at the same size, on a prefix of the sequence
    accum = torch.empty(w.P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(6, device="cuda"); mask = torch.empty(6, dtype=torch.uint8, device="cuda")
    for i in range(6):
        gaf.gaf_step(ctx, accum, count, grads[i], w.tau, dist[i:i + 1], mask[i:i + 1])
    torch.cuda.synchronize()
    assert mask.cpu().numpy().tolist() == ref[1][:6].tolist()
    assert np.max(np.abs(dist.cpu().numpy().astype(np.float64) - ref[2][:6])) <= DIST_ATOL


_FULL_MATRIX = {}


@pytest.mark.timeout(900)
def test_diagnostic_full_size(ctx, oracle):
    for seed in range(4):
        w, grads = wl.generate("diagnostic", seed, device="cuda")
        assert w.P == 124_439_808 and w.N == 64
        res = gaf.gaf_aggregate(ctx, grads, w.tau)
        torch.cuda.synchronize()
        ref = _oracle_sequential_from_device(oracle, grads, w.tau)
        if np.all(np.abs(ref[2][1:] - np.float32(w.tau)) >= MARGIN):
            break
        del grads, res
    check_against_oracle(res, ref, "f32")
    assert ref[1].tolist() == [1 if k == 0 else 0 for k in w.cluster]
    D = gaf.gaf_pairwise(ctx, grads)
    res_m = gaf.gaf_aggregate_with_matrix(ctx, grads, w.tau)       # long vectors: fused mean + matrix
    check_against_oracle(res_m[:4], ref, "f32")
    assert torch.equal(res_m[4], D)
    Dh = D.cpu().numpy().astype(np.float64)
    assert np.array_equal(Dh, Dh.T) and np.all(np.diag(Dh) == 0)
    assert Dh.min() >= 0 and Dh.max() <= 2
    # every one of the 2016 pairs against the oracle's matrix (all 64 gradients on the host: 32 GB;
    # the oracle's pass over them is the slow part and is done once for both schedules)
    key = (seed, w.P, w.N)
    if key not in _FULL_MATRIX:
        _FULL_MATRIX.clear()
        _FULL_MATRIX[key] = oracle.pairwise([wl.to_host_array(g) for g in grads])[0]
    assert np.max(np.abs(Dh - _FULL_MATRIX[key])) <= DIST_ATOL
    # row 0 against the sequential distances up to the first acceptance
    first = int(np.argmax(ref[1][1:])) + 1
    assert np.max(np.abs(Dh[0, 1:first + 1] - ref[2][1:first + 1])) <= DIST_ATOL
