"""Streaming with one step of look-ahead (gaf_step_lookahead / gaf_flush) against gaf_step and
the oracle: the update of an accepted gradient is applied by the NEXT visit's walk, or by the
flush, and everything -- decisions, distances, count, aggregate -- must come out as with
gaf_step, bit for bit."""
import ctypes

import numpy as np
import pytest
import torch

from conftest import workload_with_margin
from paper_2412_18052_amd import gaf
from paper_2412_18052_amd import workloads as wl
from test_gpu_parity import DIST_ATOL, OUT_RTOL, check_against_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = gaf.gaf_create(max_P=1 << 28, max_N=64)
    yield c
    torch.cuda.synchronize()
    gaf.gaf_destroy(c)


def _plain(ctx, dev, tau):
    P, N = dev[0].numel(), len(dev)
    accum = torch.empty(P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(N, device="cuda"); mask = torch.empty(N, dtype=torch.uint8, device="cuda")
    for i, g in enumerate(dev):
        gaf.gaf_step(ctx, accum, count, g, tau, dist[i:i + 1], mask[i:i + 1])
    torch.cuda.synchronize()
    return accum, mask, dist, count


def _lookahead(ctx, dev, tau, flush=True):
    P, N = dev[0].numel(), len(dev)
    accum = torch.empty(P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(N, device="cuda"); mask = torch.empty(N, dtype=torch.uint8, device="cuda")
    for i, g in enumerate(dev):
        gaf.gaf_step_lookahead(ctx, accum, count, g, tau, dist[i:i + 1], mask[i:i + 1])
    if flush:
        gaf.gaf_flush(ctx)
    torch.cuda.synchronize()
    return accum, mask, dist, count


@pytest.mark.parametrize("name,N,P,dtype", [("streaming", 12, 400_009, "f32"), ("streaming", 9, 1_000_003, "bf16"),
                                            ("tiny", 4, 4097, "f32"), ("resnet18", 8, 2_500_000, "f32"),
                                            ("large", 6, (1 << 26) + 77, "bf16"),      # three-launch length of gaf_step
                                            ("tiny", 1, 1000, "f32"), ("streaming", 5, 3, "f32")])
def test_lookahead_equals_step_and_oracle(ctx, oracle, name, N, P, dtype):
    if P > (1 << 24):
        w, grads = wl.generate(name, 1, P=P, N=N, device="cuda")
        dev, ref = grads, None
    else:
        w, grads, ref = workload_with_margin(name, P=P, N=N)
        if dtype == "bf16" and grads[0].dtype != torch.bfloat16:
            grads = [g.to(torch.bfloat16) for g in grads]
            from conftest import oracle_arrays
            ref = oracle.aggregate(oracle_arrays(grads), np.float32(w.tau))
            if not np.all(np.abs(ref[2][1:] - np.float32(w.tau)) >= 1e-3):
                pytest.skip("rounding to bfloat16 moved a distance next to tau")
        dev = [g.cuda() for g in grads]
    plain = _plain(ctx, dev, w.tau)
    ahead = _lookahead(ctx, dev, w.tau)
    for x, y in zip(ahead, plain):
        assert torch.equal(x, y)
    if ref is not None:
        check_against_oracle(ahead, ref, dtype)


def test_state_between_calls_and_flush_after_reject(ctx, oracle):
    """After visit i and before the next call: the counter already includes g_i, the aggregate does
    not yet. A rejected last gradient leaves nothing to flush: the aggregate stays bit for bit."""
    w, grads, ref = workload_with_margin("streaming", P=300_011, N=10)
    dev = [g.cuda() for g in grads]
    P = w.P
    # aggregates of gaf_step after every visit
    accum = torch.empty(P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    after = []
    for g in dev:
        gaf.gaf_step(ctx, accum, count, g, w.tau)
        after.append((accum.clone(), int(count.item())))
    acc2 = torch.full((P,), 123.0, device="cuda"); cnt2 = torch.zeros(1, dtype=torch.int32, device="cuda")
    for i, g in enumerate(dev):
        gaf.gaf_step_lookahead(ctx, acc2, cnt2, g, w.tau)
        torch.cuda.synchronize()
        assert int(cnt2.item()) == after[i][1]
        if i >= 1:
            assert torch.equal(acc2, after[i - 1][0]), i       # g_i not applied yet
    last_rejected = ref[1][-1] == 0
    before = acc2.clone()
    gaf.gaf_flush(ctx)
    gaf.gaf_flush(ctx)                                         # nothing pending any more: no-op
    torch.cuda.synchronize()
    assert torch.equal(acc2, after[-1][0])
    if last_rejected:
        assert torch.equal(acc2, before)
    # a sequence that ends on a rejected gradient for sure: append the negated seed
    dev.append((-grads[0]).cuda())
    res = _lookahead(ctx, dev, w.tau, flush=False)
    held = res[0].clone()
    gaf.gaf_flush(ctx)
    torch.cuda.synchronize()
    assert int(res[1][-1].item()) == 0 and torch.equal(res[0], held)


def test_resumed_and_mixed_with_other_calls(ctx, oracle):
    """The state is (accum, count) once flushed: a run interrupted by a flush, by a plain gaf_step
    (which applies the pending update itself) or by a batch call on the same context ends where an
    uninterrupted run ends."""
    w, grads, ref = workload_with_margin("streaming", P=250_007, N=12)
    dev = [g.cuda() for g in grads]
    want = _plain(ctx, dev, w.tau)
    accum = torch.empty(w.P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(w.N, device="cuda"); mask = torch.empty(w.N, dtype=torch.uint8, device="cuda")
    def ahead(i):
        gaf.gaf_step_lookahead(ctx, accum, count, dev[i], w.tau, dist[i:i + 1], mask[i:i + 1])
    for i in range(0, 4):
        ahead(i)
    gaf.gaf_flush(ctx)                                                      # explicit flush, then on
    for i in range(4, 6):
        ahead(i)
    gaf.gaf_step(ctx, accum, count, dev[6], w.tau, dist[6:7], mask[6:7])    # plain visit flushes first
    for i in range(7, 9):
        ahead(i)
    other = gaf.gaf_aggregate(ctx, dev[:5], w.tau)                          # batch call flushes first
    for i in range(9, 12):
        ahead(i)
    gaf.gaf_flush(ctx)
    torch.cuda.synchronize()
    for x, y in zip((accum, mask, dist, count), want):
        assert torch.equal(x, y)
    check_against_oracle(other, oracle.aggregate([wl.to_host_array(g) for g in grads[:5]], np.float32(w.tau)), "f32")


def test_lookahead_argument_errors(ctx):
    lib = gaf.load()
    P = 4096
    a = torch.zeros(P, device="cuda"); b = torch.zeros(P, device="cuda")
    c = torch.zeros(1, dtype=torch.int32, device="cuda"); c2 = torch.zeros(1, dtype=torch.int32, device="cuda")
    g = [torch.randn(P, device="cuda") for _ in range(3)]
    gb = torch.randn(P, device="cuda").to(torch.bfloat16)
    def call(accum, count, grad, n=P, dt=gaf.GAF_F32):
        return lib.gaf_step_lookahead(ctx.handle, ctypes.c_void_p(accum.data_ptr()), ctypes.c_void_p(count.data_ptr()),
                                      ctypes.c_void_p(grad.data_ptr()), n, dt, ctypes.c_float(1.0), None, None, None)
    assert call(a, c, g[0]) == gaf.GAF_OK
    assert call(b, c, g[1]) == gaf.GAF_EINVAL            # another aggregate while one is pending
    assert call(a, c2, g[1]) == gaf.GAF_EINVAL           # another counter
    assert call(a, c, g[1], n=P - 8) == gaf.GAF_EINVAL   # another length
    assert call(a, c, gb, dt=gaf.GAF_BF16) == gaf.GAF_EINVAL
    assert call(a, c, g[0]) == gaf.GAF_EINVAL            # the pending gradient itself
    assert call(a, c, g[1]) == gaf.GAF_OK                # the rejected calls left the pending one in place
    assert lib.gaf_flush(ctx.handle, None) == gaf.GAF_OK
    assert call(b, c2, g[2]) == gaf.GAF_OK               # after the flush anything goes
    assert lib.gaf_flush(ctx.handle, None) == gaf.GAF_OK
    assert lib.gaf_flush(None, None) == gaf.GAF_EINVAL
    torch.cuda.synchronize()
    assert int(c.item()) == 2 or int(c.item()) == 1


def test_lookahead_in_a_graph(ctx, oracle):
    """Captured like the other calls: replays, with eager work between them, equal the eager run."""
    w, grads, ref = workload_with_margin("streaming", P=500_001, N=8)
    dev = [g.cuda() for g in grads]
    accum = torch.empty(w.P, device="cuda"); count = torch.zeros(1, dtype=torch.int32, device="cuda")
    dist = torch.empty(w.N, device="cuda"); mask = torch.empty(w.N, dtype=torch.uint8, device="cuda")

    def work():
        count.fill_(0)
        for i, g in enumerate(dev):
            gaf.gaf_step_lookahead(ctx, accum, count, g, w.tau, dist[i:i + 1], mask[i:i + 1])
        gaf.gaf_flush(ctx)

    work()
    torch.cuda.synchronize()
    check_against_oracle((accum, mask, dist, count), ref, "f32")
    eager = [t.clone() for t in (accum, mask, dist, count)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work()
    for rep in range(3):
        accum.fill_(float(rep)); dist.fill_(-1.0); mask.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((accum, mask, dist, count), eager):
            assert torch.equal(got, want), rep
