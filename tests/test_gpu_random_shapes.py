"""Randomised (seeded) sweep over shapes: every batch entry point against the oracle on
sizes drawn across the kernel variants' boundaries (N around 8/16/32/48/64, P around tile,
stage and unroll multiples), both dtypes, both schedules. A second sweep uses vectors just long
enough for the batch call to carry its guess of the accept set from call to call: the contexts
are shared by all cases, so right guesses (the same batch twice in a row) and wrong ones
(another case with the same N before it) both occur."""
import numpy as np
import pytest
import torch

from conftest import MARGIN, oracle_arrays
from paper_2412_18052_amd import gaf
from paper_2412_18052_amd import workloads as wl
from test_gpu_parity import DIST_ATOL, OUT_RTOL, check_against_oracle, rel_l2

pytestmark = pytest.mark.gpu


def cases():
    rng = np.random.default_rng(20241218)
    out = []
    n_choices = [1, 2, 3, 4, 7, 8, 9, 15, 16, 17, 24, 32, 33, 47, 48, 49, 63, 64]
    p_bases = [1, 5, 32, 127, 128, 255, 256, 1024, 2048, 4096, 8192, 16384, 65536, 262144]
    for k in range(48):
        N = int(rng.choice(n_choices))
        P = int(rng.choice(p_bases)) * int(rng.integers(1, 6)) + int(rng.integers(-3, 4))
        P = max(1, min(P, 600_000))
        dtype = "bf16" if rng.random() < 0.5 else "f32"
        out.append((k, N, P, dtype))
    for k in range(48, 64):
        N = int(rng.choice([2, 2, 3, 5, 8, 9, 16, 17, 33, 48]))
        P = (1 << 21) + int(rng.integers(0, 300_000))
        out.append((k, N, P, "bf16" if rng.random() < 0.5 else "f32"))
    return out


@pytest.fixture(scope="module")
def ctxs():
    c = {}
    for name in ("sequential", "auto"):
        c[name] = gaf.gaf_create(max_P=1 << 24, max_N=64)
        gaf.gaf_set_schedule(c[name], name)
    yield c
    torch.cuda.synchronize()
    for v in c.values():
        gaf.gaf_destroy(v)


@pytest.mark.parametrize("k,N,P,dtype", cases())
def test_random_shape(ctxs, oracle, k, N, P, dtype):
    name = ["resnet18", "large", "streaming", "diagnostic"][k % 4]
    for seed in range(k * 100, k * 100 + 12):
        w, grads = wl.generate(name, seed, P=P, N=N)
        if dtype == "bf16":
            grads = [g.to(torch.bfloat16) for g in grads]
        else:
            grads = [g.to(torch.float32) for g in grads]
        a = oracle_arrays(grads)
        tau = np.float32(w.tau)
        ref = oracle.aggregate(a, tau)
        if np.all(np.abs(ref[2][1:] - float(tau)) >= MARGIN):
            break
    else:
        pytest.skip("no seed keeps the margin (tiny P: distances are coarse)")
    dev = [g.cuda() for g in grads]
    oD, oG = oracle.pairwise(a)
    for sched, ctx in ctxs.items():
        res = gaf.gaf_aggregate(ctx, dev, float(tau))
        check_against_oracle(res, ref, dtype)
        out, mask, dist, count, D = gaf.gaf_aggregate_with_matrix(ctx, dev, float(tau))
        check_against_oracle((out, mask, dist, count), ref, dtype)
        assert np.max(np.abs(D.cpu().numpy().astype(np.float64) - oD)) <= DIST_ATOL
        accum = torch.empty(P, device="cuda"); cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
        sd = torch.empty(N, device="cuda"); sm = torch.empty(N, dtype=torch.uint8, device="cuda")
        for i, g in enumerate(dev):
            gaf.gaf_step(ctx, accum, cnt, g, float(tau), sd[i:i + 1], sm[i:i + 1])
        check_against_oracle((accum, sm, sd, cnt), ref, dtype)
