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
from test_gpu_parity import DIST_ATOL, OUT_RTOL, _oracle_sequential_from_device, check_against_oracle, rel_l2

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



def long_cases():
    rng = np.random.default_rng(20250101)
    out = []
    for k, N in enumerate([2, 3, 5, 8, 9, 16, 17, 33, 48, 64, 2, 16]):
        P = (1 << 26) + int(rng.integers(0, 100_000))
        out.append((k, N, P, "bf16" if rng.random() < 0.5 else "f32"))
    return out


@pytest.fixture(scope="module")
def long_ctxs():
    c = {"auto": gaf.gaf_create(max_P=(1 << 26) + 100_000, max_N=64),     # never touched: keeps its record
         "other": gaf.gaf_create(max_P=(1 << 26) + 100_000, max_N=64)}
    yield c
    torch.cuda.synchronize()
    for v in c.values():
        gaf.gaf_destroy(v)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("k,N,P,dtype", long_cases())
def test_random_long_vectors_guessing_changes_nothing(long_ctxs, oracle, k, N, P, dtype):
    """Vectors long enough for the accept set to be guessed from a sample. One AUTO context lives
    through all cases, so its record of guesses,
    backoff included, is in whatever state the earlier cases left. The first gradients behind the
    seed are built to sit within the sample's error of tau, so that guesses do go wrong. Whatever
    was guessed, the AUTO result must equal the two-pass schedule's bit for bit, and the
    sequential schedule must agree where its distances keep a margin from tau."""
    gen = torch.Generator(device="cuda").manual_seed(5000 + k)
    hrng = np.random.default_rng(9000 + k)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    tau = 0.95
    base = torch.randn(P, generator=gen, device="cuda")
    grads = []
    for i in range(N):
        if i == 0:
            a = 0.4
        elif i <= 2:
            a = 0.111 * (1.0 + hrng.normal() * 2e-3)      # cosine to the seed close to 1 - tau
        else:
            a = 0.4 if hrng.random() < 0.6 else -0.4
        grads.append((a * base + 0.9 * torch.randn(P, generator=gen, device="cuda")).to(tdt))
    del base
    auto, other = long_ctxs["auto"], long_ctxs["other"]
    gaf.gaf_set_schedule(other, "gram")
    ref = [t.clone() for t in gaf.gaf_aggregate(other, grads, tau)]
    gaf.gaf_set_schedule(other, "sequential")
    seq = [t.clone() for t in gaf.gaf_aggregate(other, grads, tau)]
    records = []
    for rep in range(3):
        res = gaf.gaf_aggregate(auto, grads, tau)
        records.append(gaf.gaf_fused_mean_record(auto))
        for x, y in zip(res, ref):
            assert torch.equal(x, y), (k, rep, records)
    # the oracle, fed one gradient at a time: its mask up to the first distance that comes within
    # 1e-3 of tau (from there on a rounding difference may legitimately decide otherwise), its
    # distances up to that point, and everything if no distance comes that close
    o_out, o_mask, o_dist, o_count = _oracle_sequential_from_device(oracle, grads, tau)
    o_clear = np.abs(o_dist[1:] - np.float32(tau)) >= 1e-3
    upto = N if o_clear.all() else 1 + int(np.argmin(o_clear))
    assert ref[1].cpu().numpy()[:upto].tolist() == o_mask[:upto].tolist()
    assert np.max(np.abs(ref[2].cpu().numpy().astype(np.float64)[:upto] - o_dist[:upto])) <= DIST_ATOL
    if upto == N:
        check_against_oracle(ref, (o_out, o_mask, o_dist, o_count), dtype)
    del o_out
    d = ref[2].cpu().numpy().astype(np.float64)
    clear = np.abs(d - np.float32(tau)) >= 5e-4
    m_ref, m_seq = ref[1].cpu().numpy(), seq[1].cpu().numpy()
    first_unclear = int(np.argmin(clear)) if not clear.all() else N
    # up to the first borderline gradient both schedules have seen the same history
    assert np.array_equal(m_ref[:first_unclear], m_seq[:first_unclear]), (d, m_ref, m_seq)
    if clear.all():
        assert int(ref[3].item()) == int(seq[3].item())
        assert np.max(np.abs(d - seq[2].cpu().numpy())) <= 1e-5
        assert rel_l2(seq[0].cpu().numpy(), ref[0].cpu().numpy()) <= OUT_RTOL[dtype]
