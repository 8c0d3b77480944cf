"""The write windows of the Gram pass that also writes the mean are a matter of timing only: with
the windows switched off, with a short fixed period (many windows per launch) and with the
library's own choice, the same call returns the same bits. GAF_WRITE_WINDOWS is read once per
process, so each setting runs in a process of its own."""
import hashlib
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import hashlib, sys
sys.path.insert(0, %r)
import torch
from paper_2412_18052_amd import gaf
torch.cuda.set_device(0)
out_all = []
for N, tdt, P in ((16, torch.bfloat16, (1 << 26) + 333), (64, torch.float32, (1 << 26) + 8), (33, torch.float32, (1 << 26))):
    gen = torch.Generator(device="cuda").manual_seed(7 + N)
    c = torch.randn(P, generator=gen, device="cuda")
    grads = [((0.5 if i %% 3 else -0.5) * c + 0.9 * torch.randn(P, generator=gen, device="cuda")).to(tdt) for i in range(N)]
    ctx = gaf.gaf_create(P, N)
    res = gaf.gaf_aggregate(ctx, grads, 0.95)
    torch.cuda.synchronize()
    rec = gaf.gaf_fused_mean_record(ctx)
    assert rec["write"] == 1 and rec["valid"] == 1, rec     # the Gram pass wrote the result
    h = hashlib.sha256()
    for t in res:
        h.update(t.cpu().numpy().tobytes())
    out_all.append(h.hexdigest())
    gaf.gaf_destroy(ctx)
    del grads, c, res
    torch.cuda.empty_cache()
print("HASHES " + " ".join(out_all))
""" % ROOT


def _run(setting):
    env = dict(os.environ)
    env.pop("GAF_WRITE_WINDOWS", None)
    if setting is not None:
        env["GAF_WRITE_WINDOWS"] = setting
    p = subprocess.run([sys.executable, "-c", CHILD], env=env, capture_output=True, text=True, timeout=240)
    assert p.returncode == 0, p.stderr[-2000:]
    line = [l for l in p.stdout.splitlines() if l.startswith("HASHES ")]
    assert len(line) == 1, p.stdout[-2000:]
    return line[0].split()[1:]


@pytest.mark.gpu
@pytest.mark.timeout(900)
def test_results_do_not_depend_on_the_write_windows():
    default = _run(None)
    assert len(default) == 3
    assert _run("0") == default            # no windows: written whenever the ring is full
    assert _run("700:120") == default      # several hundred windows per launch
    assert _run("nonsense") == default     # an unreadable setting leaves the formula in charge
