"""Seeded synthetic micro-gradient workloads.

Input generation only: nothing in this module computes a distance, a mask or
an average. Both the HIP library's callers and the CPU oracle's callers draw
their inputs from here, so that the two sides see the same bits.

The paper's micro-gradients come from ResNet18 (about 11 M parameters) and
ViT-L/16 (about 300 M) training runs (Sec. 1) and are reported to be close to
orthogonal, with cosine distances clustered around 1, excursions to 1.1-1.6,
and above 0.96 on pure noise (Fig. 1, Fig. 5). Those runs need datasets that
are not available, so the vectors here are synthetic stand-ins with the same
shapes and the same distance structure:

    g_i = a_i * ( s_i * sqrt(rho_i) * c  +  sqrt(1 - rho_i) * z_i )

with a shared direction ``c``, private noise ``z_i``, sign ``s_i``, correlation
``rho_i`` and scale ``a_i``. The five named workloads fix N, P, dtype, tau and
the distributions of (rho, s, a, z):

  tiny        N=4   P=1,000,000     f32   tau=0.97  rho=0.3, s=[+,+,-,+], a=1
  resnet18    N=8   P=11,220,132    f32   tau=0.97  rho~U[0,0.2], P(s=-1)=.25,
                                                    a~lognormal(0,0.5)
  streaming   N=32  P=11,220,132    f32   tau=1.0   rho=0.01, s_0=+1, others +-1
                                                    with p=0.5, a=1
  large       N=16  P=1,000,000,000 bf16  tau=0.98  rho=0.1, P(s=-1)=.3,
                                                    z ~ Student-t(3)/sqrt(3)
  diagnostic  N=64  P=124,439,808   f32   tau=0.95  4 latent clusters,
                                                    g_i = 0.6 c_{i mod 4} + 0.8 z_i,
                                                    c_2 = (-c_0 + 0.5 n)/sqrt(1.25)

``P`` can be overridden to get a scaled-down instance of the same recipe.
Host-side parameters (rho, s, a) come from numpy's Philox generator keyed by
the seed; the P-length normal draws come from a ``torch.Generator`` on the
requested device keyed by the same seed. CPU and GPU generators give different
streams: generate ONCE and hand the same tensors to every consumer.
bf16 workloads are rounded to bfloat16 (round-to-nearest-even) once, here.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

_CHUNK = 1 << 25  # elements drawn at a time, bounds temporary memory


@dataclass
class Workload:
    name: str
    N: int
    P: int
    dtype: str            # "f32" | "bf16"
    tau: float
    mode: str             # "aggregate" | "step" | "pairwise"
    seed: int = 0
    rho: List[float] = field(default_factory=list)
    sign: List[float] = field(default_factory=list)
    scale: List[float] = field(default_factory=list)
    cluster: Optional[List[int]] = None
    noise: str = "normal"  # "normal" | "student_t3"

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def elem_bytes(self):
        return 4 if self.dtype == "f32" else 2


NAMES = ("tiny", "resnet18", "streaming", "large", "diagnostic")

_FULL_P = {"tiny": 1_000_000, "resnet18": 11_220_132, "streaming": 11_220_132,
           "large": 1_000_000_000, "diagnostic": 124_439_808}


def spec(name: str, seed: int = 0, P: Optional[int] = None, N: Optional[int] = None) -> Workload:
    """Host-side description of a workload (no P-length data is drawn)."""
    if name not in NAMES:
        raise KeyError("unknown workload %r (have %s)" % (name, ", ".join(NAMES)))
    rng = np.random.Generator(np.random.Philox(key=[seed, NAMES.index(name)]))
    P = _FULL_P[name] if P is None else int(P)
    if name == "tiny":
        n = 4 if N is None else N
        base = [1.0, 1.0, -1.0, 1.0]
        sign = [base[i % 4] for i in range(n)]
        return Workload(name, n, P, "f32", 0.97, "aggregate", seed,
                        rho=[0.3] * n, sign=sign, scale=[1.0] * n)
    if name == "resnet18":
        n = 8 if N is None else N
        rho = rng.uniform(0.0, 0.2, n).tolist()
        sign = np.where(rng.random(n) < 0.25, -1.0, 1.0).tolist()
        scale = rng.lognormal(0.0, 0.5, n).tolist()
        return Workload(name, n, P, "f32", 0.97, "aggregate", seed, rho=rho, sign=sign, scale=scale)
    if name == "streaming":
        n = 32 if N is None else N
        sign = np.where(rng.random(n) < 0.5, -1.0, 1.0)
        sign[0] = 1.0
        return Workload(name, n, P, "f32", 1.0, "step", seed,
                        rho=[0.01] * n, sign=sign.tolist(), scale=[1.0] * n)
    if name == "large":
        n = 16 if N is None else N
        sign = np.where(rng.random(n) < 0.3, -1.0, 1.0).tolist()
        return Workload(name, n, P, "bf16", 0.98, "aggregate", seed,
                        rho=[0.1] * n, sign=sign, scale=[1.0] * n, noise="student_t3")
    n = 64 if N is None else N
    return Workload(name, n, P, "f32", 0.95, "pairwise", seed,
                    rho=[0.36] * n, sign=[1.0] * n, scale=[1.0] * n,
                    cluster=[i % 4 for i in range(n)])


def _normal(n, gen, device):
    return torch.randn(n, generator=gen, device=device, dtype=torch.float32)


def _noise(kind, n, gen, device):
    z = _normal(n, gen, device)
    if kind == "student_t3":
        # t_3 = Z / sqrt(chi2_3 / 3); dividing by sqrt(Var t_3) = sqrt(3) gives
        # Z / sqrt(chi2_3), unit variance with cubic tails.
        chi2 = _normal(n, gen, device).square_()
        chi2 += _normal(n, gen, device).square_()
        chi2 += _normal(n, gen, device).square_()
        z /= chi2.sqrt_()
    return z


def generate(name: str, seed: int = 0, P: Optional[int] = None, N: Optional[int] = None,
             device="cpu"):
    """Draw the workload. Returns (Workload, [N tensors of length P on `device`])."""
    w = spec(name, seed, P, N)
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(1_000_003 * seed + NAMES.index(name))
    P = w.P
    if w.cluster is None:
        centres = [_chunked(lambda n: _normal(n, gen, device), P, device)]
        which = [0] * w.N
        cw = [s * np.sqrt(r) for s, r in zip(w.sign, w.rho)]
        zw = [np.sqrt(1.0 - r) for r in w.rho]
    else:
        c0 = _chunked(lambda n: _normal(n, gen, device), P, device)
        c1 = _chunked(lambda n: _normal(n, gen, device), P, device)
        c2 = _chunked(lambda n: _normal(n, gen, device), P, device)
        c2.mul_(0.5 / np.sqrt(1.25)).add_(c0, alpha=-1.0 / np.sqrt(1.25))
        c3 = _chunked(lambda n: _normal(n, gen, device), P, device)
        centres = [c0, c1, c2, c3]
        which = w.cluster
        cw = [0.6] * w.N
        zw = [0.8] * w.N
    grads = []
    for i in range(w.N):
        g = torch.empty(P, dtype=w.torch_dtype, device=device)
        c = centres[which[i]]
        for lo in range(0, P, _CHUNK):
            hi = min(P, lo + _CHUNK)
            z = _noise(w.noise, hi - lo, gen, device)
            z.mul_(float(zw[i])).add_(c[lo:hi], alpha=float(cw[i]))
            if w.scale[i] != 1.0:
                z.mul_(float(w.scale[i]))
            g[lo:hi] = z.to(w.torch_dtype)
        grads.append(g)
    return w, grads


def _chunked(draw, P, device):
    out = torch.empty(P, dtype=torch.float32, device=device)
    for lo in range(0, P, _CHUNK):
        hi = min(P, lo + _CHUNK)
        out[lo:hi] = draw(hi - lo)
    return out


def to_host_array(t: torch.Tensor) -> np.ndarray:
    """Host numpy view of a gradient with its exact bits: float32, or uint16
    holding the bfloat16 patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError("unsupported gradient dtype %s" % t.dtype)
