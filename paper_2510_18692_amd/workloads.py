"""Seeded synthetic video-token workloads for the MoGA hot path.

This module only draws inputs.  It holds none of the method's arithmetic
(no routing, no softmax, no permutation): the CPU oracle and the HIP library
both consume the tensors made here, and neither side imports the other.

Shapes follow the 480p latent grid of the paper's experiments: 30 x 52 = 1,560
tokens per latent frame (Table 5 sequence lengths are multiples of 1,560),
hidden size / heads of the two backbones it fine-tunes (1,536 / 12 and
5,120 / 40, head_dim 128), and a context of about 580k tokens (Section 4,
training settings).  No dataset is read: hidden states are i.i.d. Gaussian or
a Gaussian mixture whose component means are aligned with router rows, so that
a router applied to them produces balanced or deliberately unbalanced groups.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    N: int            # tokens (batch 1)
    H: int            # heads
    D: int            # head_dim
    d_model: int      # router input dim
    M: int            # groups
    dtype: str        # "f32" | "bf16": storage type of X, Q, K, V, dO
    hidden: str       # "iid" | "mixture" | "mixture_unaligned"
    weights: str = "uniform"   # mixture component weights: "uniform" | "zipf"
    zipf_s: float = 1.1        # exponent of the Zipf weights: component k has weight (k + 1)^-zipf_s
    absent: int = 0            # this many of the rarest components get weight 0: their groups only
                               # receive tokens that the noise pushes there (near-empty groups)
    align: float = 4.0         # length of the component mean along its router row
    noise_var: float = 1.0     # variance of the isotropic noise added to the mean
    backward: bool = False
    seed: int = 1000
    grid: str = ""             # latent grid the token count stands for

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def scale(self) -> float:
        return float(self.D) ** -0.5


WORKLOADS = {
    # tiny fp32 case the oracle finishes in seconds (latent grid 4 x 32 x 32)
    "C1": Workload("C1", 4096, 2, 64, 128, 8, "f32", "iid", seed=1001, grid="4x32x32"),
    "C1b": Workload("C1b", 4096, 2, 64, 128, 8, "f32", "iid", backward=True, seed=1001,
                    grid="4x32x32"),
    # 21 latent frames x 30 x 52, 1.3B-class backbone shape
    "C2": Workload("C2", 32760, 12, 128, 1536, 8, "bf16", "iid", seed=1002, grid="21x30x52"),
    # 64 frames, 14B-class shape, Zipf(1.1) mixture -> unbalanced groups
    "C3": Workload("C3", 99840, 40, 128, 5120, 16, "bf16", "mixture", weights="zipf",
                   seed=1003, grid="64x30x52"),
    "C3b": Workload("C3b", 99840, 40, 128, 5120, 16, "bf16", "mixture_unaligned",
                    weights="zipf", seed=1013, grid="64x30x52"),
    # C3 shapes, forward + backward, with the ~50x span of group sizes that configuration 3 asks
    # for and near-empty groups: Zipf(1.1) over 16 components spans only 16^1.1 = 21x, so the
    # exponent is raised to 1.45 (14^1.45 = 46x over the 14 components that are present) and the
    # two rarest components are left out, so that two groups receive only stray tokens
    "C3u": Workload("C3u", 99840, 40, 128, 5120, 16, "bf16", "mixture", weights="zipf",
                    zipf_s=1.45, absent=2, align=5.0, backward=True, seed=1023, grid="64x30x52"),
    # paper-scale context: 372 frames
    "C4": Workload("C4", 580320, 40, 128, 5120, 32, "bf16", "mixture", noise_var=0.5,
                   seed=1004, grid="372x30x52"),
    "C4b": Workload("C4b", 580320, 40, 128, 5120, 32, "bf16", "mixture", noise_var=0.5,
                    backward=True, seed=1004, grid="372x30x52"),
    # C3 shapes with backward
    "C5": Workload("C5", 99840, 40, 128, 5120, 16, "bf16", "mixture", weights="zipf",
                   backward=True, seed=1005, grid="64x30x52"),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of `w` with some fields replaced (used by tests to shrink a config)."""
    return replace(w, **kw)


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, gen, device, dtype, std=1.0, chunk_rows=65536):
    """N(0, std^2) drawn in float32, stored as `dtype`; drawn in row chunks to bound temporaries."""
    out = torch.empty(shape, device=device, dtype=dtype)
    n = shape[0]
    for s in range(0, n, chunk_rows):
        e = min(n, s + chunk_rows)
        t = torch.randn((e - s,) + tuple(shape[1:]), generator=gen, device=device,
                        dtype=torch.float32)
        if std != 1.0:
            t.mul_(std)
        out[s:e] = t.to(dtype)
    return out


def make_inputs(w: Workload, device="cpu"):
    """Draw every input tensor of workload `w` on `device` from its seed.

    Returns a dict of torch tensors:
      W  [M, d_model] float32, N(0, 1/d_model)
      X  [N, d_model] storage dtype: N(0, I), or mean_k + N(0, noise_var I) for a mixture
      Q, K, V [N, H, D] storage dtype, N(0, 1)
      dO [N, H, D] storage dtype, N(0, 1)  (only when w.backward)
      component [N] int64 mixture component of each token (zeros for "iid")
    Values depend on (seed, device type); both sides of a parity test read the same tensors.
    """
    dev = torch.device(device)
    gen = _gen(dev, w.seed)
    dt = w.torch_dtype
    N, H, D, d, M = w.N, w.H, w.D, w.d_model, w.M
    W = torch.randn((M, d), generator=gen, device=dev, dtype=torch.float32) * (d ** -0.5)
    if w.hidden == "iid":
        X = _randn((N, d), gen, dev, dt)
        comp = torch.zeros(N, dtype=torch.int64, device=dev)
    else:
        if w.weights == "zipf":
            pk = torch.arange(1, M + 1, dtype=torch.float64, device=dev) ** -w.zipf_s
            if w.absent > 0:
                pk[M - w.absent:] = 0.0
        else:
            pk = torch.ones(M, dtype=torch.float64, device=dev)
        pk = (pk / pk.sum()).to(torch.float32)
        comp = torch.multinomial(pk, N, replacement=True, generator=gen)
        if w.hidden == "mixture":
            means = w.align * W / W.norm(dim=1, keepdim=True)
        else:  # component means not aligned with router rows: components collide in groups
            means = w.align * torch.randn((M, d), generator=gen, device=dev,
                                          dtype=torch.float32) * (d ** -0.5)
        X = torch.empty((N, d), device=dev, dtype=dt)
        std = w.noise_var ** 0.5
        step = 65536
        for s in range(0, N, step):
            e = min(N, s + step)
            t = torch.randn((e - s, d), generator=gen, device=dev, dtype=torch.float32)
            if std != 1.0:
                t.mul_(std)
            t.add_(means[comp[s:e]])
            X[s:e] = t.to(dt)
    out = {"W": W, "X": X, "component": comp}
    for name in ("Q", "K", "V"):
        out[name] = _randn((N, H, D), gen, dev, dt, chunk_rows=max(1, (1 << 26) // (H * D)))
    if w.backward:
        out["dO"] = _randn((N, H, D), gen, dev, dt, chunk_rows=max(1, (1 << 26) // (H * D)))
    return out


def to_numpy64(t: torch.Tensor):
    """Exact widening of a stored tensor (f32 or bf16) to a float64 numpy array on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()
