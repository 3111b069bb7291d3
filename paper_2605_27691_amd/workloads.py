"""Seeded synthetic point sets standing in for the paper's datasets (Sec. 5.2).

This module only produces inputs: it holds none of the method's arithmetic and
is the one module that both the GPU tests/benchmark and the CPU checker's tests
use, so that both sides see the same bytes.  The public benchmark datasets the
paper measures on are not reproduced here; each recipe below takes only the
shape (points, dimensions, metric, element range) of one of them.

Recipes (number = position in the benchmark's list of configurations, counted from 1;
6 is this library's own addition):

1  20,000 x 32 fp32: 16 centres ~ U[-10,10]^32, uniform assignment,
   x = c + N(0,1).  k=16, squared L2.  Unit-test scale.
2  1,000,000 x 128 (shape of SIFT-1M): 1,024 centres ~ U[0,128]^128,
   x = round(clip(c + N(0,16^2), 0, 255)) stored as fp32, so every squared
   distance is an exact integer below 2^24.  k=32, squared L2.
3  1,000,000 x 96 (shape of DEEP, with a cosine metric): 4,096 centres
   ~ N(0,I), x = c + N(0,0.3^2), then each row scaled to unit length in fp32.
   k=32, 1 - <a,b>.
4  1,000,000 x 960 (shape of GIST): 256 centres; per-dimension scale
   s_j = (j+1)^-1.5; c = s * U[-10,10], x = c + s * N(0,1).  k=32, squared L2.
5  20,000,000 x 128 (one GPU's share of a ~1B-point set): 4,096 centres
   ~ U[-10,10]^128, x = c + N(0,1).  k=32, squared L2.
6  1,000,000 x 128, one connected cloud of low intrinsic dimension (what real
   descriptor sets look like to a graph search; the isolated clusters of the
   recipes above are islands of their k-NN graphs, which no walk can leave):
   z ~ N(0, I_16), x = z A + 0.05 N(0,1) with A (16 x 128) ~ N(0, 1/16).
   k=32, squared L2.  Used by the graph-search benchmark and tests.

`n` may be overridden to get a smaller set with the same per-cluster
population (the number of centres is scaled with n, at least 1).

Generation runs on the CPU with numpy (default, bit-reproducible anywhere) or,
for the large sets, on a torch device with a seeded torch.Generator (fast;
reproducible on the same device type).  Either way the caller hands the very
same array to every implementation it compares.
"""
from dataclasses import dataclass

import numpy as np

L2SQ, IP_UNIT, COSINE = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    d: int
    k: int
    metric: int
    n_centres: int
    seed: int


# number -> workload; the seeds are the ones the sets were first generated with
CONFIGS = {
    1: Workload("gmm16_20k_d32_l2", 20_000, 32, 16, L2SQ, 16, 0),
    2: Workload("u8gmm1024_1m_d128_l2", 1_000_000, 128, 32, L2SQ, 1024, 1),
    3: Workload("unitgmm4096_1m_d96_ip", 1_000_000, 96, 32, IP_UNIT, 4096, 2),
    4: Workload("powergmm256_1m_d960_l2", 1_000_000, 960, 32, L2SQ, 256, 3),
    5: Workload("gmm4096_20m_d128_l2", 20_000_000, 128, 32, L2SQ, 4096, 4),
    6: Workload("manifold16_1m_d128_l2", 1_000_000, 128, 32, L2SQ, 1, 5),
}


def number_of(name_or_number) -> int:
    """Workload number from a number or a workload name."""
    for num, w in CONFIGS.items():
        if str(name_or_number) == w.name or str(name_or_number) == str(num):
            return num
    raise ValueError(f"unknown workload {name_or_number!r}: use 1..{len(CONFIGS)} or one of "
                     + ", ".join(w.name for w in CONFIGS.values()))
LATENT_DIM = 16


def scaled(cfg: Workload, n: int) -> Workload:
    """Same recipe at n points, keeping the points-per-centre ratio."""
    nc = max(1, round(cfg.n_centres * n / cfg.n))
    return Workload(f"{cfg.name}@{n}", n, cfg.d, cfg.k, cfg.metric, nc, cfg.seed)


def _numpy_points(idx: int, w: Workload) -> np.ndarray:
    rng = np.random.default_rng(w.seed)
    n, d, nc = w.n, w.d, w.n_centres
    assign = rng.integers(0, nc, size=n)
    if idx == 1 or idx == 5:
        c = rng.uniform(-10.0, 10.0, size=(nc, d)).astype(np.float32)
        x = c[assign] + rng.standard_normal((n, d), dtype=np.float32)
    elif idx == 2:
        c = rng.uniform(0.0, 128.0, size=(nc, d)).astype(np.float32)
        x = c[assign] + 16.0 * rng.standard_normal((n, d), dtype=np.float32)
        x = np.rint(np.clip(x, 0.0, 255.0))
    elif idx == 3:
        c = rng.standard_normal((nc, d), dtype=np.float32)
        x = c[assign] + np.float32(0.3) * rng.standard_normal((n, d), dtype=np.float32)
        x = x.astype(np.float32)
        x /= np.sqrt((x.astype(np.float64) ** 2).sum(axis=1, keepdims=True)).astype(np.float32)
    elif idx == 4:
        s = ((np.arange(d, dtype=np.float64) + 1.0) ** -1.5).astype(np.float32)
        c = s * rng.uniform(-10.0, 10.0, size=(nc, d)).astype(np.float32)
        x = c[assign] + s * rng.standard_normal((n, d), dtype=np.float32)
    elif idx == 6:
        a = (rng.standard_normal((LATENT_DIM, d), dtype=np.float32) * np.float32(0.25))
        x = rng.standard_normal((n, LATENT_DIM), dtype=np.float32) @ a
        x += np.float32(0.05) * rng.standard_normal((n, d), dtype=np.float32)
    else:
        raise ValueError(idx)
    return np.ascontiguousarray(x, dtype=np.float32)


def _torch_points(idx: int, w: Workload, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(w.seed)
    n, d, nc = w.n, w.d, w.n_centres
    f32 = dict(device=device, dtype=torch.float32)
    assign = torch.randint(0, nc, (n,), generator=g, device=device)
    if idx == 1 or idx == 5:
        c = torch.rand(nc, d, generator=g, **f32) * 20.0 - 10.0
        x = c[assign]
        x += torch.randn(n, d, generator=g, **f32)
    elif idx == 2:
        c = torch.rand(nc, d, generator=g, **f32) * 128.0
        x = c[assign]
        x += 16.0 * torch.randn(n, d, generator=g, **f32)
        x = x.clamp_(0.0, 255.0).round_()
    elif idx == 3:
        c = torch.randn(nc, d, generator=g, **f32)
        x = c[assign]
        x += 0.3 * torch.randn(n, d, generator=g, **f32)
        x /= x.double().pow(2).sum(dim=1, keepdim=True).sqrt().float()
    elif idx == 4:
        s = (torch.arange(d, device=device, dtype=torch.float64) + 1.0).pow(-1.5).float()
        c = s * (torch.rand(nc, d, generator=g, **f32) * 20.0 - 10.0)
        x = c[assign]
        x += s * torch.randn(n, d, generator=g, **f32)
    elif idx == 6:
        a = torch.randn(LATENT_DIM, d, generator=g, **f32) * 0.25
        x = torch.randn(n, LATENT_DIM, generator=g, **f32) @ a
        x += 0.05 * torch.randn(n, d, generator=g, **f32)
    else:
        raise ValueError(idx)
    return x.contiguous()


def make(idx: int, n: int | None = None, device=None):
    """Points of workload number `idx` (1..6, optionally at a smaller n).

    device None -> numpy array on the host; a torch device -> torch tensor there.
    Returns (points, workload).
    """
    w = CONFIGS[idx] if n is None or n == CONFIGS[idx].n else scaled(CONFIGS[idx], n)
    if device is None:
        return _numpy_points(idx, w), w
    return _torch_points(idx, w, device), w


def sample_rows(n: int, m: int, seed: int = 12345) -> np.ndarray:
    """m distinct row indices in [0, n), ascending, int32 (for sampled checks)."""
    rng = np.random.default_rng(seed)
    return np.sort(rng.choice(n, size=min(m, n), replace=False)).astype(np.int32)
