"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws numbers: it holds none of the quantiser's arithmetic and
is shared by the tests of the CPU oracle and by the GPU path.  The parameter
vectors of the paper's experiments (Sec. 5: ResNet / AlexNet / VGG sized models)
are not available, so each configuration keeps only the model's parameter count
as its dimension and fills it with a stated distribution.

Every worker vector is generated from its own ``torch.Generator`` seeded by
``(config seed, stream id)``, on the requested device.  CPU and GPU generators
give different numbers for the same seed; a comparison always feeds both sides
the same tensor.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    d: int            # dimension of the parameter vector
    K: int            # simulated workers
    s: int            # magnitude levels {0..s-1}
    bucket: int       # bucket size (>= d means one bucket)
    rounds: int
    seed: int
    entries: str      # distribution of each worker's deviation vector
    w0: str           # distribution of the epoch snapshot
    model: str        # the model whose parameter count d is

    def scaled(self, d: int, K: Optional[int] = None, bucket: Optional[int] = None) -> "Workload":
        """Same distributions at another size (parity tests use small sizes)."""
        return replace(self, d=d, K=self.K if K is None else K,
                       bucket=self.bucket if bucket is None else bucket,
                       name=f"{self.name}@d={d}")


CONFIGS = [
    Workload("cfg1", 16_384, 4, 4, 16_384, 1, 0, "normal(0,1e-2)", "normal(0,1)", "toy"),
    Workload("cfg2", 1_048_576, 8, 16, 512, 10, 1, "normal(0,1e-3)", "uniform(-0.1,0.1)",
             "logistic-regression-shaped"),
    Workload("cfg3", 11_173_962, 8, 4, 2_048, 10, 2, "normal(0,sigma_b) sigma_b~logU[1e-5,1e-2]",
             "normal(0,5e-2)", "ResNet-18-sized"),
    Workload("cfg4", 25_557_032, 16, 256, 8_192, 5, 3, "normal(0,1e-3) with 1% exact zeros",
             "normal(0,2e-2)", "ResNet-50-sized"),
    Workload("cfg5", 138_357_544, 8, 2, 4_096, 3, 4, "1e-4*student_t(3)", "normal(0,1e-2)",
             "VGG-16-sized"),
]


def by_name(name: str) -> Workload:
    for c in CONFIGS:
        if c.name == name:
            return c
    raise KeyError(name)


def _gen(device, seed: int, stream: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) << 20) + int(stream))
    return g


def worker_vector(cfg: Workload, k: int, device="cpu", out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Deviation vector of pool slot k (fp32, length d) for the configuration."""
    d = cfg.d
    g = _gen(device, cfg.seed, 1 + k)
    x = out if out is not None else torch.empty(d, dtype=torch.float32, device=device)
    assert x.numel() == d and x.dtype == torch.float32
    if cfg.name.startswith("cfg1"):
        x.normal_(0.0, 1e-2, generator=g)
    elif cfg.name.startswith("cfg2"):
        x.normal_(0.0, 1e-3, generator=g)
    elif cfg.name.startswith("cfg3"):
        B = min(cfg.bucket, d)
        nb = (d + B - 1) // B
        u = torch.rand(nb, generator=g, device=device, dtype=torch.float32)
        sigma = torch.pow(10.0, -5.0 + 3.0 * u)
        x.normal_(0.0, 1.0, generator=g)
        x.mul_(sigma.repeat_interleave(B)[:d])
    elif cfg.name.startswith("cfg4"):
        x.normal_(0.0, 1e-3, generator=g)
        zero = torch.rand(d, generator=g, device=device, dtype=torch.float32) < 0.01
        x.masked_fill_(zero, 0.0)
    elif cfg.name.startswith("cfg5"):
        x.normal_(0.0, 1.0, generator=g)
        den = torch.zeros(d, dtype=torch.float32, device=device)
        t = torch.empty(d, dtype=torch.float32, device=device)
        for _ in range(3):
            t.normal_(0.0, 1.0, generator=g)
            den.addcmul_(t, t)
        den.div_(3.0).sqrt_()
        x.div_(den).mul_(1e-4)
        # a chi-square draw that rounds to zero would give inf/nan; the path needs finite input
        x.nan_to_num_(nan=0.0, posinf=0.0, neginf=0.0)
    else:
        raise KeyError(cfg.name)
    return x


def worker_slab(cfg: Workload, device="cpu", stride: Optional[int] = None) -> torch.Tensor:
    """[K, stride] fp32 slab; row k holds pool vector k in its first d entries (rest zero)."""
    stride = slab_stride(cfg.d) if stride is None else stride
    slab = torch.zeros(cfg.K, stride, dtype=torch.float32, device=device)
    for k in range(cfg.K):
        worker_vector(cfg, k, device, out=slab[k, :cfg.d])
    return slab


def slab_stride(d: int) -> int:
    """Row stride (in floats) that keeps every row 256-byte aligned."""
    return (d + 63) // 64 * 64


def snapshot(cfg: Workload, device="cpu") -> torch.Tensor:
    """Epoch snapshot w_t (fp32, length d)."""
    g = _gen(device, cfg.seed, 0)
    w = torch.empty(cfg.d, dtype=torch.float32, device=device)
    if cfg.name.startswith("cfg1"):
        w.normal_(0.0, 1.0, generator=g)
    elif cfg.name.startswith("cfg2"):
        w.uniform_(-0.1, 0.1, generator=g)
    elif cfg.name.startswith("cfg3"):
        w.normal_(0.0, 5e-2, generator=g)
    elif cfg.name.startswith("cfg4"):
        w.normal_(0.0, 2e-2, generator=g)
    elif cfg.name.startswith("cfg5"):
        w.normal_(0.0, 1e-2, generator=g)
    else:
        raise KeyError(cfg.name)
    return w


def random_packed_words(n_words: int, seed: int, stream: int, device="cpu") -> torch.Tensor:
    """Uniform random 32-bit words (as int32 storage) -- any bit pattern is a valid code plane."""
    g = _gen(device, seed, 1000 + stream)
    return torch.randint(-2**31, 2**31, (n_words,), dtype=torch.int64, generator=g,
                         device=device).to(torch.int32)


def random_norms(n: int, seed: int, stream: int, device="cpu", lo=1e-4, hi=1e-1) -> torch.Tensor:
    """Positive bucket scales, log-uniform in [lo, hi]."""
    g = _gen(device, seed, 2000 + stream)
    u = torch.rand(n, generator=g, device=device, dtype=torch.float32)
    return (lo * torch.pow(torch.tensor(hi / lo, device=device), u)).to(torch.float32)
