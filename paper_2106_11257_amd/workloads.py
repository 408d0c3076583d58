"""Seeded synthetic gradient slabs shaped like the paper's workloads.

Input generation only -- nothing of the method's arithmetic lives here.  The
same arrays feed the HIP library (on the GPU) and the fp64 oracle (after a
device-to-host copy), so the generator cannot affect parity.

The real gradients of the paper's experiments (ResNet-18 on CIFAR-10 with 16
peers and 7 Byzantines, Sec. 4.1; ALBERT-large with 16 and 64 peers, Sec. 4.2
and App. I.3) are not available; these stand in for them with the same peer
counts, vector lengths, clipping radii, iteration caps and attack types
(sign flip and random direction amplified by lambda = 1000, inner-product
manipulation, a shifted-mean collusion), and seeded synthetic values.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch


@dataclass
class Workload:
    name: str
    cfg: int
    n: int
    d: int
    parts: int
    tau: float
    eps: float
    max_iters: int
    seed_inputs: int
    seed_z: int
    byzantine: List[int] = field(default_factory=list)
    G: Optional[torch.Tensor] = None      # fp32 [n, d]
    offsets: Optional[List[int]] = None   # parts + 1 entries (Split rule of App. D.1)

    @property
    def slab_bytes(self) -> int:
        return 4 * self.n * self.d


# (n, d, tau, max_iters) of the five benchmark configurations
_SHAPES = {
    1: ("cfg1_n16_d2^20_scaled_negation", 16, 1 << 20, 1.0, 50),
    2: ("cfg2_resnet18_n16_signflip_randdir", 16, 11_173_962, 1.0, 50),
    3: ("cfg3_albert_large_n64_student_t_shifted_mean", 64, 17_683_968, 0.5, 100),
    4: ("cfg4_n8_d2^28_zeros_and_huge_norm", 8, 1 << 28, 0.1, 30),
    5: ("cfg5_1p3B_n16_ipm", 16, 1_315_758_080, 1.0, 20),
}


def split_offsets(d: int, parts: int) -> List[int]:
    """Partition boundaries: the first d mod parts partitions are one longer."""
    q, r = divmod(d, parts)
    off = [0]
    for j in range(parts):
        off.append(off[-1] + q + (1 if j < r else 0))
    return off


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


_CHUNK = 1 << 26   # elements generated at a time


def _fill_normal(row: torch.Tensor, gen, scale: float, mu: Optional[torch.Tensor]) -> None:
    d = row.shape[0]
    for a in range(0, d, _CHUNK):
        b = min(d, a + _CHUNK)
        noise = torch.randn(b - a, generator=gen, device=row.device, dtype=torch.float32)
        if mu is not None:
            torch.add(mu[a:b], noise, alpha=scale, out=row[a:b])
        else:
            torch.mul(noise, scale, out=row[a:b])


def _fill_student_t3(row: torch.Tensor, gen, scale: float, mu: torch.Tensor) -> None:
    d = row.shape[0]
    for a in range(0, d, _CHUNK):
        b = min(d, a + _CHUNK)
        z = torch.randn(b - a, generator=gen, device=row.device, dtype=torch.float32)
        chi = torch.zeros_like(z)
        for _ in range(3):
            e = torch.randn(b - a, generator=gen, device=row.device, dtype=torch.float32)
            chi.addcmul_(e, e)
        z.div_(torch.sqrt(chi / 3.0))
        torch.add(mu[a:b], z, alpha=scale, out=row[a:b])


def _mean_rows(G: torch.Tensor, rows: List[int]) -> torch.Tensor:
    acc = torch.zeros(G.shape[1], dtype=torch.float32, device=G.device)
    for i in rows:
        acc.add_(G[i])
    acc.div_(len(rows))
    return acc


def make_workload(cfg: int, device="cuda", d: Optional[int] = None,
                  parts: Optional[int] = None, row_align: int = 32) -> Workload:
    """Builds configuration `cfg` (1..5).  `d` overrides the vector length (for
    reduced-size test cases with the same recipe); `parts` defaults to n; `row_align` is the
    multiple of floats the row stride of G is rounded up to (1: dense rows)."""
    name, n, d_full, tau, max_iters = _SHAPES[cfg]
    d = d_full if d is None else int(d)
    parts = n if parts is None else int(parts)
    seed_inputs = 0x5EED0000 + cfg
    wl = Workload(name=name if d == d_full else f"{name}_d{d}", cfg=cfg, n=n, d=d, parts=parts,
                  tau=tau, eps=1e-6, max_iters=max_iters, seed_inputs=seed_inputs,
                  seed_z=0xB7A2D000 + cfg)
    wl.offsets = split_offsets(d, parts)
    dev = torch.device(device)
    gen = _gen(dev, seed_inputs)
    # rows start on 128-byte boundaries (row stride = d rounded up to a multiple of row_align
    # floats): every 1 KiB a wavefront reads of a row is then 8 whole cache lines
    ld = (d + row_align - 1) // row_align * row_align
    G = torch.zeros((n, ld), dtype=torch.float32, device=dev)[:, :d]

    if cfg == 1:
        # g_i = mu + N(0,1); the last 3 peers send -10 * (their own gradient)
        mu = torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
        for i in range(n):
            _fill_normal(G[i], gen, 1.0, mu)
        wl.byzantine = [13, 14, 15]
        for i in wl.byzantine:
            G[i].mul_(-10.0)
    elif cfg == 2:
        # honest g_i = mu + 0.1 N(0,1); 4 sign-flippers and 3 peers sending a common
        # random direction, both amplified by lambda = 1000 (Sec. 4.1)
        mu = torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
        for i in range(n):
            _fill_normal(G[i], gen, 0.1, mu)
        wl.byzantine = list(range(9, 16))
        honest_mean = _mean_rows(G, list(range(9)))
        u = torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
        u.mul_(honest_mean.norm() / u.norm())
        for i in (9, 10, 11, 12):
            G[i].mul_(-1000.0)
        for i in (13, 14, 15):
            torch.mul(u, 1000.0, out=G[i])
    elif cfg == 3:
        # honest g_i = mu + 1e-3 * Student-t(3), mu ~ 1e-3 N(0,1); 12 colluders send the
        # honest mean shifted by 5 "standard deviations" along one fixed unit direction
        mu = torch.randn(d, generator=gen, device=dev, dtype=torch.float32).mul_(1e-3)
        honest = list(range(52))
        wl.byzantine = list(range(52, 64))
        for i in honest:
            _fill_student_t3(G[i], gen, 1e-3, mu)
        honest_mean = _mean_rows(G, honest)
        ms = 0.0
        for i in honest:
            ms += float((G[i] - honest_mean).double().pow(2).sum())
        s = math.sqrt(ms / len(honest))
        u = torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
        u.div_(u.norm())
        attack = honest_mean + (5.0 * s) * u
        for i in wl.byzantine:
            G[i].copy_(attack)
    elif cfg == 4:
        # honest g_i = mu + N(0, 0.01) (std 0.1); two all-zero peers; one huge-norm peer
        mu = torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
        for i in range(5):
            _fill_normal(G[i], gen, 0.1, mu)
        G[5].zero_()
        G[6].zero_()
        _fill_normal(G[7], gen, 1e6, None)
        wl.byzantine = [5, 6, 7]
    elif cfg == 5:
        # honest g_i = mu + sigma_j N(0,1), sigma_j log-uniform in [1e-4, 1e-1] per
        # partition; 4 peers send -0.5 * (honest mean) (inner-product manipulation)
        mu = torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
        cpu_gen = torch.Generator(device="cpu")
        cpu_gen.manual_seed(seed_inputs)
        expo = torch.rand(parts, generator=cpu_gen, dtype=torch.float64) * 3.0 - 4.0
        sigma = [10.0 ** float(e) for e in expo]
        honest = list(range(12))
        wl.byzantine = [12, 13, 14, 15]
        for i in honest:
            for j in range(parts):
                lo, hi = wl.offsets[j], wl.offsets[j + 1]
                if hi > lo:
                    _fill_normal(G[i, lo:hi], gen, sigma[j], mu[lo:hi])
        honest_mean = _mean_rows(G, honest)
        for i in wl.byzantine:
            torch.mul(honest_mean, -0.5, out=G[i])
    else:
        raise ValueError(f"unknown configuration {cfg}")
    wl.G = G
    return wl


def generic_case(n: int, d: int, parts: int, seed: int, device="cuda", ld: Optional[int] = None,
                 spread: float = 1.0, outliers: int = 0, outlier_scale: float = 50.0):
    """Small generic slab for edge-case tests: honest rows mu + spread*N(0,1), the last
    `outliers` rows scaled away.  Returns (G view [n, d] with row stride ld, offsets)."""
    dev = torch.device(device)
    gen = _gen(dev, 0xC0FFEE00 + seed)
    ld = d if ld is None else ld
    buf = torch.randn((n, ld), generator=gen, device=dev, dtype=torch.float32).mul_(spread)
    mu = torch.randn(ld, generator=gen, device=dev, dtype=torch.float32)
    buf.add_(mu[None, :])
    for i in range(n - outliers, n):
        buf[i].mul_(-outlier_scale)
    return buf[:, :d], split_offsets(d, parts)
