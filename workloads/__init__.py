"""Seeded synthetic inputs for the bidirectional Top_K step, and the config table.

This module serves both the HIP path's tests/benchmark and the CPU oracle's
tests.  It contains none of the method's arithmetic: it only draws numbers.
Every draw is a pure function of (seed, config, step, worker, coordinate) through
a counter-based generator (SplitMix64's published output mix applied to a
per-stream key plus the coordinate), written with torch integer ops so the same
uniform bits come out on the CPU and on the GPU.  The floating-point transforms
(log, sqrt, cos) may differ in the last bit between devices, which does not
matter: a test always hands the *same generated buffer* to both sides.

The five configurations stand in for the paper's training workloads (MNIST,
Fashion-MNIST and CIFAR10 models, 20-100 workers, K = 0.1 % of d): N synchronous
workers, one flat fp32 d-vector per worker, K a small fixed fraction of d.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np
import torch

BASE_SEED = 20221001

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MIX1 = 0xBF58476D1CE4E5B9
_MIX2 = 0x94D049BB133111EB


def _s64(v: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 holds for those bits."""
    v &= _M64
    return v - (1 << 64) if v >= (1 << 63) else v


def _mix_int(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _MIX1) & _M64
    z = ((z ^ (z >> 27)) * _MIX2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, *words: int) -> int:
    """Fold a tuple of small integers (config, step, worker, stream id) into a 64-bit key."""
    k = _mix_int(seed)
    for w in words:
        k = _mix_int(k ^ ((w + 1) * _GOLDEN))
    return k


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 bit patterns."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def hash_bits(key: int, start: int, count: int, device) -> torch.Tensor:
    """64 pseudo-random bits (as int64) for counters start .. start+count-1 of a stream."""
    i = torch.arange(start, start + count, dtype=torch.int64, device=device)
    z = i * _s64(_GOLDEN) + _s64(key)
    z = (z ^ _lsr(z, 30)) * _s64(_MIX1)
    z = (z ^ _lsr(z, 27)) * _s64(_MIX2)
    return z ^ _lsr(z, 31)


def _u24_hi(z: torch.Tensor) -> torch.Tensor:
    return _lsr(z, 40)                        # top 24 bits, 0 .. 2^24-1


def _u24_lo(z: torch.Tensor) -> torch.Tensor:
    return _lsr(z, 16) & 0xFFFFFF             # next 24 bits


def normal_from_bits(z: torch.Tensor) -> torch.Tensor:
    """Standard normal by Box-Muller from one 64-bit word per value (fp32)."""
    u1 = (_u24_hi(z) + 1).to(torch.float32) * (1.0 / (1 << 24))       # (0, 1]
    u2 = _u24_lo(z).to(torch.float32) * (1.0 / (1 << 24))             # [0, 1)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def laplace_from_bits(z: torch.Tensor) -> torch.Tensor:
    """Laplace(0, 1) by inverse CDF."""
    # centred integer first, so that every step is exact in fp32 and |u| < 0.5 strictly
    u = ((_u24_hi(z) - (1 << 23)).to(torch.float32) + 0.5) * (1.0 / (1 << 24))
    return -torch.sign(u) * torch.log1p(-2.0 * torch.abs(u))


def student_t2_from_bits(z: torch.Tensor) -> torch.Tensor:
    """Student-t with 2 degrees of freedom by its closed-form inverse CDF."""
    # 23 bits: (k + 0.5) / 2^23 is exact in fp32 and stays strictly inside (0, 1)
    u = (_lsr(z, 41).to(torch.float32) + 0.5) * (1.0 / (1 << 23))
    return (2.0 * u - 1.0) / torch.sqrt(2.0 * u * (1.0 - u))


def k_from_fraction(d: int, num: int, den: int) -> int:
    """K = d - floor((1 - num/den) d), the rule of the paper's experiments section, in
    exact integer arithmetic (equals ceil(num d / den))."""
    return d - ((den - num) * d) // den


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    cfg_id: int
    N: int
    d: int
    K_up: int
    K_dn: int
    steps: int
    dist: str                 # normal | shared_normal | laplace | student_dup | segments
    p_kind: str = "uniform"   # uniform | dirichlet
    alpha: float = 0.01
    n_segments: int = 200

    @property
    def seed(self) -> int:
        return BASE_SEED + self.cfg_id

    def scaled(self, d: int, N: Optional[int] = None, steps: Optional[int] = None) -> "Config":
        """Same recipe at a smaller d (K keeps its fraction of d), for tests the oracle
        finishes in seconds."""
        fu = (self.K_up, self.d)
        fd = (self.K_dn, self.d)
        return dataclasses.replace(
            self, name=f"{self.name}@d={d}", d=d, N=self.N if N is None else N,
            K_up=max(1, -(-fu[0] * d // fu[1])), K_dn=max(1, -(-fd[0] * d // fd[1])),
            steps=self.steps if steps is None else steps,
            n_segments=min(self.n_segments, max(2, d // 64)))


def _mk(name, cfg_id, N, d, up, dn, steps, dist, p_kind="uniform"):
    return Config(name, cfg_id, N, d, k_from_fraction(d, *up), k_from_fraction(d, *dn), steps,
                  dist, p_kind)


CONFIGS: Dict[str, Config] = {
    "C1": _mk("C1", 1, 4, 1 << 20, (1, 1000), (1, 1000), 3, "normal"),
    "C2": _mk("C2", 2, 16, 11_173_962, (1, 100), (1, 100), 10, "shared_normal"),
    "C3": _mk("C3", 3, 32, 25_557_032, (1, 1000), (1, 1000), 10, "laplace"),
    "C4": _mk("C4", 4, 64, 25_557_032, (1, 1000), (1, 2000), 10, "student_dup", "dirichlet"),
    "C5": _mk("C5", 5, 64, 110_000_000, (1, 10000), (1, 10000), 5, "segments"),
}

# stream ids
_S_GRAD, _S_SHARED, _S_DUP_PICK, _S_DUP_PARTNER, _S_CUTS, _S_SCALES, _S_P, _S_W = range(8)


def p_weights(cfg: Config) -> np.ndarray:
    """Worker weights p_q (fp32, length N)."""
    if cfg.p_kind == "uniform":
        return np.full(cfg.N, 1.0 / cfg.N, dtype=np.float32)
    z = hash_bits(stream_key(cfg.seed, _S_P), 0, cfg.N, "cpu")
    u = ((_lsr(z, 11).to(torch.float64) + 0.5) / float(1 << 53)).numpy()
    e = -np.log(u)                       # Exp(1) draws; normalised -> Dirichlet(1)
    return (e / e.sum()).astype(np.float32)


def weights0(cfg: Config, device) -> torch.Tensor:
    """w_0 ~ N(0, 0.01) (variance), fp32 length d."""
    z = hash_bits(stream_key(cfg.seed, _S_W), 0, cfg.d, device)
    return normal_from_bits(z) * 0.1


def _segment_scale(cfg: Config, device) -> torch.Tensor:
    """Per-coordinate scale for the segmented config: n_segments contiguous segments with
    hashed cut points (same for every worker and step), scale 10^U(-5,-1) per segment."""
    ns = cfg.n_segments
    z = hash_bits(stream_key(cfg.seed, _S_CUTS), 0, 4 * ns, "cpu")
    cand = (1 + (_lsr(z, 1) % (cfg.d - 1))).numpy()
    cuts = []
    seen = set()
    for c in cand:
        c = int(c)
        if c not in seen:
            seen.add(c)
            cuts.append(c)
        if len(cuts) == ns - 1:
            break
    cuts = torch.tensor(sorted(cuts), dtype=torch.int64)
    zs = hash_bits(stream_key(cfg.seed, _S_SCALES), 0, ns, "cpu")
    u = (_u24_hi(zs).to(torch.float64) + 0.5) / float(1 << 24)
    scales = torch.pow(10.0, -5.0 + 4.0 * u).to(torch.float32)
    seg = torch.bucketize(torch.arange(cfg.d, dtype=torch.int64, device=device),
                          cuts.to(device), right=True)
    return scales.to(device)[seg]


class GradientSource:
    """Draws g_t (N x d fp32) for a config; caches what is shared across rows/steps."""

    def __init__(self, cfg: Config, device):
        self.cfg = cfg
        self.device = torch.device(device)
        self._scale = _segment_scale(cfg, self.device) if cfg.dist == "segments" else None

    def row(self, step: int, q: int) -> torch.Tensor:
        cfg, dev = self.cfg, self.device
        z = hash_bits(stream_key(cfg.seed, _S_GRAD, step, q), 0, cfg.d, dev)
        if cfg.dist == "normal":
            return normal_from_bits(z)
        if cfg.dist == "shared_normal":
            sigma = math.sqrt(1e-3)
            zs = hash_bits(stream_key(cfg.seed, _S_SHARED, step), 0, cfg.d, dev)
            return normal_from_bits(zs) * sigma + normal_from_bits(z) * sigma
        if cfg.dist == "laplace":
            return laplace_from_bits(z) * 1e-3
        if cfg.dist == "student_dup":
            g = student_t2_from_bits(z) * 1e-3
            pick = hash_bits(stream_key(cfg.seed, _S_DUP_PICK, q), 0, cfg.d, dev)
            dup = (_lsr(pick, 8) % 20) == 0                       # fixed 5 % of coordinates
            part = hash_bits(stream_key(cfg.seed, _S_DUP_PARTNER, q), 0, cfg.d, dev)
            partner = _lsr(part, 1) % cfg.d
            mag = torch.abs(g)[partner]
            return torch.where(dup, torch.copysign(mag, g), g)
        if cfg.dist == "segments":
            return normal_from_bits(z) * self._scale
        raise ValueError(cfg.dist)

    def fill(self, step: int, out: torch.Tensor) -> torch.Tensor:
        """Write g for `step` into out (N x d, fp32, on self.device)."""
        assert out.shape == (self.cfg.N, self.cfg.d) and out.dtype == torch.float32
        for q in range(self.cfg.N):
            out[q].copy_(self.row(step, q))
        return out

    def step(self, step: int) -> torch.Tensor:
        out = torch.empty((self.cfg.N, self.cfg.d), dtype=torch.float32, device=self.device)
        return self.fill(step, out)


def checksum(t: torch.Tensor) -> int:
    """64-bit wrap-around sum of the fp32 bit patterns (logged so runs can be compared).
    A matrix is summed row by row (the widened copy of a 28 GB batch would not fit)."""
    if t.dim() >= 2:
        return sum(checksum(r) for r in t) & _M64
    return int(t.contiguous().view(torch.int32).to(torch.int64).sum().item()) & _M64
