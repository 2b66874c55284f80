"""Counter-based seeded generator for the synthetic inputs.

Every value is a pure function of (seed, stream tags, element index), evaluated with 64-bit
integer arithmetic and one table lookup, so that the same call gives bit-identical results
on the host and on the GPU and any subset of elements can be produced on its own.  That is
what lets a full-size GPU run be checked against the CPU oracle on sampled coordinates: the
oracle's inputs for those coordinates are regenerated on the host, never copied from the GPU.

* bits:    splitmix64 stream, element i = finaliser(key + (i + 1) * golden-ratio increment)
* uniform: top 23 bits, (u + 1/2) / 2^23  (exact in fp32)
* normal:  top 20 bits index a table of standard-normal quantiles at the midpoints
           (i + 1/2) / 2^20 -- a normal law discretised to 2^20 equiprobable levels
           (|z| <= 4.9), built once on the host in fp64 and rounded to fp32.
"""
from __future__ import annotations

from dataclasses import dataclass
from functools import lru_cache
from typing import Dict, Optional, Sequence

import numpy as np
import torch

from .configs import Config
from .shapes import ParamSet

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_NBITS_NORMAL = 20
_CHUNK = 1 << 26        # elements generated per pass on large requests (bounds temporaries)


def _s64(u: int) -> int:
    """Reinterpret an unsigned 64-bit value as the signed value torch.int64 holds."""
    u &= _M64
    return u - (1 << 64) if u >= (1 << 63) else u


def _mix_py(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, *tags: int) -> int:
    """Hash (seed, tags...) to a 64-bit stream key (host-side Python integers)."""
    k = _mix_py(int(seed) + _GOLDEN)
    for t in tags:
        k = _mix_py((k ^ (int(t) & _M64)) + _GOLDEN)
    return k


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 (torch's >> is arithmetic)."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def random_bits(key: int, idx: torch.Tensor) -> torch.Tensor:
    """64 random bits per element of idx (int64 tensor of element indices), as int64."""
    z = idx * _s64(_GOLDEN) + _s64(key + _GOLDEN)
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def uniform01(key: int, idx: torch.Tensor) -> torch.Tensor:
    """fp32 uniform on (0, 1) with 2^23 levels."""
    u = _lsr(random_bits(key, idx), 64 - 23)
    return (u.to(torch.float32) + 0.5) * (1.0 / (1 << 23))


@lru_cache(maxsize=1)
def _normal_table_host() -> torch.Tensor:
    from scipy.special import ndtri
    n = 1 << _NBITS_NORMAL
    # symmetric by construction: build the upper half, mirror it
    p = (np.arange(n // 2, n, dtype=np.float64) + 0.5) / n
    upper = ndtri(p).astype(np.float32)
    table = np.concatenate([-upper[::-1], upper])
    return torch.from_numpy(table)


_table_cache: Dict[str, torch.Tensor] = {}


def _normal_table(device: torch.device) -> torch.Tensor:
    key = str(device)
    if key not in _table_cache:
        _table_cache[key] = _normal_table_host().to(device)
    return _table_cache[key]


def standard_normal(key: int, idx: torch.Tensor) -> torch.Tensor:
    """fp32 standard normal (discretised to 2^20 quantile midpoints) per element of idx."""
    u = _lsr(random_bits(key, idx), 64 - _NBITS_NORMAL)
    return _normal_table(idx.device)[u]


def _index(P: int, device, idx: Optional[torch.Tensor]) -> torch.Tensor:
    if idx is not None:
        return idx.to(device=device, dtype=torch.int64)
    return torch.arange(P, device=device, dtype=torch.int64)


def normal_like_flat(key: int, P: int, device="cpu", idx: Optional[torch.Tensor] = None,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Standard normal values for flat indices 0..P-1 (or for the given subset idx)."""
    if idx is not None:
        r = standard_normal(key, _index(P, device, idx))
        if out is not None:
            out.copy_(r)
            return out
        return r
    if out is None:
        out = torch.empty(P, dtype=torch.float32, device=device)
    for lo in range(0, P, _CHUNK):
        hi = min(P, lo + _CHUNK)
        ii = torch.arange(lo, hi, device=device, dtype=torch.int64)
        out[lo:hi] = standard_normal(key, ii)
    return out


# stream tags
_TAG_INIT, _TAG_GRAD, _TAG_H, _TAG_C, _TAG_CJ, _TAG_NOISE = 1, 2, 3, 4, 5, 6


def _per_element(params: ParamSet, per_tensor: Sequence[float], device,
                 idx: Optional[torch.Tensor]) -> torch.Tensor:
    """Expand one fp32 value per tensor to one per flat element (or per element of idx)."""
    vals = torch.tensor(list(per_tensor), dtype=torch.float32, device=device)
    if idx is None:
        counts = torch.tensor(params.numel, dtype=torch.int64, device=device)
        return torch.repeat_interleave(vals, counts)
    bounds = torch.tensor(params.offsets[1:], dtype=torch.int64, device=device)
    t = torch.bucketize(idx.to(device=device, dtype=torch.int64), bounds, right=True)
    return vals[t]


def init_std_per_tensor(cfg: Config) -> list:
    ps = cfg.params
    if cfg.init == "zero":
        return [0.0] * ps.n_tensors
    if cfg.init == "normal":
        return [cfg.init_std] * ps.n_tensors
    if cfg.init == "kaiming":
        return [float(np.sqrt(2.0 / ps.fan_in(t))) for t in range(ps.n_tensors)]
    raise ValueError(cfg.init)


def init_weights(cfg: Config, device="cpu", idx: Optional[torch.Tensor] = None) -> torch.Tensor:
    """w0 as one flat fp32 vector over the unpadded concatenation (the same for every replica:
    all local models start from one point, as the paper's analysis assumes, Lemma 1)."""
    P = cfg.P
    if cfg.init == "zero":
        n = P if idx is None else idx.numel()
        return torch.zeros(n, dtype=torch.float32, device=device)
    z = normal_like_flat(stream_key(cfg.seed, _TAG_INIT), P, device, idx)
    return z * _per_element(cfg.params, init_std_per_tensor(cfg), device, idx)


@lru_cache(maxsize=8)
def _grad_sigma_per_tensor(cfg: Config) -> tuple:
    """Per-tensor gradient std.  For relative configs: grad_rel * ||w0_t||_2 / sqrt(n_t), with the
    norm taken once at init, always on the host in fp64 so every consumer sees the same value."""
    ps = cfg.params
    if cfg.grad_rel == 0.0:
        return tuple([cfg.grad_std] * ps.n_tensors)
    w0 = init_weights(cfg, "cpu").double()
    out, off = [], ps.offsets
    for t in range(ps.n_tensors):
        n = ps.numel[t]
        nrm = float(torch.sqrt(torch.sum(w0[off[t]:off[t + 1]] ** 2)))
        out.append(float(np.float32(cfg.grad_rel * nrm / np.sqrt(n))))
    return tuple(out)


def grad_sigma_vector(cfg: Config, device="cpu", idx: Optional[torch.Tensor] = None) -> torch.Tensor:
    return _per_element(cfg.params, _grad_sigma_per_tensor(cfg), device, idx)


def gradient(cfg: Config, step: int, worker: int, device="cpu", idx: Optional[torch.Tensor] = None,
             sigma: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """External gradient of one worker at one step: sigma_t * N(0,1), flat fp32 of length P
    (or one value per element of idx).  `sigma` may pass a cached grad_sigma_vector."""
    if cfg.kind != "external":
        raise ValueError("gradient() is for configs whose gradients are pure inputs")
    if sigma is None:
        sigma = grad_sigma_vector(cfg, device, idx)
    z = normal_like_flat(stream_key(cfg.seed, _TAG_GRAD, step, worker), cfg.P, device, idx, out=out)
    return z.mul_(sigma)


@dataclass
class QuadraticProblem:
    """Worker j minimises 0.5 * sum_i h_i (w_i - c_ij)^2 with noisy gradients:
    g_j(w) = h * (w - c_j) + noise,  h ~ U[0.1, 1],  c ~ N(0,1),  c_j = c + 0.1 N(0,1)."""
    cfg: Config
    h: torch.Tensor            # [P]
    c: torch.Tensor            # [W, P]
    noise_std: float

    @classmethod
    def build(cls, cfg: Config, device="cpu", idx: Optional[torch.Tensor] = None,
              noise: bool = True) -> "QuadraticProblem":
        P = cfg.P
        ii = _index(P, device, idx)
        u = uniform01(stream_key(cfg.seed, _TAG_H), ii)
        h = (u.double() * 0.9 + 0.1).to(torch.float32)
        c0 = standard_normal(stream_key(cfg.seed, _TAG_C), ii)
        c = torch.stack([c0 + standard_normal(stream_key(cfg.seed, _TAG_CJ, j), ii) * 0.1
                         for j in range(cfg.W)])
        return cls(cfg, h, c, cfg.grad_std if noise else 0.0)

    def noise(self, step: int, worker: int, device, idx: Optional[torch.Tensor]) -> torch.Tensor:
        ii = _index(self.cfg.P, device, idx)
        z = standard_normal(stream_key(self.cfg.seed, _TAG_NOISE, step, worker), ii)
        return z * self.noise_std

    def grad(self, x_j: torch.Tensor, step: int, worker: int,
             idx: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Gradient of worker `worker` at its current iterate x_j, in x_j's dtype (the fp32
        inputs are widened exactly when x_j is fp64).  Three separately rounded operations."""
        dt = x_j.dtype
        g = (x_j - self.c[worker].to(dt)) * self.h.to(dt)
        if self.noise_std != 0.0:
            g = g + self.noise(step, worker, x_j.device, idx).to(dt)
        return g
