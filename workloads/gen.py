"""Counter-based, device-independent generator of bf16 test tensors.

Element i of tensor `tensor_id` under `seed` is table[h >> 48] where h is a splitmix64
hash of the counter and `table` holds the 65536 mid-point quantiles of N(0, 1) (scaled by
the requested std, rounded to bf16 with round-to-nearest-even).  Only integer arithmetic
and one table lookup run per element, so torch on the CPU and torch on the GPU return the
same bits, and the oracle and the HIP path read identical bytes wherever they were made.
The 16-bit quantile grid truncates the tails at about +-4.3 sigma.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from functools import lru_cache
from typing import List, Optional

import numpy as np
import torch

from .configs import MoEConfig

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1


def _i64(v: int) -> int:
    """Two's-complement reinterpretation of a 64-bit unsigned constant."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exact."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def torch_bf16_to_u16(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def u16_to_torch_bf16(a: np.ndarray, device="cpu") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)


@lru_cache(maxsize=None)
def _quantiles() -> np.ndarray:
    from scipy.special import ndtri
    p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
    return ndtri(p)


@lru_cache(maxsize=None)
def _table_bits(std: float) -> np.ndarray:
    z = (_quantiles() * float(std)).astype(np.float32)
    return f32_to_bf16_bits(z)


_dev_tables = {}


def _table(std: float, device) -> torch.Tensor:
    key = (float(std), str(device))
    if key not in _dev_tables:
        _dev_tables[key] = torch.from_numpy(_table_bits(float(std)).view(np.int16).copy()).to(device)
    return _dev_tables[key]


def _hash_index(seed: int, tensor_id: int, start: int, n: int, device) -> torch.Tensor:
    """Top 16 bits of splitmix64(key + (i+1)*GOLDEN), i = start..start+n-1, as int64 in [0, 65536)."""
    key = (seed * _M2 + tensor_id * _M1 + 0x1234567) & _MASK64
    i = torch.arange(start + 1, start + n + 1, dtype=torch.int64, device=device)
    z = i * _i64(_GOLDEN) + _i64(key)
    z = (z ^ ((z >> 30) & ((1 << 34) - 1))) * _i64(_M1)
    z = (z ^ ((z >> 27) & ((1 << 37) - 1))) * _i64(_M2)
    z = z ^ ((z >> 31) & ((1 << 33) - 1))
    return (z >> 48) & 0xFFFF


def hash_index_reference(seed: int, tensor_id: int, start: int, n: int) -> np.ndarray:
    """The same hash in numpy uint64 (wrapping) arithmetic; used by the generator's self-test."""
    key = np.uint64((seed * _M2 + tensor_id * _M1 + 0x1234567) & _MASK64)
    with np.errstate(over="ignore"):
        i = np.arange(start + 1, start + n + 1, dtype=np.uint64)
        z = i * np.uint64(_GOLDEN) + key
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
        z = z ^ (z >> np.uint64(31))
    return (z >> np.uint64(48)).astype(np.int64)


def normal_bf16(seed: int, tensor_id: int, shape, std: float = 1.0, device="cpu",
                chunk: int = 1 << 24) -> torch.Tensor:
    """bf16 tensor of `shape`, values ~ N(0, std^2) on the quantile grid, same bits on any device."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=torch.int16, device=device)
    tab = _table(std, device)
    for s in range(0, n, chunk):
        m = min(chunk, n - s)
        out[s:s + m] = tab[_hash_index(seed, tensor_id, s, m, device)]
    return out.view(torch.bfloat16).view(*shape)


def gate_bias(cfg: MoEConfig) -> Optional[np.ndarray]:
    """Per-expert additive gate-logit bias (float32 [E]) or None."""
    rng = np.random.default_rng(cfg.seed)
    if cfg.bias == "none":
        return None
    if cfg.bias == "normal":
        return rng.standard_normal(cfg.E).astype(np.float32)
    if cfg.bias == "logzipf_rank":
        rank = rng.permutation(cfg.E).astype(np.float64) + 1.0
        return (-1.1 * np.log(rank)).astype(np.float32)
    if cfg.bias == "logzipf_sample":
        return np.log(rng.zipf(1.1, cfg.E).astype(np.float64)).astype(np.float32)
    raise ValueError(cfg.bias)


# tensor ids: 0 = x, 1 = Wg, 16 + 3*e + {0,1,2} = W1/W3/W2 of expert e (routed first, then shared)
@dataclass
class LayerInputs:
    cfg: MoEConfig
    x: torch.Tensor                 # [T, H] bf16
    wg: torch.Tensor                # [H, E] bf16
    bias: Optional[np.ndarray]      # [E] float32 or None
    w1: List[torch.Tensor] = field(default_factory=list)   # E+Ns tensors [H, F] bf16 (gate proj)
    w3: List[torch.Tensor] = field(default_factory=list)   # E+Ns tensors [H, F] bf16 (up proj)
    w2: List[torch.Tensor] = field(default_factory=list)   # E+Ns tensors [F, H] bf16 (down proj)


def make_layer_inputs(cfg: MoEConfig, device="cpu", x_std: float = 1.0, w_std: float = 0.02,
                      experts: bool = True) -> LayerInputs:
    """All tensors of one synthetic MoE layer: x ~ N(0,1), Wg/W1/W3/W2 ~ N(0, 0.02^2), bf16."""
    li = LayerInputs(
        cfg=cfg,
        x=normal_bf16(cfg.seed, 0, (cfg.T, cfg.H), x_std, device),
        wg=normal_bf16(cfg.seed, 1, (cfg.H, cfg.E), w_std, device),
        bias=gate_bias(cfg),
    )
    if experts:
        for e in range(cfg.E + cfg.num_shared):
            li.w1.append(normal_bf16(cfg.seed, 16 + 3 * e, (cfg.H, cfg.F), w_std, device))
            li.w3.append(normal_bf16(cfg.seed, 17 + 3 * e, (cfg.H, cfg.F), w_std, device))
            li.w2.append(normal_bf16(cfg.seed, 18 + 3 * e, (cfg.F, cfg.H), w_std, device))
    return li
