"""Counter-based normal random values that are bit-identical on CPU and GPU.

Every K/V/Q element is a pure function of (seed, tensor tag, node key, token
index, head, dim) and never of where the element ends up in physical memory, so
permuting page placement or rebuilding an identical token path reproduces the
same logical values.  The construction uses only integer tensor operations
(64-bit wrapping multiply, xor, shifts) followed by a table gather, which is why
the CPU and the GPU produce the same bits: a 64-bit mixing function yields a
20-bit index into a table of standard-normal quantiles that is computed once on
the host in fp64 and rounded to fp32.  The resulting distribution is N(0,1)
discretised to 2^20 equiprobable levels (tails to about +-4.9 sigma).
"""

from __future__ import annotations

import functools

import numpy as np
import torch

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB
_ELEM = 0xD6E8FEB86659FD93
TABLE_BITS = 20


def _signed(x: int) -> int:
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_int(x: int) -> int:
    """SplitMix64 finaliser on Python ints (unsigned 64-bit)."""
    z = (x + _GOLDEN) & _M64
    z = ((z ^ (z >> 30)) * _MUL1) & _M64
    z = ((z ^ (z >> 27)) * _MUL2) & _M64
    return z ^ (z >> 31)


def hash_key(*parts: int) -> int:
    """Fold integers into one signed 64-bit key (host side, Python ints)."""
    h = 0x243F6A8885A308D3
    for p in parts:
        h = _mix_int(h ^ (int(p) & _M64))
    return _signed(h)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right of int64 tensors."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix_tensor(x: torch.Tensor) -> torch.Tensor:
    """SplitMix64 finaliser on int64 tensors; multiplication wraps modulo 2^64."""
    z = x + _signed(_GOLDEN)
    z = (z ^ _lsr(z, 30)) * _signed(_MUL1)
    z = (z ^ _lsr(z, 27)) * _signed(_MUL2)
    return z ^ _lsr(z, 31)


@functools.lru_cache(maxsize=None)
def _quantile_table_host() -> torch.Tensor:
    from scipy.special import ndtri
    n = 1 << TABLE_BITS
    u = (np.arange(n, dtype=np.float64) + 0.5) / n
    return torch.from_numpy(ndtri(u).astype(np.float32))


@functools.lru_cache(maxsize=None)
def _quantile_table(device: str) -> torch.Tensor:
    return _quantile_table_host().to(device)


def normal_values(seed: int, tag: int, node_keys, token_idx, n_heads: int, head_dim: int,
                  scale: float = 1.0, device="cpu") -> torch.Tensor:
    """fp32 tensor [n_tok, n_heads, head_dim] of scale * N(0,1) samples.

    node_keys and token_idx are per-token int64 tensors (or Python ints / ranges):
    token t of the result is keyed by (seed, tag, node_keys[t], token_idx[t]).
    scale must be a power of two so that scaling is exact.
    """
    device = torch.device(device)
    token_idx = torch.as_tensor(token_idx, dtype=torch.int64, device=device).reshape(-1)
    node_keys = torch.as_tensor(node_keys, dtype=torch.int64, device=device).reshape(-1)
    if node_keys.numel() == 1 and token_idx.numel() != 1:
        node_keys = node_keys.expand(token_idx.numel())
    base = _signed(_mix_int((int(seed) & _M64) * 0x100000001B3 + int(tag)))
    tok = _mix_tensor(_mix_tensor(node_keys ^ base) + token_idx * _signed(_GOLDEN))
    lane = (torch.arange(n_heads * head_dim, dtype=torch.int64, device=device) + 1) * _signed(_ELEM)
    h = _mix_tensor(tok[:, None] + lane[None, :])
    idx = _lsr(h, 64 - TABLE_BITS)
    vals = _quantile_table(str(device))[idx]
    if scale != 1.0:
        vals = vals * scale
    return vals.reshape(-1, n_heads, head_dim)
