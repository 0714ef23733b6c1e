"""Seeded synthetic inputs, shared by the CPU oracle's tests and the GPU path.

This module holds no arithmetic of the method (no scores, no selection, no
softmax): it only fabricates Q/K/V tensors.  Values come from a counter-based
generator -- element value = f(seed, tensor id, linear element index) -- built
from integer torch ops and a table gather only, so the same call yields the
same bits on the CPU and on the GPU and any slice of a huge tensor can be
regenerated alone.
"""
from __future__ import annotations

import math
from functools import lru_cache

import torch

_M32 = 0xFFFFFFFF
# odd multipliers below 2**31, so that (x < 2**32) * c never overflows int64
_C1 = 0x7FEB352D
_C2 = 0x3243F6A9
_C3 = 0x1B873593


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """Avalanche a tensor of int64 values in [0, 2**32)."""
    x = x ^ (x >> 16)
    x = (x * _C1) & _M32
    x = x ^ (x >> 15)
    x = (x * _C2) & _M32
    x = x ^ (x >> 16)
    return x


def _seed_word(seed: int, tensor_id: int) -> int:
    s = (seed * 0x9E3779B1 + tensor_id * 0x85EBCA77 + 0x165667B1) & _M32
    # scalar avalanche, same recipe as _mix32
    s ^= s >> 16
    s = (s * _C1) & _M32
    s ^= s >> 15
    s = (s * _C2) & _M32
    s ^= s >> 16
    return s


def hash_u32(index: torch.Tensor, seed: int, tensor_id: int) -> torch.Tensor:
    """32 pseudo-random bits (as int64) per int64 element index."""
    sw = _seed_word(seed, tensor_id)
    lo = index & _M32
    hi = (index >> 32) & _M32
    h = _mix32(hi ^ sw)
    h = _mix32(lo ^ h)
    h = _mix32(((h * _C3) & _M32) ^ sw)
    return h


@lru_cache(maxsize=None)
def _normal_table_cpu() -> torch.Tensor:
    """65536 quantiles of N(0,1) at (i+0.5)/65536, rounded to bf16 (RNE)."""
    u = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
    z = math.sqrt(2.0) * torch.erfinv(2.0 * u - 1.0)
    return z.to(torch.float32).to(torch.bfloat16)


_table_cache: dict = {}


def normal_table(device) -> torch.Tensor:
    device = torch.device(device)
    key = str(device)
    if key not in _table_cache:
        _table_cache[key] = _normal_table_cpu().to(device)
    return _table_cache[key]


def _slice_index(full_shape, b0, b1, h0, h1, t0, t1, device) -> torch.Tensor:
    """Linear indices (int64) of the slice [b0:b1, h0:h1, t0:t1, :] of a
    contiguous [B,H,T,d] tensor."""
    B, H, T, d = full_shape
    bi = torch.arange(b0, b1, dtype=torch.int64, device=device).view(-1, 1, 1, 1)
    hi = torch.arange(h0, h1, dtype=torch.int64, device=device).view(1, -1, 1, 1)
    ti = torch.arange(t0, t1, dtype=torch.int64, device=device).view(1, 1, -1, 1)
    di = torch.arange(0, d, dtype=torch.int64, device=device).view(1, 1, 1, -1)
    return ((bi * H + hi) * T + ti) * d + di


def normal_bf16(seed, tensor_id, full_shape, device="cpu", sl=None) -> torch.Tensor:
    """bf16 ~ N(0,1) values of (a slice of) a logical [B,H,T,d] tensor.

    sl = (b0, b1, h0, h1, t0, t1) or None for everything."""
    B, H, T, d = full_shape
    if sl is None:
        sl = (0, B, 0, H, 0, T)
    idx = _slice_index(full_shape, *sl, device)
    h = hash_u32(idx, seed, tensor_id)
    return normal_table(device)[h & 0xFFFF]


def small_int_bf16(seed, tensor_id, full_shape, device="cpu", sl=None) -> torch.Tensor:
    """bf16 values uniform in {-2,-1,0,1,2}: every dot product of such
    vectors is a small integer, exact in fp32 in any summation order."""
    B, H, T, d = full_shape
    if sl is None:
        sl = (0, B, 0, H, 0, T)
    idx = _slice_index(full_shape, *sl, device)
    h = hash_u32(idx, seed, tensor_id)
    return ((h >> 8) % 5 - 2).to(torch.float32).to(torch.bfloat16)


def fill_(out: torch.Tensor, seed, tensor_id, kind="normal", t_step=None) -> torch.Tensor:
    """Fill a (possibly huge, possibly strided) [B,H,T,d] tensor in place, a
    bounded slab of tokens at a time, so temporaries stay small."""
    B, H, T, d = out.shape
    fn = normal_bf16 if kind == "normal" else small_int_bf16
    if t_step is None:              # ~0.3 G elements per slab on a GPU (few launches), 8 M on the CPU
        t_step = max(1, ((1 << 28) if out.is_cuda else (1 << 23)) // (H * d))
    for b in range(B):
        for t0 in range(0, T, t_step):
            t1 = min(T, t0 + t_step)
            out[b, :, t0:t1, :] = fn(seed, tensor_id, (B, H, T, d), out.device,
                                     (b, b + 1, 0, H, t0, t1))[0]
    return out


def uniform_ints(seed, tensor_id, n, modulus, device="cpu") -> torch.Tensor:
    """n pseudo-random int64 values in [0, modulus)."""
    idx = torch.arange(n, dtype=torch.int64, device=device)
    return hash_u32(idx, seed, tensor_id) % modulus


def distinct_ints(seed, tensor_id, n, modulus) -> torch.Tensor:
    """n distinct values in [0, modulus), in seeded random order (CPU)."""
    assert n <= modulus
    got, seen, i = [], set(), 0
    while len(got) < n:
        cand = uniform_ints(seed, tensor_id + 7919 * (i // 4096 + 1), 4096, modulus)
        for c in cand.tolist():
            if c not in seen:
                seen.add(c)
                got.append(c)
                if len(got) == n:
                    break
        i += 4096
    return torch.tensor(got, dtype=torch.int64)


def zipf_ranks(seed, tensor_id, n, modulus, exponent=1.1) -> torch.Tensor:
    """n draws (CPU, int64) from a Zipf(exponent) law truncated to ranks
    [0, modulus): P(rank r) ~ (r+1)**-exponent, by inverse-CDF lookup."""
    w = (torch.arange(1, modulus + 1, dtype=torch.float64)) ** (-exponent)
    cdf = torch.cumsum(w, 0)
    cdf = cdf / cdf[-1]
    u = (uniform_ints(seed, tensor_id, n, 1 << 24).to(torch.float64) + 0.5) / float(1 << 24)
    return torch.searchsorted(cdf, u).clamp_(max=modulus - 1)


def rope_table(n_pos: int, d: int, base: float = 10000.0, device="cpu"):
    """cos / sin (float32 [n_pos, d/2]) of position i times the angle base**(-2j/d) of frequency j:
    the rotary-embedding table of Su et al. for head dimension d."""
    j = torch.arange(d // 2, dtype=torch.float64)
    ang = torch.arange(n_pos, dtype=torch.float64).view(-1, 1) * base ** (-2.0 * j / d).view(1, -1)
    return ang.cos().to(torch.float32).to(device), ang.sin().to(torch.float32).to(device)


def quarter_turn_table(n_pos: int, d: int, device="cpu"):
    """A rotary table whose angles are whole quarter turns (frequency j turns (j+1) quarters per
    position), so cos and sin are exactly 0 or +-1 and rotating integer-valued vectors stays exact."""
    j = torch.arange(d // 2, dtype=torch.int64).view(1, -1)
    q = (torch.arange(n_pos, dtype=torch.int64).view(-1, 1) * (j + 1)) % 4
    cos = torch.tensor([1.0, 0.0, -1.0, 0.0])[q]
    sin = torch.tensor([0.0, 1.0, 0.0, -1.0])[q]
    return cos.to(torch.float32).to(device), sin.to(torch.float32).to(device)


def to_e4m3(x: torch.Tensor, scale: float) -> torch.Tensor:
    """Quantise a tensor to FP8 E4M3 bytes (uint8) with one scale: byte = e4m3(x / scale), values
    beyond the format's largest finite number (448) saturating to it."""
    y = (x.float() / scale).clamp_(-448.0, 448.0)
    return y.to(torch.float8_e4m3fn).view(torch.uint8)
