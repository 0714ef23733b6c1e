"""Named synthetic workloads (shapes, stage plans, needle recipe).

Shapes follow Llama-3-8B attention (32 query heads, 8 KV heads, d = 128).
Nothing here computes a score or a selection; needles are fabricated from q
by a fixed recipe so that some keys are known to matter.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import List, Tuple

import torch

from . import gen

# tensor ids of the counter-based generator
TID_Q, TID_K, TID_V, TID_NEEDLE_NOISE, TID_NEEDLE_POS = 1, 2, 3, 4, 5


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    T: int                      # keys visible (context including the new tokens)
    Tq: int = 1                 # new query tokens (1 = decode)
    b_q: int = 1                # query block size
    Hq: int = 32
    Hkv: int = 8
    d: int = 128
    n_sink: int = 128
    n_stream: int = 1024
    # pruning stages: (chunk size l_c, chunks kept K = k / l_c)
    stages: Tuple[Tuple[int, int], ...] = ()
    n_needles: int = 16         # per (sequence, KV head); 0 = none
    needle_gain: float = 4.0
    needle_noise: float = 0.1

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def Mq(self) -> int:
        return self.Tq // self.b_q


CFG1 = Workload("cfg1-decode-8k", B=1, T=8192,
                stages=((64, 64), (16, 64), (4, 128)))
CFG2 = Workload("cfg2-decode-128k", B=1, T=131072,
                stages=((64, 512), (16, 512), (4, 512)))
CFG3 = Workload("cfg3-decode-1m-b8", B=8, T=1048576,
                stages=((256, 256), (64, 256), (16, 512), (4, 1024)))
CFG4 = Workload("cfg4-prefill-4k-on-256k", B=1, T=262144 + 4096, Tq=4096, b_q=64,
                stages=((64, 256), (16, 256)), n_needles=0)
CFG5 = Workload("cfg5-decode-3m-offload", B=1, T=3145728,
                stages=((256, 256), (64, 256), (16, 512), (4, 1024)))

# The preset the paper prints as its default (appendix "Hyperparameters": sink 256, window 1024, chunks
# 256 / 32 / 8 keeping 32K / 8K / 2K tokens), one sequence of 1M keys: context for the paper's own
# latency table, not one of the graded configurations.
PAPER_3K = Workload("paper-3k-preset-decode-1m", B=1, T=1048576, n_sink=256,
                    stages=((256, 128), (32, 256), (8, 256)))

BY_NAME = {w.name: w for w in (CFG1, CFG2, CFG3, CFG4, CFG5, PAPER_3K)}


def shrink(w: Workload, **kw) -> Workload:
    return replace(w, **kw)


def make_q(w: Workload, seed: int, device="cpu", kind="normal") -> torch.Tensor:
    fn = gen.normal_bf16 if kind == "normal" else gen.small_int_bf16
    return fn(seed, TID_Q, (w.B, w.Hq, w.Tq, w.d), device)


def make_kv(w: Workload, seed: int, device="cpu", kind="normal"):
    """K, V as contiguous bf16 [B,Hkv,T,d]."""
    shape = (w.B, w.Hkv, w.T, w.d)
    k = torch.empty(shape, dtype=torch.bfloat16, device=device)
    v = torch.empty(shape, dtype=torch.bfloat16, device=device)
    gen.fill_(k, seed, TID_K, kind)
    gen.fill_(v, seed, TID_V, kind)
    return k, v


def needle_rows(w: Workload, q: torch.Tensor, seed: int):
    """Positions [B,Hkv,n] (int64) and bf16 key rows [B,Hkv,n,d] of the planted
    needles: n distinct full stage-1 chunks of the middle range per (sequence,
    KV head), an arithmetic progression (offset + i*stride) mod n_chunks with a
    seeded offset and a seeded stride coprime to n_chunks; the key at the
    chunk's first position is gain*q_h/|q_h| + noise*N(0,1) for query head
    h = g*G + (i mod G), using the first query.  Computed on the CPU in fp32
    whatever device q lives on."""
    l1 = w.stages[0][0]
    E = (w.T - w.Tq) + w.b_q                      # first query block (decode: the only one)
    n_chunks = (E - w.n_sink - w.n_stream) // l1  # full chunks only
    n = w.n_needles
    assert n <= n_chunks
    q0 = q.detach()[:, :, 0].to("cpu", torch.float32)                       # [B,Hq,d]
    qn = q0 / q0.norm(dim=-1, keepdim=True)
    par = gen.uniform_ints(seed, TID_NEEDLE_POS, 2 * w.B * w.Hkv, 1 << 30).view(w.B, w.Hkv, 2)
    off = par[..., 0] % n_chunks
    stride = par[..., 1] % n_chunks
    for b in range(w.B):
        for g in range(w.Hkv):
            st = max(1, int(stride[b, g]))
            while math.gcd(st, n_chunks) != 1:
                st += 1
            stride[b, g] = st
    i = torch.arange(n, dtype=torch.int64)
    chunks = (off[..., None] + i * stride[..., None]) % n_chunks            # [B,Hkv,n]
    pos = w.n_sink + chunks * l1
    heads = (torch.arange(w.Hkv).view(1, -1, 1) * w.G + (i % w.G).view(1, 1, -1)).expand(w.B, -1, -1)
    qsel = torch.gather(qn, 1, heads.reshape(w.B, -1, 1).expand(-1, -1, w.d)).view(w.B, w.Hkv, n, w.d)
    noise = gen.normal_bf16(seed, TID_NEEDLE_NOISE, (w.B, w.Hkv, n, w.d)).float()
    rows = (w.needle_gain * qsel + w.needle_noise * noise).to(torch.bfloat16)
    return pos, rows


def plant_needles(w: Workload, k: torch.Tensor, q: torch.Tensor, seed: int) -> torch.Tensor:
    """Overwrite the needle rows of K in place; returns positions [B,Hkv,n]."""
    if w.n_needles == 0:
        return torch.empty((w.B, w.Hkv, 0), dtype=torch.int64)
    pos, rows = needle_rows(w, q, seed)
    bi = torch.arange(w.B).view(-1, 1, 1).expand_as(pos).to(k.device)
    gi = torch.arange(w.Hkv).view(1, -1, 1).expand_as(pos).to(k.device)
    k[bi, gi, pos.to(k.device)] = rows.to(k.device)
    return pos


def make_inputs(w: Workload, seed: int, device="cpu", kind="normal"):
    """(q, k, v, seq_lens, needle_positions) for one layer call."""
    q = make_q(w, seed, device, kind)
    k, v = make_kv(w, seed, device, kind)
    pos = plant_needles(w, k, q, seed) if kind == "normal" else \
        torch.empty((w.B, w.Hkv, 0), dtype=torch.int64)
    seq_lens = torch.full((w.B,), w.T, dtype=torch.int32, device=device)
    return q, k, v, seq_lens, pos
