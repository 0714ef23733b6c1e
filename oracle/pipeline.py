"""Multi-stage context pruning (Alg. 1) and the per-layer sequence on top of
the C leaf routines of ihip_oracle.c.  TEST INFRASTRUCTURE ONLY (see the
package docstring).

One "problem" is (sequence b, KV head g, query block m).  Reading of the
paper used here: the mask is chosen per KV head, the chunk score being pooled
over the query heads that share it (the paper writes H heads and never
mentions grouped-query attention).
"""
from __future__ import annotations

import ctypes
import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch


def _u16(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> contiguous uint16 numpy array of its bit patterns."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class StageResult:
    l_c: int
    starts: np.ndarray          # int64 [n]   chunk start positions, ascending
    lens: np.ndarray            # int32 [n]   valid lengths (1..l_c)
    scores: np.ndarray          # float32 [n] chunk scores
    reps: np.ndarray            # int64 [G,n] representative positions
    kept_ids: np.ndarray        # int32 [kept] ascending chunk ids
    touched_pos: np.ndarray     # int64, ascending: distinct K rows (positions) scored by this stage

    @property
    def rows_touched(self) -> int:
        return len(self.touched_pos)

    @property
    def kept_starts(self):
        return self.starts[self.kept_ids]

    @property
    def kept_lens(self):
        return self.lens[self.kept_ids]


@dataclass
class ProblemResult:
    b: int
    g: int
    m: int
    lo: int                     # first middle position  (= n_sink)
    hi: int                     # one past the last middle position (= E - n_stream)
    E: int                      # one past the last key visible to the block
    stages: List[StageResult] = field(default_factory=list)

    @property
    def block_starts(self) -> np.ndarray:
        return self.stages[-1].kept_starts if self.stages else np.zeros(0, np.int64)

    @property
    def block_lens(self) -> np.ndarray:
        return self.stages[-1].kept_lens if self.stages else np.zeros(0, np.int32)


@dataclass
class RopeSpec:
    """Dynamic RoPE (Sec. 4 "Dynamic RoPE for OOL generalization").  cos / sin:
    float32 [n_pos, d/2], cos and sin of (position x frequency j's angle);
    prune: None, "relative" or "chunk"; attn: None or "streaming"."""
    cos: np.ndarray
    sin: np.ndarray
    prune: Optional[str] = None
    attn: Optional[str] = None


def stage1_chunks(lo: int, hi: int, l_c: int):
    """Alg. 1 step 1 + Alg. 2 chunking: the middle range [lo, hi) cut into
    l_c-sized chunks, the last one cut short if the range is ragged."""
    starts = np.arange(lo, hi, l_c, dtype=np.int64)
    lens = np.minimum(l_c, hi - starts).astype(np.int32)
    return starts, lens


def child_chunks(kept_starts, kept_lens, l_child: int):
    """The next stage's chunks: the kept tokens, in position order, cut into
    l_child-sized pieces.  Every kept chunk is a multiple of l_child long except
    a ragged last one, so the pieces never straddle two parents; empty pieces
    are dropped."""
    starts, lens = [], []
    for s, n in zip(kept_starts.tolist(), kept_lens.tolist()):
        for c in range(0, n, l_child):
            starts.append(s + c)
            lens.append(min(l_child, n - c))
    return np.asarray(starts, dtype=np.int64), np.asarray(lens, dtype=np.int32)


class Oracle:
    """Holds one layer's Q/K/V (as bf16 bit patterns on the host) and the
    shape; runs pruning and attention problem by problem."""

    def __init__(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, seq_lens,
                 b_q: int, n_sink: int, n_stream: int, rope: Optional[RopeSpec] = None,
                 kv_scales: Optional[Tuple[float, float]] = None, stage_b_q: Optional[Sequence[int]] = None):
        """kv_scales = (k_scale, v_scale): K and V are uint8 tensors of E4M3 bytes (FP8 KV cache),
        an element being its scale times the decoded byte; otherwise they are bf16.

        stage_b_q: query-block size of every pruning stage (Sec. 4, the m' rule after Eq. for
        I^(i); Alg. 1: a stage's result for block m is handed to the finer blocks of the next stage
        that lie inside it).  Non-increasing, each dividing the one before, the last equal to b_q
        (the block size of the attention).  Alg. 1 step 1 defines the candidate range with the first
        stage's block, so the middle range of every finer block ends at that coarse block's end
        minus n_stream; a finer block's own window then runs from there to its own queries."""
        from . import lib, Tensors, Rope
        self.L = lib()
        self.rope = rope
        if rope is not None:
            self._cos = np.ascontiguousarray(rope.cos, np.float32)
            self._sin = np.ascontiguousarray(rope.sin, np.float32)
            assert self._cos.shape == self._sin.shape and self._cos.shape[1] * 2 == q.shape[-1]
            self._rope = Rope(self._cos.ctypes.data, self._sin.ctypes.data, self._cos.shape[0])
        if kv_scales is None:
            self.q, self.k, self.v = _u16(q), _u16(k), _u16(v)
        else:
            assert k.dtype == torch.uint8 and v.dtype == torch.uint8
            self.q = _u16(q)
            self.k, self.v = k.detach().cpu().contiguous().numpy(), v.detach().cpu().contiguous().numpy()
        self.B, self.Hq, self.Tq, self.d = q.shape
        _, self.Hkv, self.T_alloc, _ = k.shape
        assert self.Hq % self.Hkv == 0 and self.Tq % b_q == 0
        self.G = self.Hq // self.Hkv
        self.seq_lens = [int(x) for x in seq_lens]
        self.b_q, self.n_sink, self.n_stream = b_q, n_sink, n_stream
        self.stage_b_q = None if stage_b_q is None else [int(x) for x in stage_b_q]
        if self.stage_b_q is not None:
            sb = self.stage_b_q
            assert sb[-1] == b_q and all(sb[i] % sb[i + 1] == 0 for i in range(len(sb) - 1))
            assert self.Tq % sb[0] == 0 and n_stream >= sb[0]
        self.t = Tensors(self.q.ctypes.data, self.k.ctypes.data, self.v.ctypes.data,
                         self.B, self.Hq, self.Hkv, self.d, self.Tq, self.T_alloc,
                         0 if kv_scales is None else 1,
                         1.0 if kv_scales is None else kv_scales[0], 1.0 if kv_scales is None else kv_scales[1])

    # -- geometry ---------------------------------------------------------
    def ranges(self, b: int, m: int) -> Tuple[int, int, int]:
        """(lo, hi, E): middle range [lo, hi) and exclusive end E of the keys
        visible to query block m (Alg. 1 step 1: sink and streaming tokens are
        excluded, causality is kept because hi never exceeds the position of
        the block's first query)."""
        E = (self.seq_lens[b] - self.Tq) + (m + 1) * self.b_q
        if self.stage_b_q is None:
            return self.n_sink, E - self.n_stream, E
        first = self.stage_b_q[0]                       # the block that defines the candidate range
        E_first = (self.seq_lens[b] - self.Tq) + (m * self.b_q // first + 1) * first
        return self.n_sink, E_first - self.n_stream, E

    def stage_queries(self, b: int, m: int, i: Optional[int]) -> Tuple[int, int, int]:
        """(first query row, number of queries, position of the first query) of the block of
        stage i that holds block m of the last stage (the block itself without stage_b_q)."""
        nq = self.b_q if self.stage_b_q is None or i is None else self.stage_b_q[i]
        q0 = (m * self.b_q // nq) * nq
        return q0, nq, (self.seq_lens[b] - self.Tq) + q0

    # -- Alg. 2 -----------------------------------------------------------
    def prune_stage(self, b, g, m, starts, lens, l_c, keep, exhaustive=False, stage=None) -> StageResult:
        n = len(starts)
        q0, nq, qpos0 = self.stage_queries(b, m, stage)
        scores = np.empty(n, np.float32)
        reps = np.empty((self.G, n), np.int64)
        touched = np.zeros(self.T_alloc, np.uint8)
        starts = np.ascontiguousarray(starts, np.int64)
        lens = np.ascontiguousarray(lens, np.int32)
        if self.rope is not None and self.rope.prune is not None:
            assert not exhaustive
            style = {"relative": 1, "chunk": 2}[self.rope.prune]
            need = self.n_stream + 2 if style == 1 else n + self.n_stream
            assert self._cos.shape[0] >= need, "RoPE table too short"
            self.L.orc_prune_stage_rope(ctypes.byref(self.t), b, g, q0, nq, qpos0, n,
                                        _p(starts), _p(lens), l_c, ctypes.byref(self._rope), style,
                                        self.n_stream, _p(scores), _p(reps), _p(touched))
        else:
            self.L.orc_prune_stage(ctypes.byref(self.t), b, g, q0, nq, n,
                                   _p(starts), _p(lens), l_c, int(exhaustive),
                                   _p(scores), _p(reps), _p(touched))
        ids = np.empty(max(min(keep, n), 1), np.int32)
        kept = self.L.orc_topk(n, _p(scores), keep, _p(ids))
        return StageResult(l_c, starts, lens, scores, reps, ids[:kept].copy(), np.nonzero(touched)[0].astype(np.int64))

    # -- Alg. 1 -----------------------------------------------------------
    def prune(self, b, g, m, stages: Sequence[Tuple[int, int]], exhaustive=False) -> ProblemResult:
        """stages: (chunk size l_c, chunks kept K) per stage, coarse to fine."""
        lo, hi, E = self.ranges(b, m)
        pr = ProblemResult(b, g, m, lo, hi, E)
        if hi <= lo:
            return pr                       # nothing between sink and window
        starts, lens = stage1_chunks(lo, hi, stages[0][0])
        for i, (l_c, keep) in enumerate(stages):
            assert l_c & (l_c - 1) == 0, "chunk sizes are powers of two"
            if i > 0:
                assert stages[i - 1][0] % l_c == 0
                starts, lens = child_chunks(pr.stages[-1].kept_starts, pr.stages[-1].kept_lens, l_c)
            pr.stages.append(self.prune_stage(b, g, m, starts, lens, l_c, keep, exhaustive, stage=i))
        return pr

    # -- Alg. 2 as printed: one mask per layer ---------------------------------
    def prune_all_heads(self, b, m, stages: Sequence[Tuple[int, int]]) -> List[ProblemResult]:
        """The paper's own pooling (Sec. 4: the chunk score is max-pooled over all
        H attention heads, Alg. 2 `max_{h=1..H, t}`): every stage scores the chunks
        per KV group as usual, the group scores are max-pooled and one arg-top-K
        decides the chunks kept for all heads.  Returns one ProblemResult per KV
        head (scores = the pooled ones, representatives its own heads')."""
        lo, hi, E = self.ranges(b, m)
        prs = [ProblemResult(b, g, m, lo, hi, E) for g in range(self.Hkv)]
        if hi <= lo:
            return prs
        starts, lens = stage1_chunks(lo, hi, stages[0][0])
        for i, (l_c, keep) in enumerate(stages):
            if i > 0:
                starts, lens = child_chunks(prs[0].stages[-1].kept_starts, prs[0].stages[-1].kept_lens, l_c)
            per_g = [self.prune_stage(b, g, m, starts, lens, l_c, keep, stage=i) for g in range(self.Hkv)]
            pooled = np.max(np.stack([r.scores for r in per_g]), axis=0) if len(starts) else np.zeros(0, np.float32)
            pooled = np.ascontiguousarray(pooled, np.float32)
            ids = np.empty(max(min(keep, len(starts)), 1), np.int32)
            kept = self.L.orc_topk(len(starts), _p(pooled), keep, _p(ids))
            for g in range(self.Hkv):
                r = per_g[g]
                prs[g].stages.append(StageResult(l_c, r.starts, r.lens, pooled, r.reps, ids[:kept].copy(), r.touched_pos))
        return prs

    # -- Alg. 4: cached masks ------------------------------------------------
    def prune_from(self, b, g, m, stages, first_stage, cached_kept):
        """Mask caching (Sec. 4 "Sparse Attention Mask Caching", Alg. 4): stages
        first_stage.. are re-run with the current queries, the earlier ones keep
        the index lists cached from an earlier step.  cached_kept: per stage, the
        kept chunk starts (int64 arrays) of that earlier step.  Returns the per
        stage kept starts after this step and the final blocks (starts, lens).
        Lengths always follow the current end of the middle range."""
        return self.prune_due(b, g, m, stages, [i >= first_stage for i in range(len(stages))], cached_kept)

    def prune_due(self, b, g, m, stages, due, cached_kept):
        """One decode step of Alg. 4's stage loop for one problem: stage i is re-run
        (with the current queries, on the list stage i-1 holds at this moment, be it
        re-run in this step or cached) iff due[i]; a stage that is not due keeps
        its cached list, also when an earlier stage was re-run.  Returns as
        prune_from."""
        lo, hi, E = self.ranges(b, m)
        kept = [np.asarray(x, np.int64) for x in cached_kept]
        if hi <= lo:
            return [np.zeros(0, np.int64) for _ in stages], np.zeros(0, np.int64), np.zeros(0, np.int32)
        for i, (l_c, keep) in enumerate(stages):
            if not due[i]:
                continue
            if i == 0:
                starts, lens = stage1_chunks(lo, hi, l_c)
            else:
                ps = kept[i - 1]
                plens = np.minimum(stages[i - 1][0], hi - ps).astype(np.int32)
                starts, lens = child_chunks(ps, plens, l_c)
            kept[i] = self.prune_stage(b, g, m, starts, lens, l_c, keep).kept_starts
        bs = kept[-1]
        return kept, bs, np.minimum(stages[-1][0], hi - bs).astype(np.int32)

    # -- block-sparse attention --------------------------------------------
    def attend(self, b, g, m, block_starts, block_lens, scale=None):
        """fp64 output [G, b_q, d] and log-sum-exp [G, b_q] of the block's
        queries over sink + kept blocks + causal window."""
        lo, hi, E = self.ranges(b, m)
        scale = 1.0 / math.sqrt(self.d) if scale is None else scale
        out = np.empty((self.G, self.b_q, self.d), np.float64)
        lse = np.empty((self.G, self.b_q), np.float64)
        bs = np.ascontiguousarray(block_starts, np.int64)
        bl = np.ascontiguousarray(block_lens, np.int32)
        if len(bs):
            assert bs.min() >= lo and (bs + bl).max() <= hi
        if self.rope is not None and self.rope.attn is not None:
            assert self.rope.attn == "streaming"
            assert self._cos.shape[0] >= self.attended_tokens(b, m, bl), "RoPE table too short"
            self.L.orc_sparse_attention_rope(ctypes.byref(self.t), b, g, m * self.b_q, self.b_q,
                                             E - self.b_q, self.n_sink, max(hi, self.n_sink),
                                             len(bs), _p(bs), _p(bl), scale, ctypes.byref(self._rope),
                                             _p(out), _p(lse))
        else:
            self.L.orc_sparse_attention(ctypes.byref(self.t), b, g, m * self.b_q, self.b_q,
                                        E - self.b_q, self.n_sink, max(hi, self.n_sink),
                                        len(bs), _p(bs), _p(bl), scale, _p(out), _p(lse))
        return out, lse

    def attended_positions(self, b, m, block_starts, block_lens) -> np.ndarray:
        """Every key position the block's attention reads (last query's view)."""
        lo, hi, E = self.ranges(b, m)
        parts = [np.arange(0, min(self.n_sink, E))]
        parts += [np.arange(s, s + n) for s, n in zip(block_starts.tolist(), block_lens.tolist())]
        parts.append(np.arange(max(hi, self.n_sink), E))
        return np.concatenate(parts).astype(np.int64)

    def attended_tokens(self, b, m, block_lens) -> int:
        """Keys the last query of the block attends to (for byte counts)."""
        lo, hi, E = self.ranges(b, m)
        return min(self.n_sink, E) + int(np.sum(block_lens)) + max(0, E - max(hi, self.n_sink))

    # -- one layer ----------------------------------------------------------
    def layer(self, stages, scale=None, problems=None, exhaustive=False):
        """Pruning + attention for every (b, g, m) (or the listed ones).
        Returns {(b,g,m): (ProblemResult, out[G,b_q,d], lse[G,b_q])}."""
        if problems is None:
            problems = [(b, g, m) for b in range(self.B) for g in range(self.Hkv)
                        for m in range(self.Tq // self.b_q)]
        res = {}
        for (b, g, m) in problems:
            pr = self.prune(b, g, m, stages, exhaustive)
            out, lse = self.attend(b, g, m, pr.block_starts, pr.block_lens, scale)
            res[(b, g, m)] = (pr, out, lse)
        return res
