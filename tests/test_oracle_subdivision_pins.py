"""Pins of the oracle's per-stage query blocks (Sec. 4, the m' rule; Alg. 1: a
stage's result for block m is handed to the finer blocks of the next stage
inside it) against what the algorithm fixes, none of it through the oracle's
own code: brute force with a perfect in-chunk search where every stage scores
with its own block's queries, reduction to the single-block-size path, shared
coarse results between sibling blocks, the shortened window of the earlier
siblings, and dense causal attention when nothing is pruned."""
import math

import numpy as np
import pytest
import torch

from oracle import Oracle
from test_oracle_pins import all_scores, final_tokens, make

pytestmark = pytest.mark.usefixtures("oracle_lib")


def brute_force_subdivided(q, k, b, g, G, m, T, Tq, n_sink, n_stream, stages, stage_b_q):
    """Alg. 1 for block m of the last stage, every stage with a perfect search: the candidate range
    ends n_stream before the end of the first stage's block holding m; stage i scores chunks with
    the queries of its own block holding m; top K by (score desc, index asc)."""
    fine = stage_b_q[-1]
    first = stage_b_q[0]
    hi = (T - Tq) + (m * fine // first + 1) * first - n_stream
    idx = np.arange(n_sink, max(hi, n_sink))
    for (l_c, keep), bq in zip(stages, stage_b_q):
        q0 = (m * fine // bq) * bq
        S = all_scores(q, k, b, g, G, q0, bq)
        n = math.ceil(len(idx) / l_c)
        chunks = [idx[j * l_c:(j + 1) * l_c] for j in range(n)]
        sc = np.array([S[:, c].max() for c in chunks])
        order = np.lexsort((np.arange(n), -sc))[:min(keep, n)]
        idx = np.concatenate([chunks[j] for j in sorted(order)]) if len(order) else idx[:0]
    return idx


@pytest.mark.parametrize("kind", ["int", "normal"])
@pytest.mark.parametrize("stage_b_q,stages", [((8, 4), ((16, 5), (4, 7))), ((8, 4, 2), ((32, 4), (8, 6), (2, 9))),
                                               ((4, 4, 2), ((16, 6), (4, 8), (2, 10))), ((8, 2), ((8, 9), (2, 11)))])
def test_exhaustive_search_equals_brute_force_with_each_stages_own_queries(kind, stage_b_q, stages):
    T, Tq, n_sink, n_stream = 4 + 300 + 16, 16, 4, 12
    q, k, v = make(T=T, Tq=Tq, d=32, seed=7, kind=kind)
    # the last key of every coarse block's candidate range is made the best one for all of that
    # block's queries, so every finer block inside must keep it: a range that ended with the finer
    # block instead would lose it
    k = k.clone()
    last = []
    for mc in range(Tq // stage_b_q[0]):
        pos = (T - Tq) + (mc + 1) * stage_b_q[0] - n_stream - 1
        qs = q[0, :, mc * stage_b_q[0]:(mc + 1) * stage_b_q[0]].float()
        k[0, :, pos] = (8.0 * torch.sign(qs.sum(dim=(0, 1)))).to(torch.bfloat16)
        last.append(pos)
    o = Oracle(q, k, v, [T], stage_b_q[-1], n_sink, n_stream, stage_b_q=stage_b_q)
    planted_kept = 0
    for g in range(2):
        for m in range(Tq // stage_b_q[-1]):
            pe = o.prune(0, g, m, stages, exhaustive=True)
            want = brute_force_subdivided(q, k, 0, g, 2, m, T, Tq, n_sink, n_stream, stages, stage_b_q)
            assert final_tokens(pe).tolist() == want.tolist(), (g, m)
            planted_kept += last[m * stage_b_q[-1] // stage_b_q[0]] in want.tolist()
    assert planted_kept >= Tq // stage_b_q[-1]           # the planted keys do decide something


def test_equal_block_sizes_reduce_to_the_plain_path():
    T, Tq = 4 + 400 + 16, 16
    q, k, v = make(T=T, Tq=Tq, d=32, seed=3)
    stages = ((32, 4), (8, 6), (2, 9))
    a = Oracle(q, k, v, [T], 4, 4, 12)
    b = Oracle(q, k, v, [T], 4, 4, 12, stage_b_q=(4, 4, 4))
    for g in range(2):
        for m in range(Tq // 4):
            pa, pb = a.prune(0, g, m, stages), b.prune(0, g, m, stages)
            assert a.ranges(0, m) == b.ranges(0, m)
            for sa, sb in zip(pa.stages, pb.stages):
                assert np.array_equal(sa.scores, sb.scores) and np.array_equal(sa.reps, sb.reps)
                assert np.array_equal(sa.kept_starts, sb.kept_starts)
            oa, la = a.attend(0, g, m, pa.block_starts, pa.block_lens)
            ob, lb = b.attend(0, g, m, pb.block_starts, pb.block_lens)
            assert np.array_equal(oa, ob) and np.array_equal(la, lb)


def test_sibling_blocks_share_the_coarse_stage_and_differ_after_it():
    T, Tq, n_sink, n_stream = 4 + 500 + 16, 16, 4, 16
    q, k, v = make(T=T, Tq=Tq, d=32, seed=11)
    stages = ((16, 6), (4, 8))
    o = Oracle(q, k, v, [T], 4, n_sink, n_stream, stage_b_q=(8, 4))
    plain = Oracle(q, k, v, [T], 4, n_sink, n_stream)
    differ_fine = differ_plain = 0
    for g in range(2):
        for mc in range(Tq // 8):
            p0, p1 = o.prune(0, g, 2 * mc, stages), o.prune(0, g, 2 * mc + 1, stages)
            # one coarse block, one first-stage result: same candidates, scores and survivors
            assert (p0.lo, p0.hi) == (p1.lo, p1.hi)
            assert p0.hi == (T - Tq) + (mc + 1) * 8 - n_stream
            assert np.array_equal(p0.stages[0].scores, p1.stages[0].scores)
            assert np.array_equal(p0.stages[0].kept_starts, p1.stages[0].kept_starts)
            # the second stage scores the same chunks with each sibling's own queries
            assert np.array_equal(p0.stages[1].starts, p1.stages[1].starts)
            differ_fine += not np.array_equal(p0.stages[1].scores, p1.stages[1].scores)
            q0, q1 = plain.prune(0, g, 2 * mc, stages), plain.prune(0, g, 2 * mc + 1, stages)
            differ_plain += not np.array_equal(q0.stages[0].scores[:4], q1.stages[0].scores[:4])
            # the earlier sibling's window is shorter by the queries that follow it in the coarse block
            assert o.attended_tokens(0, 2 * mc + 1, p1.block_lens) - int(p1.block_lens.sum()) == n_sink + n_stream
            assert o.attended_tokens(0, 2 * mc, p0.block_lens) - int(p0.block_lens.sum()) == n_sink + n_stream - 4
    assert differ_fine > 0 and differ_plain > 0          # the option changes something on random data


@pytest.mark.parametrize("stage_b_q", [(8, 4), (16, 4, 2)])
def test_keep_everything_is_dense_causal_attention(stage_b_q):
    # sink + all of the coarse block's middle range + the window from there to the query = every
    # key up to the query, for every block of the last stage
    T, Tq, n_sink, n_stream, d = 4 + 200 + 16, 16, 4, 16, 32
    q, k, v = make(T=T, Tq=Tq, d=d, seed=5)
    stages = tuple((c, 10 ** 6) for c in (16, 4, 2)[:len(stage_b_q)])
    fine = stage_b_q[-1]
    o = Oracle(q, k, v, [T], fine, n_sink, n_stream, stage_b_q=stage_b_q)
    mask = torch.arange(T).view(1, -1) <= torch.arange(T - Tq, T).view(-1, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(2, 1), v.double().repeat_interleave(2, 1), attn_mask=mask)
    for g in range(2):
        for m in range(Tq // fine):
            pr = o.prune(0, g, m, stages)
            out, _ = o.attend(0, g, m, pr.block_starts, pr.block_lens)
            want = ref[0, g * 2:(g + 1) * 2, m * fine:(m + 1) * fine].numpy()
            assert np.abs(out - want).max() <= 1e-9
