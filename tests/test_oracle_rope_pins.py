"""Pins of the oracle's dynamic-RoPE routines (Sec. 4 "Dynamic RoPE for OOL
generalization"; ApplyRopeQ / ApplyRopeK after Alg. 3) against things that do
not come from the oracle: hand-worked examples on quarter-turn tables,
rotation identities, the RoPE-free routines under an identity table, and an
independent complex-number implementation of rotary attention in torch."""
import ctypes
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import Oracle, RopeSpec
from workloads import gen


def vec(pairs, d=128):
    """bf16 row with the given (dim, value) entries."""
    x = torch.zeros(d)
    for c, v in pairs:
        x[c] = v
    return x.to(torch.bfloat16)


def make(q_rows, k_rows, n_sink=0, n_stream=1, rope=None, v_rows=None, b_q=1):
    """One sequence, one head: q [Tq rows], k [T rows]."""
    q = torch.stack(q_rows).view(1, 1, len(q_rows), -1)
    k = torch.stack(k_rows).view(1, 1, len(k_rows), -1)
    v = k.clone() if v_rows is None else torch.stack(v_rows).view(1, 1, len(v_rows), -1)
    return Oracle(q, k, v, [k.shape[2]], b_q, n_sink, n_stream, rope=rope)


def score(o, p, qpos, kpos):
    qp = np.asarray(qpos, np.int64)
    return o.L.orc_score_rope(ctypes.byref(o.t), 0, 0, 0, len(qp), p, ctypes.byref(o._rope),
                              qp.ctypes.data_as(ctypes.c_void_p), kpos)


def test_pair_layout_and_direction_on_quarter_turns():
    # Su et al.: dims (2j, 2j+1) are one pair; frequency 0 of the quarter-turn table turns 90 degrees
    # per position.  q = e0 at position a, k = e0 at position b: q~ . k~ = cos((a - b) * 90 deg).
    cos, sin = gen.quarter_turn_table(8, 128)
    o = make([vec([(0, 1.0)])], [vec([(0, 1.0)]), vec([(1, 1.0)])], rope=RopeSpec(cos.numpy(), sin.numpy()))
    assert [score(o, 0, [a], 0) for a in range(4)] == [1.0, 0.0, -1.0, 0.0]
    assert [score(o, 0, [3], b) for b in range(4)] == [0.0, -1.0, 0.0, 1.0]
    # q = e0 turned by one position is e1 (counter-clockwise); a layout pairing dims (0, 64) would give 0
    assert score(o, 1, [1], 0) == 1.0
    assert score(o, 1, [3], 0) == -1.0
    # frequency 1 (dims 2, 3) turns two quarters per position
    o2 = make([vec([(2, 1.0)])], [vec([(2, 1.0)])], rope=RopeSpec(cos.numpy(), sin.numpy()))
    assert [score(o2, 0, [a], 0) for a in range(4)] == [1.0, -1.0, 1.0, -1.0]


def test_rotation_identities_on_a_real_table():
    cos, sin = gen.rope_table(64, 128)
    torch.manual_seed(0)
    q = torch.randn(128).to(torch.bfloat16)
    k = torch.randn(128).to(torch.bfloat16)
    o = make([q], [k, q], rope=RopeSpec(cos.numpy(), sin.numpy()))
    plain = float((q.double() * k.double()).sum())
    # same position on both sides leaves the product unchanged; so does position 0
    for a in (0, 1, 17, 63):
        assert score(o, 0, [a], a) == pytest.approx(plain, rel=1e-5, abs=1e-4)
    # only the difference of the positions matters
    for a, b in ((5, 2), (40, 37), (63, 60)):
        assert score(o, 0, [a], b) == pytest.approx(score(o, 0, [3], 0), rel=1e-5, abs=1e-4)
    # norm is preserved: the key q (row 1) against the query q at equal positions
    assert score(o, 1, [9], 9) == pytest.approx(float((q.double() ** 2).sum()), rel=1e-5)
    # and it matches e^{i theta} multiplication of the (even, odd) pairs
    ang = 7 * 10000.0 ** (-2.0 * np.arange(64) / 128)
    qc = (q.double().numpy()[0::2] + 1j * q.double().numpy()[1::2]) * np.exp(1j * ang)
    kc = k.double().numpy()[0::2] + 1j * k.double().numpy()[1::2]
    assert score(o, 0, [7], 0) == pytest.approx(float((qc * kc.conj()).real.sum()), rel=1e-5, abs=1e-4)


def test_relative_style_worked_example():
    # One pair in use, quarter turns, n_stream = 1: the query e0 sits at position 2, i.e. q~ = -e0.
    # A left-branch key (x, y) stays (x, y): score -x.  A right-branch key is turned by 90 degrees to
    # (-y, x): score y.  Chunk of 4 keys K0..K3:
    #   iteration 1: K0 = (-1, 0) as left scores 1, K2 = (0, 3) as right scores 3  -> right half
    #   iteration 2: K2 as left scores -0 = 0 (not the 3 it had as a right key), K3 = (5, 1) as right
    #                scores 1 -> right: representative = 3 (a carried score would have kept K2)
    #   chunk score: K3 as branch 2: 1
    cos, sin = gen.quarter_turn_table(8, 128)
    keys = [vec([(0, -1.0)]), vec([(0, 9.0), (1, 9.0)]), vec([(1, 3.0)]), vec([(0, 5.0), (1, 1.0)])]
    k_rows = keys + [vec([])]                     # one streaming token behind the chunk
    o = make([vec([(0, 1.0)])], k_rows, n_sink=0, n_stream=1,
             rope=RopeSpec(cos.numpy(), sin.numpy(), prune="relative"))
    st = o.prune_stage(0, 0, 0, np.array([0]), np.array([4], np.int32), 4, 1)
    assert st.reps[0, 0] == 3 and st.scores[0] == 1.0
    # K1 is never looked at: the first key of each half only
    assert st.touched_pos.tolist() == [0, 2, 3]
    # without RoPE the same data gives scores x: -1 vs 0 -> right, 0 vs 5 -> right, score 5
    o0 = make([vec([(0, 1.0)])], k_rows, n_sink=0, n_stream=1)
    st0 = o0.prune_stage(0, 0, 0, np.array([0]), np.array([4], np.int32), 4, 1)
    assert st0.reps[0, 0] == 3 and st0.scores[0] == 5.0


@pytest.mark.parametrize("T,expect", [(5, [1.0, 0.0, -1.0, 0.0]), (3, [-1.0, 0.0, 1.0, 0.0])])
def test_chunk_indexed_worked_example(T, expect):
    # Four one-key chunks, every key e0, the query e0.  Chunk j sits at position j, the query at
    # min(original position, (n_chunk - 1) + n_stream): the score is cos((qpos - j) * 90 deg).
    #   T = 5: original position 4 = cap 4 -> offsets 4, 3, 2, 1;  T = 3: original position 2 -> 2, 1, 0, -1
    cos, sin = gen.quarter_turn_table(8, 128)
    k_rows = [vec([(0, 1.0)]) for _ in range(5)]
    o = make([vec([(0, 1.0)])], k_rows, n_sink=0, n_stream=1,
             rope=RopeSpec(cos.numpy(), sin.numpy(), prune="chunk"))
    o.seq_lens = [T]
    st = o.prune_stage(0, 0, 0, np.arange(4), np.ones(4, np.int32), 1, 4)
    assert st.scores.tolist() == expect


def test_identity_table_reduces_to_the_plain_routines():
    torch.manual_seed(1)
    B, Hq, Hkv, T, d = 1, 4, 2, 700, 128
    q = torch.randn(B, Hq, 1, d).to(torch.bfloat16)
    k = torch.randn(B, Hkv, T, d).to(torch.bfloat16)
    v = torch.randn(B, Hkv, T, d).to(torch.bfloat16)
    ones, zeros = np.ones((T + 8, d // 2), np.float32), np.zeros((T + 8, d // 2), np.float32)
    stages = [(32, 6), (8, 10), (2, 24)]
    plain = Oracle(q, k, v, [T], 1, 16, 64)
    for prune in ("relative", "chunk"):
        r = Oracle(q, k, v, [T], 1, 16, 64, rope=RopeSpec(ones, zeros, prune=prune, attn="streaming"))
        for g in range(Hkv):
            a, b = plain.prune(0, g, 0, stages), r.prune(0, g, 0, stages)
            for sa, sb in zip(a.stages, b.stages):
                assert np.array_equal(sa.scores, sb.scores) and np.array_equal(sa.reps, sb.reps)
                assert np.array_equal(sa.kept_ids, sb.kept_ids)
            oa, la = plain.attend(0, g, 0, a.block_starts, a.block_lens)
            ob, lb = r.attend(0, g, 0, b.block_starts, b.block_lens)
            assert np.array_equal(oa, ob) and np.array_equal(la, lb)


def test_streaming_style_equals_rotary_attention_when_everything_is_kept():
    # All keys kept: sequential ids are the true positions, so the result is ordinary rotary
    # attention -- computed here with complex multiplication in torch, fp64.
    torch.manual_seed(2)
    B, Hq, Hkv, T, d = 1, 4, 2, 300, 128
    q = torch.randn(B, Hq, 1, d).to(torch.bfloat16)
    k = torch.randn(B, Hkv, T, d).to(torch.bfloat16)
    v = torch.randn(B, Hkv, T, d).to(torch.bfloat16)
    cos, sin = gen.rope_table(T, d)
    o = Oracle(q, k, v, [T], 1, 8, 32, rope=RopeSpec(cos.numpy(), sin.numpy(), attn="streaming"))
    ang = torch.arange(T, dtype=torch.float64).view(-1, 1) * 10000.0 ** (-2.0 * torch.arange(d // 2, dtype=torch.float64) / d)
    rot = torch.polar(torch.ones_like(ang), ang)                          # [T, d/2]
    kc = torch.view_as_complex(k.double().view(B, Hkv, T, d // 2, 2).contiguous()) * rot
    qc = torch.view_as_complex(q.double().view(B, Hq, 1, d // 2, 2).contiguous()) * rot[T - 1]
    G = Hq // Hkv
    for g in range(Hkv):
        blocks = np.arange(8, T - 32, 4, dtype=np.int64)
        lens = np.minimum(4, T - 32 - blocks).astype(np.int32)
        out, lse = o.attend(0, g, 0, blocks, lens)
        for hh in range(G):
            logits = (qc[0, g * G + hh, 0] * kc[0, g].conj()).real.sum(-1) / math.sqrt(d)
            w = torch.softmax(logits, 0)
            ref = (w.view(-1, 1) * v[0, g].double()).sum(0)
            assert np.abs(out[hh, 0] - ref.numpy()).max() < 1e-6
            assert lse[hh, 0] == pytest.approx(float(torch.logsumexp(logits, 0)), abs=1e-6)


def test_streaming_ids_count_only_attended_keys():
    # Keys that are not attended do not advance the ids: two key sets with the same attended rows in
    # the same order, separated by different numbers of skipped rows, give the same output.
    torch.manual_seed(3)
    d = 128
    rows = [torch.randn(d).to(torch.bfloat16) for _ in range(12)]
    filler = [torch.randn(d).to(torch.bfloat16) for _ in range(8)]
    cos, sin = gen.rope_table(64, d)
    q = torch.randn(d).to(torch.bfloat16)
    # layout A: [sink 2][block 4][4 skipped][block 4][window 2]; layout B: 8 skipped rows instead of 4
    def run(skip):
        k_rows = rows[0:2] + rows[2:6] + filler[:skip] + rows[6:10] + rows[10:12]
        o = make([q], k_rows, n_sink=2, n_stream=2, rope=RopeSpec(cos.numpy(), sin.numpy(), attn="streaming"))
        return o.attend(0, 0, 0, np.array([2, 6 + skip]), np.array([4, 4], np.int32))
    (oa, la), (ob, lb) = run(4), run(8)
    assert np.array_equal(oa, ob) and np.array_equal(la, lb)
