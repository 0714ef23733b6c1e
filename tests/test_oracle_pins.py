"""Pins of the CPU oracle against what the paper and the mathematics fix.

The paper prints no worked numeric example of Alg. 1-3, so the oracle is
pinned by: exactness on integer data, reduction to dense attention (library
SDPA) when nothing is pruned, equality with brute force where the search is
provably exact, an independent literal re-implementation of Alg. 3 in its
printed 1-based form, structural invariants, needle retention, and library
sort / softmax routines.
"""
import math

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from oracle import Oracle
from oracle.pipeline import stage1_chunks, child_chunks
from workloads import configs, gen

pytestmark = pytest.mark.usefixtures("oracle_lib")


# --------------------------------------------------------------------------
# helpers independent of the oracle
# --------------------------------------------------------------------------
def f64(t):
    return t.to(torch.float64).numpy()


def make(B=1, Hq=4, Hkv=2, T=300, Tq=1, d=16, seed=0, kind="normal"):
    q = (gen.normal_bf16 if kind == "normal" else gen.small_int_bf16)(seed, 1, (B, Hq, Tq, d))
    k = (gen.normal_bf16 if kind == "normal" else gen.small_int_bf16)(seed, 2, (B, Hkv, T, d))
    v = (gen.normal_bf16 if kind == "normal" else gen.small_int_bf16)(seed, 3, (B, Hkv, T, d))
    return q, k, v


def all_scores(q, k, b, g, G, q0, bq):
    """S[hh, p] = max_t q_{g*G+hh, q0+t} . k_p  in float64 (exact for bf16 data
    up to fp64 rounding; exact outright for small-integer data)."""
    qq = f64(q[b, g * G:(g + 1) * G, q0:q0 + bq])          # [G,bq,d]
    kk = f64(k[b, g])                                       # [T,d]
    return np.einsum("gtd,pd->gtp", qq, kk).max(axis=1)     # [G,T]


def brute_force_prune(S, lo, hi, stages):
    """Paper-literal pruning with a perfect in-chunk search: the index list is
    cut into l_c-long pieces *of the list* (Sec. 4, definition of C_{m,j}), a
    chunk's score is the true maximum over heads and positions, the top K by
    (score desc, index asc) survive, and their union in position order is the
    next list."""
    idx = np.arange(lo, hi)
    for l_c, keep in stages:
        n = math.ceil(len(idx) / l_c)
        chunks = [idx[j * l_c:(j + 1) * l_c] for j in range(n)]
        sc = np.array([S[:, c].max() for c in chunks])
        order = np.lexsort((np.arange(n), -sc))[:min(keep, n)]
        idx = np.concatenate([chunks[j] for j in sorted(order)]) if len(order) else idx[:0]
    return idx


def final_tokens(pr):
    out = []
    for s, n in zip(pr.block_starts.tolist(), pr.block_lens.tolist()):
        out.extend(range(s, s + n))
    return np.asarray(out, dtype=np.int64)


def literal_select_rep(score_of, chunk):
    """Alg. 3 as printed, 1-based: both branch scores are computed in every
    iteration; the midpoint (first+last)/2 is rounded half up; arg-max ties go
    to branch 1; the result is the first index of the final range."""
    l_c = len(chunk)
    n_iter = math.ceil(math.log2(l_c)) if l_c > 1 else 0
    first, last = 1, l_c
    for _ in range(n_iter):
        mid = (first + last + 1) // 2                       # round half up
        b1, b2 = (first, mid - 1), (mid, last)
        s1 = score_of(chunk[b1[0] - 1])
        s2 = score_of(chunk[b2[0] - 1])
        first, last = b2 if s2 > s1 else b1
    return chunk[first - 1]


# --------------------------------------------------------------------------
# 1. scores are exact on integer data
# --------------------------------------------------------------------------
def test_score_exact_on_integer_data():
    q, k, v = make(Hq=4, Hkv=2, T=64, Tq=8, d=128, kind="int")
    o = Oracle(q, k, v, [64], b_q=4, n_sink=0, n_stream=4)
    import ctypes
    for h in range(4):
        for q0 in (0, 4):
            for p in range(0, 64, 7):
                want = (q[0, h, q0:q0 + 4].long() @ k[0, h // 2, p].long()).max().item()
                got = o.L.orc_score(ctypes.byref(o.t), 0, h, q0, 4, p)
                assert got == float(want)


# --------------------------------------------------------------------------
# 2. nothing pruned  =>  dense causal attention (library SDPA)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("T,Tq,b_q,n_sink,n_stream,stages", [
    (300, 1, 1, 8, 16, ((16, 1000), (4, 1000))),            # decode
    (301, 1, 1, 8, 16, ((16, 1000), (4, 1000))),            # ragged middle
    (200, 32, 8, 4, 8, ((8, 1000), (2, 1000))),             # chunked prefill
    (20, 1, 1, 8, 16, ((4, 10),)),                          # middle range empty
    (5, 1, 1, 8, 16, ((4, 10),)),                           # shorter than the sink
])
def test_keep_everything_equals_dense_sdpa(T, Tq, b_q, n_sink, n_stream, stages):
    B, Hq, Hkv, d = 2, 4, 2, 16
    q, k, v = make(B, Hq, Hkv, T, Tq, d, seed=3)
    o = Oracle(q, k, v, [T] * B, b_q, n_sink, n_stream)
    res = o.layer(stages)
    G = Hq // Hkv
    kk = k.double().repeat_interleave(G, dim=1)
    vv = v.double().repeat_interleave(G, dim=1)
    qpos = torch.arange(T - Tq, T).view(-1, 1)
    mask = torch.arange(T).view(1, -1) <= qpos
    ref = torch.nn.functional.scaled_dot_product_attention(q.double(), kk, vv, attn_mask=mask)
    for (b, g, m), (pr, out, lse) in res.items():
        want = ref[b, g * G:(g + 1) * G, m * b_q:(m + 1) * b_q].numpy()
        np.testing.assert_allclose(out, want, rtol=0, atol=1e-12)
        if pr.stages:
            assert pr.hi <= (T - Tq) + m * b_q + 1          # middle keys precede every query
            assert final_tokens(pr).tolist() == list(range(pr.lo, pr.hi))


# --------------------------------------------------------------------------
# 3. the search is exact  =>  whole pipeline == brute force
# --------------------------------------------------------------------------
@pytest.mark.parametrize("kind", ["int", "normal"])
@pytest.mark.parametrize("stages", [((2, 40), (1, 30)), ((2, 17),), ((1, 50),), ((2, 64), (2, 16))])
def test_chunks_of_two_are_exact(kind, stages):
    # (2,64),(2,16): second stage re-chunks the survivors at the same size
    for seed in range(4):
        q, k, v = make(T=256, d=32, seed=seed, kind=kind)
        o = Oracle(q, k, v, [256], 1, 4, 12)
        for g in range(2):
            pr = o.prune(0, g, 0, stages)
            S = all_scores(q, k, 0, g, 2, 0, 1)
            want = brute_force_prune(S, pr.lo, pr.hi, stages)
            assert final_tokens(pr).tolist() == want.tolist()


@pytest.mark.parametrize("stages", [((32, 4), (8, 6), (4, 5)), ((16, 9), (4, 11))])
def test_chunk_constant_keys_are_exact(stages):
    # every key of a coarsest-stage chunk is the same vector: any representative
    # has the chunk's true maximum at every stage, so the approximate search
    # loses nothing; the finer stages are all ties and test the tie order.
    l_coarse = stages[0][0]
    for seed in range(3):
        q, k, v = make(T=4 + 512 + 12, d=32, seed=seed, Tq=1)
        k = k.clone()
        kb = k[:, :, 4:4 + 512].reshape(1, 2, 512 // l_coarse, l_coarse, 32)
        kb[:] = kb[:, :, :, :1].clone()
        k[:, :, 4:4 + 512] = kb.reshape(1, 2, 512, 32)
        o = Oracle(q, k, v, [528], 1, 4, 12)
        for g in range(2):
            pr = o.prune(0, g, 0, stages)
            pe = o.prune(0, g, 0, stages, exhaustive=True)
            S = all_scores(q, k, 0, g, 2, 0, 1)
            want = brute_force_prune(S, pr.lo, pr.hi, stages)
            assert final_tokens(pr).tolist() == want.tolist()
            assert final_tokens(pe).tolist() == want.tolist()


@pytest.mark.parametrize("stages", [((32, 4), (8, 6), (4, 5)), ((64, 3), (16, 5), (2, 20))])
def test_descending_chunks_are_exact(stages):
    # keys are a_p * u with a_p strictly decreasing inside every coarsest chunk
    # (random level per chunk) and q_h = c_h * u, c_h > 0: inside any chunk of
    # any stage the first key is the best one, which the search always scores.
    l_coarse, d, T = stages[0][0], 16, 4 + 512 + 12
    rng = np.random.default_rng(11)
    for trial in range(3):
        level = rng.permutation(512 // l_coarse).repeat(l_coarse) * 1.0
        a = level * 4.0 - (np.arange(512) % l_coarse) / 32.0 + 1.0
        a = np.concatenate([np.zeros(4), a, np.zeros(12)])
        u = torch.ones(d)
        k = (torch.from_numpy(a).float().view(1, 1, T, 1) * u).to(torch.bfloat16).expand(1, 2, T, d)
        q = (torch.tensor([1.0, 2.0, 0.5, 1.5]).view(1, 4, 1, 1) * u).to(torch.bfloat16)
        o = Oracle(q, k.contiguous(), k.contiguous(), [T], 1, 4, 12)
        for g in range(2):
            pr = o.prune(0, g, 0, stages)
            S = all_scores(q, k, 0, g, 2, 0, 1)
            assert final_tokens(pr).tolist() == brute_force_prune(S, pr.lo, pr.hi, stages).tolist()
            for st in pr.stages:
                assert (st.reps == st.starts[None]).all()


def test_exhaustive_switch_equals_brute_force_on_any_data():
    stages = ((32, 5), (8, 7), (2, 9))
    for kind in ("int", "normal"):
        q, k, v = make(T=4 + 512 + 12, d=32, seed=5, kind=kind)
        o = Oracle(q, k, v, [528], 1, 4, 12)
        pe = o.prune(0, 1, 0, stages, exhaustive=True)
        S = all_scores(q, k, 0, 1, 2, 0, 1)
        assert final_tokens(pe).tolist() == brute_force_prune(S, pe.lo, pe.hi, stages).tolist()


@pytest.mark.parametrize("direction", ["up", "down", "flat"])
def test_monotone_chunks(direction):
    # keys are multiples a_p * u of one vector with q.u > 0: the score is
    # monotone in a_p, so the search must end on the last / first key.
    d, l_c, T = 16, 16, 4 + 64 + 4
    u = torch.ones(d)
    q = torch.ones(1, 1, 1, d).to(torch.bfloat16)
    a = torch.arange(T, dtype=torch.float32)
    a = {"up": a, "down": -a, "flat": torch.zeros(T)}[direction]
    k = (a.view(1, 1, T, 1) * u.view(1, 1, 1, d)).to(torch.bfloat16)
    o = Oracle(q, k, k.clone(), [T], 1, 4, 4)
    pr = o.prune(0, 0, 0, ((l_c, 100),))
    st = pr.stages[0]
    want = st.starts + (l_c - 1 if direction == "up" else 0)
    assert st.reps[0].tolist() == want.tolist()


# --------------------------------------------------------------------------
# 4. independent literal Alg. 3
# --------------------------------------------------------------------------
@pytest.mark.parametrize("kind", ["int", "normal"])
@pytest.mark.parametrize("l_c", [1, 2, 4, 8, 32, 64])
@pytest.mark.parametrize("b_q", [1, 4])
def test_select_rep_equals_literal_algorithm(kind, l_c, b_q):
    T = 8 + 4 * l_c + 8
    for seed in range(6):
        q, k, v = make(T=T, Tq=b_q, d=16, seed=seed, kind=kind)
        o = Oracle(q, k, v, [T], b_q, 0, 8)
        # middle range = [0, T - 8): take the full chunks only
        lo, hi, E = o.ranges(0, 0)
        starts, lens = stage1_chunks(lo, lo + ((hi - lo) // l_c) * l_c, l_c)
        st = o.prune_stage(0, 1, 0, starts, lens, l_c, keep=3)
        S = all_scores(q, k, 0, 1, 2, 0, b_q)               # float64; exact for ints
        if kind == "normal":
            S = S.astype(np.float32)                        # the compare precision
        for hh in range(2):
            for j, s in enumerate(starts.tolist()):
                chunk = list(range(s, s + l_c))
                r = literal_select_rep(lambda p: S[hh, p], chunk)
                assert st.reps[hh, j] == r
        np.testing.assert_allclose(
            st.scores, np.max(S[np.arange(2)[:, None], st.reps], axis=0), rtol=1e-6)


def test_ragged_last_chunk_never_leaves_the_range():
    T, l_c = 8 + 100 + 8, 32
    q, k, v = make(T=T, d=16, seed=1)
    # make the tail past hi irresistible: it must still never be picked
    k = k.clone()
    k[:, :, 108:] = 50.0
    o = Oracle(q, k, v, [T], 1, 8, 8)
    pr = o.prune(0, 0, 0, ((l_c, 2), (8, 3), (2, 5)))
    for st in pr.stages:
        assert (st.reps < pr.hi).all() and (st.reps >= pr.lo).all()
        assert ((st.starts + st.lens) <= pr.hi).all() and (st.lens >= 1).all()
    assert pr.stages[0].lens.tolist() == [32, 32, 32, 4]


# --------------------------------------------------------------------------
# 5. structural invariants on the smallest named workload
# --------------------------------------------------------------------------
def test_structure_on_cfg1():
    w = configs.CFG1
    q, k, v, sl, pos = configs.make_inputs(w, 0)
    o = Oracle(q, k, v, sl, w.b_q, w.n_sink, w.n_stream)
    import ctypes
    for g in (0, 5):
        pr = o.prune(0, g, 0, w.stages)
        assert (pr.lo, pr.hi, pr.E) == (128, 8192 - 1024, 8192)
        parent = None
        for (l_c, keep), st in zip(w.stages, pr.stages):
            n = len(st.starts)
            logl = int(math.log2(l_c))
            assert (np.diff(st.starts) > 0).all()
            assert ((st.starts - pr.lo) % l_c == 0).all()
            assert (st.reps >= st.starts).all() and (st.reps < st.starts + st.lens).all()
            # sigma == score(rep), chunk score == max over the group's heads
            for j in range(0, n, 17):
                s = max(o.L.orc_score(ctypes.byref(o.t), 0, g * w.G + hh, 0, 1, int(st.reps[hh, j]))
                        for hh in range(w.G))
                assert s == st.scores[j]
            # reads: 1 + log2(l_c) keys per (chunk, head); the first two are shared
            assert st.rows_touched <= n * min(l_c, 2 + w.G * (logl - 1))
            assert st.rows_touched >= n * (1 + logl)
            assert len(st.kept_ids) == min(keep, n)
            assert (np.diff(st.kept_ids) > 0).all()
            if parent is not None:                           # children lie inside kept parents
                ps = parent.kept_starts
                inside = (st.starts[:, None] >= ps[None]) & \
                         (st.starts[:, None] < (ps + parent.kept_lens)[None])
                assert inside.any(axis=1).all()
                assert n == len(ps) * (parent.l_c // l_c)
            parent = st
        assert len(final_tokens(pr)) == w.stages[-1][0] * w.stages[-1][1]   # |I^(N)| = k^(N)


def test_reads_are_local():
    # The keys a search scores are fixed by where it ended: the chunk's first
    # key, then at each halving the first key of the right half of the range
    # the result lies in.  Rebuild that set from the representatives alone,
    # check the oracle's own counter against it, and scribble over every other
    # middle key: nothing may change.
    w = configs.shrink(configs.CFG1, T=2048 + 37, n_stream=256, stages=((64, 8), (16, 8), (4, 16)))
    q, k, v, sl, _ = configs.make_inputs(w, 1)
    o = Oracle(q, k, v, sl, 1, w.n_sink, w.n_stream)
    pr = o.prune(0, 0, 0, w.stages)
    touched_all = np.zeros(w.T, bool)
    for st in pr.stages:
        touched = np.zeros(w.T, bool)
        for hh in range(w.G):
            for s, n, r in zip(st.starts.tolist(), st.lens.tolist(), st.reps[hh].tolist()):
                touched[s] = True
                off, half = 0, st.l_c // 2
                while half >= 1:
                    if off + half < n:
                        touched[s + off + half] = True
                    if (r - s) & half:
                        off += half
                    half //= 2
                assert off == r - s
        assert int(touched.sum()) == st.rows_touched
        touched_all |= touched
    free = ~touched_all
    free[:w.n_sink] = False
    free[w.T - w.n_stream:] = False
    assert free.sum() > 1000
    k2 = k.clone()
    k2[0, 0, torch.from_numpy(np.nonzero(free)[0])] = 99.0
    o2 = Oracle(q, k2, v, sl, 1, w.n_sink, w.n_stream)
    pr2 = o2.prune(0, 0, 0, w.stages)
    for a, b in zip(pr.stages, pr2.stages):
        assert a.kept_ids.tolist() == b.kept_ids.tolist()
        assert np.array_equal(a.scores, b.scores) and np.array_equal(a.reps, b.reps)


# --------------------------------------------------------------------------
# 6. needles planted at a chunk's first position survive every stage
# --------------------------------------------------------------------------
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_needles_are_retained_cfg1(seed):
    w = configs.CFG1
    q, k, v, sl, pos = configs.make_inputs(w, seed)
    o = Oracle(q, k, v, sl, w.b_q, w.n_sink, w.n_stream)
    for g in range(w.Hkv):
        kept = set(final_tokens(o.prune(0, g, 0, w.stages)).tolist())
        assert all(int(p) in kept for p in pos[0, g])


# --------------------------------------------------------------------------
# 7. top-K against a library sort
# --------------------------------------------------------------------------
def test_topk_matches_lexsort(oracle_lib):
    import ctypes
    rng = np.random.default_rng(0)
    for n, keep, ties in [(1, 1, False), (10, 3, False), (257, 64, True), (1000, 1000, True),
                          (50, 80, True), (4092, 256, False), (300, 0, True)]:
        s = rng.standard_normal(n).astype(np.float32)
        if ties:
            s = np.round(s * 2) / 2
            s[::7] = -0.0
            s[3::7] = 0.0
        ids = np.empty(max(1, min(keep, n)), np.int32)
        got = oracle_lib.orc_topk(n, s.ctypes.data_as(ctypes.c_void_p), keep,
                                  ids.ctypes.data_as(ctypes.c_void_p))
        want = np.sort(np.lexsort((np.arange(n), -s.astype(np.float64)))[:min(keep, n)])
        assert got == len(want)
        assert ids[:got].tolist() == want.tolist()


# --------------------------------------------------------------------------
# 8. attention against library softmax on explicit key sets
# --------------------------------------------------------------------------
@pytest.mark.parametrize("b_q,Tq", [(1, 1), (4, 8)])
def test_sparse_attention_matches_scipy_softmax(b_q, Tq):
    T, d, n_sink, n_stream = 200, 32, 6, 10
    q, k, v = make(T=T, Tq=Tq, d=d, seed=7)
    o = Oracle(q, k, v, [T], b_q, n_sink, n_stream)
    scale = 0.3
    for m in range(Tq // b_q):
        lo, hi, E = o.ranges(0, m)
        bs = np.array([lo + 3, lo + 40, hi - 5], np.int64)
        bl = np.array([4, 4, 2], np.int32)
        out, lse = o.attend(0, 1, m, bs, bl, scale)
        for hh in range(2):
            for i in range(b_q):
                p = E - b_q + i
                keys = list(range(0, n_sink)) + [x for s, n in zip(bs, bl) for x in range(s, s + n)] \
                    + list(range(hi, p + 1))
                keys = np.array(keys)
                # permutation must not matter
                keys = keys[np.random.default_rng(i).permutation(len(keys))]
                s = scale * f64(k[0, 1])[keys] @ f64(q[0, 2 + hh, m * b_q + i])
                w = scipy.special.softmax(s)
                np.testing.assert_allclose(out[hh, i], w @ f64(v[0, 1])[keys], rtol=0, atol=1e-12)
                np.testing.assert_allclose(lse[hh, i], scipy.special.logsumexp(s), rtol=1e-13)


def test_causality_in_prefill():
    # values after a query's own position are huge: they must never leak in
    T, Tq, b_q = 96, 16, 4
    q, k, v = make(T=T, Tq=Tq, d=16, seed=2)
    o = Oracle(q, k, v, [T], b_q, 4, 8)
    res = o.layer(((8, 3), (2, 6)))
    for (b, g, m), (pr, out, lse) in res.items():
        for i in range(b_q):
            p = T - Tq + m * b_q + i
            v2 = v.clone()
            v2[:, :, p + 1:] = 1e4
            o2 = Oracle(q, k, v2, [T], b_q, 4, 8)
            out2, _ = o2.attend(b, g, m, pr.block_starts, pr.block_lens)
            np.testing.assert_array_equal(out2[:, i], out[:, i])


def test_child_chunks_equal_list_chunking():
    # cutting each kept parent into l-sized pieces == cutting the concatenated
    # index list into l-sized pieces, whenever only the last parent is ragged
    ks = np.array([10, 74, 202, 330], np.int64)
    kl = np.array([64, 64, 64, 23], np.int32)
    for l in (16, 4, 64):
        s, n = child_chunks(ks, kl, l)
        idx = np.concatenate([np.arange(a, a + b) for a, b in zip(ks, kl)])
        pieces = [idx[i:i + l] for i in range(0, len(idx), l)]
        assert s.tolist() == [p[0] for p in pieces]
        assert n.tolist() == [len(p) for p in pieces]
        assert all((np.diff(p) == 1).all() for p in pieces)


# --------------------------------------------------------------------------
# 9. mask caching (Alg. 4): identities that hold whatever the data
# --------------------------------------------------------------------------
def test_mask_caching_identities():
    w = configs.shrink(configs.CFG1, T=2048, n_stream=256, stages=((64, 8), (16, 8), (4, 16)))
    q, k, v, sl, _ = configs.make_inputs(w, 2)
    o = Oracle(q, k, v, sl, 1, w.n_sink, w.n_stream)
    full = o.prune(0, 1, 0, w.stages)
    want = [st.kept_starts.tolist() for st in full.stages]
    none = [np.zeros(0, np.int64)] * 3
    # refreshing every stage == no caching
    kept, bs, bl = o.prune_from(0, 1, 0, w.stages, 0, none)
    assert [x.tolist() for x in kept] == want
    assert bs.tolist() == full.block_starts.tolist() and bl.tolist() == full.block_lens.tolist()
    # same queries, same length: reusing any prefix of cached stages changes nothing
    for first in (1, 2, 3):
        kept2, bs2, bl2 = o.prune_from(0, 1, 0, w.stages, first, kept)
        assert [x.tolist() for x in kept2] == want and bs2.tolist() == bs.tolist()
    # different queries: cached stages stay, later stages follow the new queries inside them
    q2 = gen.normal_bf16(9, 1, tuple(q.shape))
    o2 = Oracle(q2, k, v, sl, 1, w.n_sink, w.n_stream)
    kept3, bs3, _ = o2.prune_from(0, 1, 0, w.stages, 1, kept)
    assert kept3[0].tolist() == want[0]
    parents = set(kept3[0].tolist())
    assert all((s - w.n_sink) // 64 * 64 + w.n_sink in parents for s in kept3[1].tolist())
    assert all(any(p <= s < p + 16 for p in kept3[1].tolist()) for s in bs3.tolist())
    assert kept3[1].tolist() != want[1]      # (new queries do pick different chunks)


# ---------------------------------------------------------------------------
# Paper-literal pooling over all heads (Sec. 4 / Alg. 2: max over h = 1..H)
# ---------------------------------------------------------------------------
def _small_layer(seed, Hq=8, Hkv=4, T=900, kind="normal"):
    torch.manual_seed(seed)
    if kind == "int":
        mk = lambda *s: torch.randint(-2, 3, s).to(torch.bfloat16)
    else:
        mk = lambda *s: torch.randn(*s).to(torch.bfloat16)
    return mk(1, Hq, 1, 128), mk(1, Hkv, T, 128), mk(1, Hkv, T, 128)


def test_all_heads_pooling_with_one_kv_head_is_the_group_pooling():
    q, k, v = _small_layer(0, Hq=4, Hkv=1)
    o = oracle.Oracle(q, k, v, [900], 1, 16, 64)
    stages = [(32, 8), (8, 12), (2, 20)]
    a, b = o.prune(0, 0, 0, stages), o.prune_all_heads(0, 0, stages)[0]
    for sa, sb in zip(a.stages, b.stages):
        assert np.array_equal(sa.scores, sb.scores) and np.array_equal(sa.kept_ids, sb.kept_ids)


def test_all_heads_pooling_is_the_max_over_every_head_and_one_mask():
    q, k, v = _small_layer(1, kind="int")
    o = oracle.Oracle(q, k, v, [900], 1, 16, 64)
    stages = [(32, 8), (8, 12)]
    prs = o.prune_all_heads(0, 0, stages)
    G = o.G
    for i in range(len(stages)):
        st0 = prs[0].stages[i]
        # the pooled score of chunk j is the best q_h . k_{rep_h} over all Hq heads, each head
        # against its own KV head's keys (recomputed here from the raw tensors)
        for j in range(len(st0.starts)):
            best = -np.inf
            for g in range(o.Hkv):
                for hh in range(G):
                    r = int(prs[g].stages[i].reps[hh, j])
                    best = max(best, float((q[0, g * G + hh, 0].double() * k[0, g, r].double()).sum()))
            assert st0.scores[j] == best
        # one mask for the layer
        for g in range(1, o.Hkv):
            assert np.array_equal(prs[g].stages[i].kept_ids, st0.kept_ids)
            assert np.array_equal(prs[g].stages[i].starts, st0.starts)


def test_all_heads_pooling_ignores_the_order_of_the_kv_heads():
    q, k, v = _small_layer(2)
    o = oracle.Oracle(q, k, v, [900], 1, 16, 64)
    perm = [2, 0, 3, 1]
    G = 2
    qp = torch.cat([q[:, g * G:(g + 1) * G] for g in perm], 1)
    op = oracle.Oracle(qp, k[:, perm], v[:, perm], [900], 1, 16, 64)
    stages = [(32, 8), (8, 12), (2, 20)]
    a, b = o.prune_all_heads(0, 0, stages), op.prune_all_heads(0, 0, stages)
    for sa, sb in zip(a[0].stages, b[0].stages):
        assert np.array_equal(sa.kept_starts, sb.kept_starts) and np.array_equal(sa.scores, sb.scores)
