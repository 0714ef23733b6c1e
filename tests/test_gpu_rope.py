"""GPU parity of the decode path with dynamic RoPE (Sec. 4 "Dynamic RoPE for
OOL generalization") against the CPU oracle, through the C ABI.

Bit-exact bar: integer-valued Q/K/V with a quarter-turn rotary table (cos and
sin are 0 or +-1, so every rotated vector and every product stays an exact
integer on both sides).  Real tables on Gaussian inputs: block recall >= 0.99
and outputs within 2e-2, as for the plain path.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import configs, gen  # noqa: E402


@pytest.fixture(scope="module")
def ihip():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_08910_amd as pkg
    pkg.lib()
    return pkg


@pytest.fixture(scope="module")
def orc():
    import oracle
    oracle.build(force=False)
    return oracle


STYLE = {"relative": 1, "chunk": 2}


def run_gpu(ihip, w, q, k, v, sl, cos, sin, prune, attn):
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    rp = ihip.Rope(cos.cuda(), sin.cuda(), STYLE[prune] if prune else ihip.ROPE_NONE,
                   ihip.ROPE_STREAMING if attn else ihip.ROPE_NONE)
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    stages, parents, pchunk = [], None, 0
    for (l_c, keep) in w.stages:
        scores, rep = L.prune_stage(qd, kd, l_c, parents, pchunk, want_rep=True, rope=rp if prune else None)
        kept = L.select_blocks(scores, l_c, keep, parents, pchunk)
        stages.append((scores, rep, kept))
        parents, pchunk = kept, l_c
    out, lse = L.sparse_attn_decode(qd, kd, vd, parents, pchunk, want_lse=True, rope=rp if attn else None)
    fused = L.decode_layer(qd, kd, vd, [s[0] for s in w.stages], [s[1] for s in w.stages], rope=rp)
    torch.cuda.synchronize()
    return stages, out, lse, fused


def compare(w, o, stages, out, lse, exact):
    G = w.G
    worst, min_recall = 0.0, 1.0
    for b in range(w.B):
        for g in range(w.Hkv):
            p = b * w.Hkv + g
            pr = o.prune(b, g, 0, w.stages)
            for i, st in enumerate(pr.stages):
                scores, rep, kept = stages[i]
                n = len(st.starts)
                sc, kp = scores[p].cpu().numpy(), kept[p].cpu().numpy()
                if exact:
                    assert np.array_equal(sc[:n], st.scores), (b, g, i)
                    assert np.isneginf(sc[n:]).all()
                    rp = rep[b, g * G:(g + 1) * G, 0].cpu().numpy()
                    assert np.array_equal(rp[:, :n], st.reps), (b, g, i)
                    assert np.array_equal(kp[:len(st.kept_starts)], st.kept_starts), (b, g, i)
                    assert (kp[len(st.kept_starts):] == -1).all()
                else:
                    np.testing.assert_allclose(sc[:n], st.scores, rtol=2e-5, atol=2e-4)
                    want, got = set(st.kept_starts.tolist()), set(kp[kp >= 0].tolist())
                    assert len(got) == len(want)
                    min_recall = min(min_recall, len(got & want) / max(1, len(want)))
            ref, ref_lse = o.attend(b, g, 0, pr.block_starts, pr.block_lens)
            got = out[b, g * G:(g + 1) * G, 0].float().cpu().numpy()
            worst = max(worst, np.abs(got - ref[:, 0]).max())
            if exact:
                np.testing.assert_allclose(lse[b, g * G:(g + 1) * G, 0].cpu().numpy(), ref_lse[:, 0],
                                           rtol=1e-5, atol=1e-5)
    return worst, min_recall


@pytest.mark.parametrize("prune", ["relative", "chunk"])
@pytest.mark.parametrize("T,B", [(8192, 1), (4096 + 37, 2)])
def test_quarter_turn_table_bit_exact(ihip, orc, prune, T, B):
    w = configs.shrink(configs.CFG1, T=T, B=B, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if B == 2:
        sl = torch.tensor([T, T - 1001], dtype=torch.int32)
    cos, sin = gen.quarter_turn_table(T, w.d)
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream,
                   rope=orc.RopeSpec(cos.numpy(), sin.numpy(), prune=prune, attn="streaming"))
    stages, out, lse, fused = run_gpu(ihip, w, q, k, v, sl, cos, sin, prune, True)
    worst, _ = compare(w, o, stages, out, lse, exact=True)
    assert worst <= 2e-2
    assert torch.equal(fused, out)          # the one-enqueue layer call runs the same kernels


def test_rope_changes_the_selection(ihip, orc):
    # guards against a path that silently ignores the table: same inputs, with and without RoPE
    w = configs.shrink(configs.CFG1, T=4096, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    cos, sin = gen.quarter_turn_table(4096, w.d)
    with_rope = run_gpu(ihip, w, q, k, v, sl, cos, sin, "relative", True)
    without = run_gpu(ihip, w, q, k, v, sl, cos, sin, None, False)
    assert not torch.equal(with_rope[0][0][0], without[0][0][0])
    assert not torch.equal(with_rope[1], without[1])


@pytest.mark.parametrize("prune", ["relative", "chunk"])
def test_real_table_gaussian_recall_and_output(ihip, orc, prune):
    w = configs.CFG1
    q, k, v, sl, _ = configs.make_inputs(w, 1)
    cos, sin = gen.rope_table(w.T, w.d)
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream,
                   rope=orc.RopeSpec(cos.numpy(), sin.numpy(), prune=prune, attn="streaming"))
    stages, out, lse, fused = run_gpu(ihip, w, q, k, v, sl, cos, sin, prune, True)
    worst, recall = compare(w, o, stages, out, lse, exact=False)
    assert recall >= 0.99
    assert worst <= 2e-2


def test_streaming_attention_alone_on_oracle_indices(ihip, orc):
    # few kept blocks, many empty slots in the block list: window keys must skip them when numbered
    w = configs.shrink(configs.CFG1, T=3000, n_needles=0, stages=((64, 6), (16, 40), (4, 200)))
    q, k, v, sl, _ = configs.make_inputs(w, 2)
    cos, sin = gen.rope_table(4096, w.d)
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream,
                   rope=orc.RopeSpec(cos.numpy(), sin.numpy(), attn="streaming"))
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    rp = ihip.Rope(cos.cuda(), sin.cuda(), ihip.ROPE_NONE, ihip.ROPE_STREAMING)
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    n_slots = w.stages[-1][1]
    starts = np.full((w.Hkv, n_slots), -1, np.int32)
    refs = []
    for g in range(w.Hkv):
        pr = o.prune(0, g, 0, w.stages)
        assert len(pr.block_starts) < n_slots          # some slots stay empty
        starts[g, :len(pr.block_starts)] = pr.block_starts
        refs.append(o.attend(0, g, 0, pr.block_starts, pr.block_lens))
    out, lse = L.sparse_attn_decode(qd, kd, vd, torch.from_numpy(starts).cuda(), w.stages[-1][0],
                                    want_lse=True, rope=rp)
    for g in range(w.Hkv):
        got = out[0, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy()
        assert np.abs(got - refs[g][0][:, 0]).max() <= 4e-3
        np.testing.assert_allclose(lse[0, g * w.G:(g + 1) * w.G, 0].cpu().numpy(), refs[g][1][:, 0],
                                   rtol=2e-5, atol=2e-5)


def test_short_table_is_refused(ihip):
    w = configs.shrink(configs.CFG1, T=2048, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    cos, sin = gen.quarter_turn_table(8, w.d)
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    rp = ihip.Rope(cos.cuda(), sin.cuda(), ihip.ROPE_RELATIVE, ihip.ROPE_STREAMING)
    with pytest.raises(ihip.IhipError):
        L.prune_stage(qd, kd, 64, rope=rp)
