"""GPU parity of the paper-literal pooling of chunk scores over all heads (one
mask per layer; Sec. 4 and Alg. 2, max over h = 1..H) against the oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import configs  # noqa: E402


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


def stagewise(ihip, L, w, q, k):
    stages, parents, pchunk = [], None, 0
    for (l_c, keep) in w.stages:
        scores, _ = L.prune_stage(q, k, l_c, parents, pchunk)
        kept = L.select_blocks(scores, l_c, keep, parents, pchunk, pooling=ihip.POOL_ALL_HEADS)
        stages.append((scores, kept))
        parents, pchunk = kept, l_c
    return stages


@pytest.mark.parametrize("T,B", [(8192, 1), (4096 + 37, 2)])
def test_decode_integer_inputs_bit_exact(ihip, orc, T, B):
    w = configs.shrink(configs.CFG1, T=T, B=B, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if B == 2:
        sl = torch.tensor([T, T - 1001], dtype=torch.int32)
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    stages = stagewise(ihip, L, w, qd, kd)
    blocks = torch.empty((L.P, w.stages[-1][1]), dtype=torch.int32, device="cuda")
    out = L.decode_layer(qd, kd, vd, [s[0] for s in w.stages], [s[1] for s in w.stages],
                         pooling=ihip.POOL_ALL_HEADS, out_blocks=blocks)
    torch.cuda.synchronize()
    for b in range(B):
        prs = o.prune_all_heads(b, 0, w.stages)
        for g in range(w.Hkv):
            p = b * w.Hkv + g
            for i, st in enumerate(prs[g].stages):
                scores, kept = stages[i]
                # the per-KV-head scores the stage writes, pooled on the host, are the oracle's pooled scores
                pooled = scores[b * w.Hkv:(b + 1) * w.Hkv].max(0).values.cpu().numpy()
                assert np.array_equal(pooled[:len(st.scores)], st.scores)
                kp = kept[p].cpu().numpy()
                assert np.array_equal(kp[:len(st.kept_starts)], st.kept_starts), (b, g, i)
                assert (kp[len(st.kept_starts):] == -1).all()
            fb = blocks[p].cpu().numpy()
            assert np.array_equal(fb[fb >= 0], prs[g].block_starts)
            ref, _ = o.attend(b, g, 0, prs[g].block_starts, prs[g].block_lens)
            got = out[b, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy()
            assert np.abs(got - ref[:, 0]).max() <= 2e-2
        # one mask per layer
        assert all(torch.equal(blocks[b * w.Hkv], blocks[b * w.Hkv + g]) for g in range(1, w.Hkv))


def test_kv_head_pooling_flag_is_the_default_path(ihip):
    w = configs.shrink(configs.CFG1, T=4096, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 1)
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    a = L.decode_layer(qd, kd, vd, chunks, keeps)
    b = L.decode_layer(qd, kd, vd, chunks, keeps, pooling=ihip.POOL_KV_HEAD)
    c = L.decode_layer(qd, kd, vd, chunks, keeps, pooling=ihip.POOL_ALL_HEADS)
    assert torch.equal(a, b) and not torch.equal(a, c)


def test_prefill_layer_all_heads_bit_exact_sets(ihip, orc):
    w = configs.shrink(configs.CFG4, B=1, Hq=8, Hkv=2, T=2048 + 256, Tq=256, b_q=64, n_stream=256,
                       stages=((64, 8), (16, 16)))
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    o = orc.Oracle(q, k, v, sl.tolist(), w.b_q, w.n_sink, w.n_stream)
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    L = ihip.Layer(qd, kd, sld, w.b_q, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, w.stages[-1][1]), dtype=torch.int32, device="cuda")
    out = L.prefill_layer(qd, kd, vd, [s[0] for s in w.stages], [s[1] for s in w.stages],
                          pooling=ihip.POOL_ALL_HEADS, out_blocks=blocks)
    torch.cuda.synchronize()
    for m in range(w.Mq):
        prs = o.prune_all_heads(0, m, w.stages)
        for g in range(w.Hkv):
            p = g * w.Mq + m
            fb = blocks[p].cpu().numpy()
            assert np.array_equal(fb[fb >= 0], prs[g].block_starts), (g, m)
            ref, _ = o.attend(0, g, m, prs[g].block_starts, prs[g].block_lens)
            got = out[0, g * w.G:(g + 1) * w.G, m * w.b_q:(m + 1) * w.b_q].float().cpu().numpy()
            assert np.abs(got - ref).max() <= 2e-2
