"""GPU parity of chunked prefill with a query-block size per pruning stage
(Sec. 4, the m' rule; Alg. 1 "subdivide query blocks") against the oracle run
with the same block sizes, through the C ABI: bit-exact scores and kept lists
on integer inputs, stage by stage and through the combined layer call, with
the variants on top; dense causal attention when nothing is pruned."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import configs, gen  # noqa: E402
from test_gpu_random_shapes import scatter_to_pages  # noqa: E402


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


def small(stage_b_q, Tq=256, prefix=2048, B=1, Hq=32, Hkv=8, n_stream=256, stages=((64, 8), (16, 16)), **kw):
    return configs.shrink(configs.CFG4, B=B, Hq=Hq, Hkv=Hkv, T=prefix + Tq, Tq=Tq, b_q=stage_b_q[-1],
                          n_stream=n_stream, stages=stages, **kw)


CASES = [
    ((64, 32), dict()),                                                        # Llama shape
    ((64, 16), dict(Hq=8, Hkv=2, prefix=2048 + 37, B=2)),                      # ragged middle, two sequences
    ((64, 32, 16), dict(Hq=4, Hkv=2, stages=((32, 8), (8, 16), (2, 40)))),
    ((32, 32, 16), dict(Hq=16, Hkv=2, Tq=64, stages=((32, 8), (8, 16), (2, 40)))),   # G = 8, drop at the last stage
    ((64, 64), dict(Hq=8, Hkv=8, Tq=128)),                                     # no drop: the plain path
    ((32, 16), dict(Hq=2, Hkv=2, Tq=96, n_stream=70, n_sink=5)),               # window no multiple of anything
]
IDS = ["llama-64-32", "ragged-b2-64-16", "three-stages", "g8-32-32-16", "equal", "odd-window"]


@pytest.mark.parametrize("stage_b_q,kw", CASES, ids=IDS)
def test_integer_inputs_bit_exact_stage_by_stage_and_fused(ihip, orc, stage_b_q, kw):
    w = small(stage_b_q, **kw)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if w.B == 2:
        sl = torch.tensor([w.T, w.T - 517], dtype=torch.int32)
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    o = orc.Oracle(q, k, v, sl.tolist(), w.b_q, w.n_sink, w.n_stream, stage_b_q=stage_b_q)
    first = stage_b_q[0]

    # stage by stage: a layer object per block size, kept lists subdivided where it drops
    per_stage, parents, pchunk = [], None, 0
    for i, (l_c, keep) in enumerate(w.stages):
        Li = ihip.Layer(qd, kd, sld, stage_b_q[i], w.n_sink, w.n_stream, b_q_range=first)
        scores, rep = Li.prune_stage(qd, kd, l_c, parents, pchunk, want_rep=True)
        kept = Li.select_blocks(scores, l_c, keep, parents, pchunk)
        per_stage.append((scores, rep, kept))
        parents, pchunk = kept, l_c
        if i + 1 < len(w.stages) and stage_b_q[i + 1] != stage_b_q[i]:
            parents = Li.subdivide_blocks(kept, stage_b_q[i + 1])
    La = ihip.Layer(qd, kd, sld, w.b_q, w.n_sink, w.n_stream, b_q_range=first)
    out, lse = La.sparse_attn_prefill(qd, kd, vd, parents, pchunk, want_lse=True)

    # the combined call
    L = ihip.Layer(qd, kd, sld, w.b_q, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, w.stages[-1][1]), dtype=torch.int32, device="cuda")
    fused = L.prefill_layer(qd, kd, vd, [s[0] for s in w.stages], [s[1] for s in w.stages], stage_b_q=stage_b_q,
                            out_blocks=blocks)
    torch.cuda.synchronize()
    assert torch.equal(blocks, parents) and torch.equal(fused, out)

    G, fine = w.G, w.b_q
    for b in range(w.B):
        for g in range(w.Hkv):
            for m in range(w.Tq // fine):
                pr = o.prune(b, g, m, w.stages)
                for i, st in enumerate(pr.stages):
                    scores, rep, kept = per_stage[i]
                    bq = stage_b_q[i]
                    mi = m * fine // bq
                    p = (b * w.Hkv + g) * (w.Tq // bq) + mi
                    n = len(st.starts)
                    sc = scores[p].cpu().numpy()
                    assert np.array_equal(sc[:n], st.scores) and np.isneginf(sc[n:]).all(), (b, g, m, i)
                    rp = rep[b, g * G:(g + 1) * G, mi].cpu().numpy()
                    assert np.array_equal(rp[:, :n], st.reps), (b, g, m, i)
                    kp = kept[p].cpu().numpy()
                    assert np.array_equal(kp[kp >= 0], st.kept_starts), (b, g, m, i)
                ref, ref_lse = o.attend(b, g, m, pr.block_starts, pr.block_lens)
                got = out[b, g * G:(g + 1) * G, m * fine:(m + 1) * fine].float().cpu().numpy()
                assert np.abs(got - ref).max() <= 2e-2, (b, g, m)
                np.testing.assert_allclose(lse[b, g * G:(g + 1) * G, m * fine:(m + 1) * fine].cpu().numpy(), ref_lse,
                                           rtol=2e-5, atol=2e-5)


@pytest.mark.parametrize("rope", [None, "relative", "chunk"])
@pytest.mark.parametrize("fp8,page", [(False, 0), (True, 16), (False, 64)])
def test_with_rope_pages_fp8_and_pooling_bit_exact(ihip, orc, rope, fp8, page):
    stage_b_q = (64, 32, 16)
    w = small(stage_b_q, Hq=8, Hkv=2, Tq=128, stages=((32, 8), (8, 16), (2, 40)))
    q, k, v, sl, _ = configs.make_inputs(w, 4, kind="int")
    scales = (0.5, 0.25) if fp8 else None
    if fp8:
        k, v = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    cos, sin = gen.quarter_turn_table(w.T + 64, w.d)
    spec = orc.RopeSpec(cos.numpy(), sin.numpy(), prune=rope, attn="streaming") if rope else None
    rp = None
    if rope:
        style = ihip.ROPE_RELATIVE if rope == "relative" else ihip.ROPE_CHUNK_INDEXED
        rp = ihip.Rope(cos.cuda(), sin.cuda(), style, ihip.ROPE_STREAMING)
    pg = None
    if page:
        k_pool, v_pool, table = scatter_to_pages(k, v, page, 13, 7)
        pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    L = ihip.Layer(qd, kd, sl.cuda(), w.b_q, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    o = orc.Oracle(q, k, v, sl.tolist(), w.b_q, w.n_sink, w.n_stream, rope=spec, kv_scales=scales, stage_b_q=stage_b_q)
    for pooling in (None, ihip.POOL_ALL_HEADS):
        blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
        out = L.prefill_layer(qd, kd, vd, chunks, keeps, rope=rp, paged=pg, pooling=pooling, kv_scales=scales,
                              stage_b_q=stage_b_q, out_blocks=blocks)
        torch.cuda.synchronize()
        for m in range(w.Mq):
            prs = o.prune_all_heads(0, m, w.stages) if pooling else [o.prune(0, g, m, w.stages) for g in range(w.Hkv)]
            for g in range(w.Hkv):
                p = g * w.Mq + m
                kp = blocks[p].cpu().numpy()
                assert np.array_equal(kp[kp >= 0], prs[g].block_starts), (pooling, g, m)
                ref, _ = o.attend(0, g, m, prs[g].block_starts, prs[g].block_lens)
                got = out[0, g * w.G:(g + 1) * w.G, m * w.b_q:(m + 1) * w.b_q].float().cpu().numpy()
                assert np.abs(got - ref).max() <= 2e-2, (pooling, g, m)


@pytest.mark.parametrize("stage_b_q", [(64, 32), (64, 16)])
def test_keep_everything_is_dense_causal(ihip, stage_b_q):
    # sink + the coarse block's whole middle range + the window from there to the query = every
    # key up to the query (torch, fp64), for Gaussian inputs
    prefix = 3000
    keep = (prefix + 256) // 64 + 1
    w = small(stage_b_q, Tq=256, prefix=prefix, n_stream=128, Hq=8, Hkv=2, stages=((64, keep), (16, 4 * keep)))
    q, k, v, sl, _ = configs.make_inputs(w, 5)
    L = ihip.Layer(q.cuda(), k.cuda(), sl.cuda(), w.b_q, w.n_sink, w.n_stream)
    out = L.prefill_layer(q.cuda(), k.cuda(), v.cuda(), [s[0] for s in w.stages], [s[1] for s in w.stages],
                          stage_b_q=stage_b_q)
    torch.cuda.synchronize()
    G, T, Tq = w.G, w.T, w.Tq
    mask = torch.arange(T).view(1, -1) <= torch.arange(T - Tq, T).view(-1, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(G, 1), v.double().repeat_interleave(G, 1), attn_mask=mask)
    assert (out.cpu().double() - ref).abs().max().item() <= 2e-2


def test_bad_block_sizes_are_refused(ihip):
    w = small((64, 32), Hq=8, Hkv=2)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    L = ihip.Layer(qd, kd, sl.cuda(), 32, w.n_sink, w.n_stream)
    chunks, keeps = [64, 16], [8, 16]
    for bad in ([32, 64], [64, 16], [48, 32], [16, 32]):     # growing, last != b_q, not 16/32/64
        with pytest.raises(ihip.IhipError):
            L.prefill_layer(qd, kd, vd, chunks, keeps, stage_b_q=bad)
    with pytest.raises(ihip.IhipError):        # range block larger than the window
        ihip.Layer(qd, kd, sl.cuda(), 32, w.n_sink, 32, b_q_range=64).prune_stage(qd, kd, 64)
