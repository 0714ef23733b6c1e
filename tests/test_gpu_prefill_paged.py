"""GPU parity of the chunked-prefill path reading K/V from a paged pool through a
block table: the logical tensors are scattered into randomly ordered pages; the
result must equal the library's own contiguous path exactly (same arithmetic,
other addresses) and the oracle on the logical tensors (bit-exact kept sets on
integer inputs)."""
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


def small(Tq=256, prefix=2048, b_q=64, B=1, Hq=32, Hkv=8, n_stream=256, stages=((64, 8), (16, 16)), **kw):
    return configs.shrink(configs.CFG4, B=B, Hq=Hq, Hkv=Hkv, T=prefix + Tq, Tq=Tq, b_q=b_q,
                          n_stream=n_stream, stages=stages, **kw)


def scatter_to_pages(k, v, page, seed, spare=5):
    """[B,Hkv,T,d] -> pools [n_pages,Hkv,page,d] with a seeded random page order + block table."""
    B, Hkv, T, d = k.shape
    per_seq = (T + page - 1) // page
    n_pages = B * per_seq + spare
    order = gen.distinct_ints(seed, 77, B * per_seq, n_pages).view(B, per_seq)
    k_pool = torch.full((n_pages, Hkv, page, d), 7.0, dtype=torch.bfloat16)      # unused rows hold junk
    v_pool = torch.full((n_pages, Hkv, page, d), -7.0, dtype=torch.bfloat16)
    pad = per_seq * page - T
    kp = torch.nn.functional.pad(k, (0, 0, 0, pad)).view(B, Hkv, per_seq, page, d)
    vp = torch.nn.functional.pad(v, (0, 0, 0, pad)).view(B, Hkv, per_seq, page, d)
    for b in range(B):
        k_pool[order[b]] = kp[b].permute(1, 0, 2, 3)
        v_pool[order[b]] = vp[b].permute(1, 0, 2, 3)
    return k_pool, v_pool, order.to(torch.int32)


@pytest.mark.parametrize("page", [16, 64])
@pytest.mark.parametrize("w", [
    small(),                                              # Llama shape, 4 query blocks
    small(prefix=2048 + 37, B=2, Hq=8, Hkv=2),            # ragged middle, two sequences
    small(b_q=16, Tq=64, Hq=4, Hkv=2, stages=((32, 8), (8, 16), (2, 40))),     # the 16x16 attention kernel
    small(Hq=16, Hkv=2, Tq=64),                           # G = 8
], ids=["llama", "ragged-b2", "bq16-3stage", "g8"])
def test_paged_prefill_matches_contiguous_path_and_oracle(ihip, orc, w, page):
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if w.B == 2:
        sl = torch.tensor([w.T, w.T - 517], dtype=torch.int32)
    k_pool, v_pool, table = scatter_to_pages(k, v, page, seed=3)
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    L = ihip.Layer(qd, kd, sld, w.b_q, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]

    parents, pchunk = None, 0
    for (l_c, keep) in w.stages:
        scores, rep = L.prune_stage(qd, None, l_c, parents, pchunk, want_rep=True, paged=pg)
        ref_scores, ref_rep = L.prune_stage(qd, kd, l_c, parents, pchunk, want_rep=True)
        assert torch.equal(scores, ref_scores) and torch.equal(rep, ref_rep), l_c
        parents, pchunk = L.select_blocks(scores, l_c, keep, parents, pchunk), l_c
    out, lse = L.sparse_attn_prefill(qd, None, None, parents, pchunk, want_lse=True, paged=pg)
    ref_out, ref_lse = L.sparse_attn_prefill(qd, kd, vd, parents, pchunk, want_lse=True)
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    blocks = torch.empty_like(parents)
    fused = L.prefill_layer(qd, None, None, chunks, keeps, paged=pg, out_blocks=blocks)
    assert torch.equal(fused, out) and torch.equal(blocks, parents)

    # and against the oracle on the logical tensors (a sample of the problems)
    o = orc.Oracle(q, k, v, sl.tolist(), w.b_q, w.n_sink, w.n_stream)
    for (b, g, m) in [(0, 0, 0), (w.B - 1, w.Hkv - 1, w.Mq - 1)]:
        p = (b * w.Hkv + g) * w.Mq + m
        pr = o.prune(b, g, m, w.stages)
        kp = parents[p].cpu().numpy()
        assert np.array_equal(kp[kp >= 0], pr.block_starts)
        ref, _ = o.attend(b, g, m, pr.block_starts, pr.block_lens)
        got = out[b, g * w.G:(g + 1) * w.G, m * w.b_q:(m + 1) * w.b_q].float().cpu().numpy()
        assert np.abs(got - ref).max() <= 2e-2


@pytest.mark.parametrize("w", [small(), small(b_q=16, Tq=64, Hq=4, Hkv=2, stages=((32, 8), (8, 16), (2, 40)))],
                         ids=["llama", "bq16-3stage"])
def test_paged_prefill_with_rope_and_pooling_equals_contiguous(ihip, w):
    q, k, v, sl, _ = configs.make_inputs(w, 1)
    cos, sin = gen.rope_table(w.T, w.d)
    k_pool, v_pool, table = scatter_to_pages(k, v, 16, seed=5)
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    rp = ihip.Rope(cos.cuda(), sin.cuda(), ihip.ROPE_RELATIVE, ihip.ROPE_STREAMING)
    L = ihip.Layer(qd, kd, sld, w.b_q, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    for pooling in (None, ihip.POOL_ALL_HEADS):
        b1 = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
        b2 = torch.empty_like(b1)
        got = L.prefill_layer(qd, None, None, chunks, keeps, rope=rp, paged=pg, pooling=pooling, out_blocks=b1)
        if pooling is None:
            ref = L.prefill_layer(qd, kd, vd, chunks, keeps, rope=rp, out_blocks=b2)
        else:       # contiguous RoPE + pooling also goes through the combined entry point
            ref = L.prefill_layer(qd, kd, vd, chunks, keeps, rope=rp, pooling=pooling, out_blocks=b2)
        torch.cuda.synchronize()
        assert torch.equal(b1, b2)
        assert torch.equal(got, ref)
    # and the attention alone, paged + RoPE against contiguous + RoPE
    out, _ = L.sparse_attn_prefill(qd, None, None, b1, chunks[-1], rope=rp, paged=pg)
    ref, _ = L.sparse_attn_prefill(qd, kd, vd, b1, chunks[-1], rope=rp)
    assert torch.equal(out, ref)


@pytest.mark.parametrize("prefix", [11000, 13440, 15000])
def test_keep_everything_paged_is_dense_causal(ihip, prefix):
    # every chunk kept -> dense causal attention (torch, fp64), read through 16-token pages.
    # prefix 13440: exactly the key slots the 32x32 kernel keeps in LDS with page ids (14,272);
    # prefix 15000: above them -> the 16x16 kernel runs.
    keep = (prefix + 512) // 64 + 1
    w = small(Tq=512, prefix=prefix, n_stream=128, stages=((64, keep), (16, 4 * keep)))
    q, k, v, sl, _ = configs.make_inputs(w, 5)
    k_pool, v_pool, table = scatter_to_pages(k, v, 16, seed=9)
    qd, kd, sld = q.cuda(), k.cuda(), sl.cuda()
    pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    L = ihip.Layer(qd, kd, sld, w.b_q, w.n_sink, w.n_stream)
    out = L.prefill_layer(qd, None, None, [s[0] for s in w.stages], [s[1] for s in w.stages], paged=pg)
    torch.cuda.synchronize()
    G, T, Tq = w.G, w.T, w.Tq
    mask = torch.arange(T).view(1, -1) <= torch.arange(T - Tq, T).view(-1, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(G, 1), v.double().repeat_interleave(G, 1), attn_mask=mask)
    assert (out.cpu().double() - ref).abs().max().item() <= 2e-2
