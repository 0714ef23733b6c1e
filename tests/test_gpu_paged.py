"""GPU parity of the decode path reading K/V from a paged pool through a block
table: the logical tensors are scattered into randomly ordered pages; the
result must equal the oracle on the logical tensors (bit-exact sets on integer
inputs) and the library's own contiguous path exactly."""
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
@pytest.mark.parametrize("T,B", [(8192, 1), (4096 + 37, 2)])
def test_paged_decode_matches_oracle_and_contiguous_path(ihip, orc, page, T, B):
    w = configs.shrink(configs.CFG1, T=T, B=B, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if B == 2:
        sl = torch.tensor([T, T - 1001], dtype=torch.int32)
    k_pool, v_pool, table = scatter_to_pages(k, v, page, seed=3)
    qd, kd, vd, sld = [t.cuda() for t in (q, k, v, sl)]
    pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]

    # stage by stage through the paged entry points
    parents, pchunk, per_stage = None, 0, []
    for (l_c, keep) in w.stages:
        scores, rep = L.prune_stage(qd, None, l_c, parents, pchunk, want_rep=True, paged=pg)
        ref_scores, ref_rep = L.prune_stage(qd, kd, l_c, parents, pchunk, want_rep=True)
        assert torch.equal(scores, ref_scores) and torch.equal(rep, ref_rep)
        parents, pchunk = L.select_blocks(scores, l_c, keep, parents, pchunk), l_c
        per_stage.append(parents)
    out, lse = L.sparse_attn_decode(qd, None, None, parents, pchunk, want_lse=True, paged=pg)
    ref_out, ref_lse = L.sparse_attn_decode(qd, kd, vd, parents, pchunk, want_lse=True)
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    fused = L.decode_layer(qd, None, None, chunks, keeps, paged=pg)
    assert torch.equal(fused, out)

    # and against the oracle on the logical tensors
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
    for b in range(B):
        for g in range(w.Hkv):
            pr = o.prune(b, g, 0, w.stages)
            kp = per_stage[-1][b * w.Hkv + g].cpu().numpy()
            assert np.array_equal(kp[kp >= 0], pr.block_starts)
            ref, _ = o.attend(b, g, 0, pr.block_starts, pr.block_lens)
            got = out[b, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy()
            assert np.abs(got - ref[:, 0]).max() <= 2e-2


def test_short_block_table_is_refused(ihip):
    w = configs.shrink(configs.CFG1, T=2048, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    k_pool, v_pool, table = scatter_to_pages(k, v, 16, seed=1)
    pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table[:, :10].contiguous().cuda())
    L = ihip.Layer(q.cuda(), k.cuda(), sl.cuda(), 1, w.n_sink, w.n_stream)
    with pytest.raises(ihip.IhipError):
        L.prune_stage(q.cuda(), None, 64, paged=pg)
