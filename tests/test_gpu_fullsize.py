"""Parity at the full benchmark sizes, in the launch configuration bench.py
times (the fused ihip_decode_layer call), on sampled problems the oracle
computes one by one from the same data (copied to the host)."""
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


def check_samples(ihip, orc, w, kind, samples, seed=0):
    dev = torch.device("cuda:0")
    q, k, v, sl, pos = configs.make_inputs(w, seed, device=dev, kind=kind)
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    L = ihip.Layer(q, k, sl, 1, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device=dev)
    out = L.decode_layer(q, k, v, chunks, keeps, out_blocks=blocks)
    torch.cuda.synchronize()
    G = w.G
    for (b, g) in samples:
        p = b * w.Hkv + g
        o = orc.Oracle(q[b:b + 1, g * G:(g + 1) * G].cpu(), k[b:b + 1, g:g + 1].cpu(),
                       v[b:b + 1, g:g + 1].cpu(), [w.T], 1, w.n_sink, w.n_stream)
        pr = o.prune(0, 0, 0, w.stages)
        got = blocks[p].cpu().numpy()
        got = got[got >= 0]
        assert (np.diff(got) > 0).all()
        want = pr.block_starts
        if kind == "int":
            assert np.array_equal(got, want), (b, g)
        else:
            recall = len(set(got.tolist()) & set(want.tolist())) / len(want)
            assert recall >= 0.99, (b, g, recall)
            l_n = chunks[-1]
            kept = set((got[:, None] + np.arange(l_n)[None]).ravel().tolist())
            assert all(int(x) in kept for x in pos[b, g]), "a planted needle was dropped"
        ref, _ = o.attend(0, 0, 0, pr.block_starts, pr.block_lens)
        err = np.abs(out[b, g * G:(g + 1) * G, 0].float().cpu().numpy() - ref[:, 0]).max()
        assert err <= 2e-2, (b, g, err)
        # properties that hold at any size
        assert len(got) == keeps[-1]
        assert got.min() >= w.n_sink and got.max() + l_n_of(w) <= w.T - w.n_stream


def l_n_of(w):
    return w.stages[-1][0]


@pytest.mark.parametrize("kind", ["normal", "int"])
def test_cfg2_128k(ihip, orc, kind):
    check_samples(ihip, orc, configs.CFG2, kind, [(0, 0), (0, 3), (0, 7)])


@pytest.mark.parametrize("kind", ["normal", "int"])
def test_cfg3_1m_batch8(ihip, orc, kind):
    print("cfg3", kind, flush=True)
    check_samples(ihip, orc, configs.CFG3, kind, [(0, 0), (3, 5), (7, 7)])
    torch.cuda.empty_cache()


@pytest.mark.parametrize("kind", ["normal", "int"])
def test_cfg4_prefill_4k_on_256k(ihip, orc, kind):
    """Chunked prefill at full size through the fused ihip_prefill_layer call;
    three (KV head, query block) problems are checked against the oracle."""
    w = configs.CFG4
    dev = torch.device("cuda:0")
    q, k, v, sl, _ = configs.make_inputs(w, 0, device=dev, kind=kind)
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    L = ihip.Layer(q, k, sl, w.b_q, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device=dev)
    out = L.prefill_layer(q, k, v, chunks, keeps, out_blocks=blocks)
    torch.cuda.synchronize()
    G = w.G
    for (g, m) in [(0, 0), (3, 31), (7, 63)]:
        print("cfg4", kind, g, m, flush=True)
        p = g * w.Mq + m
        o = orc.Oracle(q[:, g * G:(g + 1) * G].cpu(), k[:, g:g + 1].cpu(), v[:, g:g + 1].cpu(), [w.T],
                       w.b_q, w.n_sink, w.n_stream)
        pr = o.prune(0, 0, m, w.stages)
        got = blocks[p].cpu().numpy()
        got = got[got >= 0]
        want = pr.block_starts
        assert len(got) == len(want) == keeps[-1]
        if kind == "int":
            assert np.array_equal(got, want), (g, m)
        else:
            recall = len(set(got.tolist()) & set(want.tolist())) / len(want)
            assert recall >= 0.99, (g, m, recall)
        ref, _ = o.attend(0, 0, m, pr.block_starts, pr.block_lens)
        err = np.abs(out[0, g * G:(g + 1) * G, m * w.b_q:(m + 1) * w.b_q].float().cpu().numpy() - ref).max()
        assert err <= 2e-2, (g, m, err)


def device_pools(k, v, page, seed):
    """[B,Hkv,T,d] device tensors -> page pools [n_pages,Hkv,page,d] in a seeded random page order + block table."""
    B, Hkv, T, d = k.shape
    per_seq = T // page
    assert per_seq * page == T
    g = torch.Generator(device=k.device)
    g.manual_seed(seed)
    order = torch.randperm(B * per_seq, generator=g, device=k.device).view(B, per_seq)
    k_pool = torch.empty((B * per_seq, Hkv, page, d), dtype=k.dtype, device=k.device)
    v_pool = torch.empty_like(k_pool)
    for b in range(B):
        k_pool[order[b]] = k[b].view(Hkv, per_seq, page, d).permute(1, 0, 2, 3)
        v_pool[order[b]] = v[b].view(Hkv, per_seq, page, d).permute(1, 0, 2, 3)
    return k_pool, v_pool, order.to(torch.int32).contiguous()


def serving_variant(ihip, orc, w, dev):
    """Integer-valued inputs, E4M3 rows with power-of-two scales, 16-token pages in random order, the
    quarter-turn rotary table: every score is exact on both sides."""
    from workloads import gen
    q, k, v, sl, _ = configs.make_inputs(w, 0, device=dev, kind="int")
    scales = (0.5, 0.25)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    del k, v
    k_pool, v_pool, table = device_pools(k8, v8, 16, 7)
    cos, sin = gen.quarter_turn_table(w.n_sink + w.n_stream + w.stages[-1][0] * w.stages[-1][1] + 64, w.d)
    rp = ihip.Rope(cos.to(dev), sin.to(dev), ihip.ROPE_RELATIVE, ihip.ROPE_STREAMING)
    spec = orc.RopeSpec(cos.numpy(), sin.numpy(), prune="relative", attn="streaming")
    return q, k8, v8, sl, scales, ihip.PagedKV(k_pool, v_pool, table), rp, spec


def test_cfg3_decode_full_size_rope_fp8_pages(ihip, orc):
    """The serving configuration (relative RoPE + E4M3 + pages) at the headline size through
    ihip_decode_layer_ex: kept lists of sampled problems bit-exact, outputs within 2e-2."""
    w, dev = configs.CFG3, torch.device("cuda:0")
    q, k8, v8, sl, scales, pg, rp, spec = serving_variant(ihip, orc, w, dev)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    L = ihip.Layer(q, k8, sl, 1, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device=dev)
    out = L.decode_layer(q, None, None, chunks, keeps, out_blocks=blocks, rope=rp, kv_scales=scales, paged=pg)
    torch.cuda.synchronize()
    G = w.G
    for (b, g) in [(0, 0), (5, 6)]:
        print("cfg3 serving", b, g, flush=True)
        o = orc.Oracle(q[b:b + 1, g * G:(g + 1) * G].cpu(), k8[b:b + 1, g:g + 1].cpu(), v8[b:b + 1, g:g + 1].cpu(),
                       [w.T], 1, w.n_sink, w.n_stream, rope=spec, kv_scales=scales)
        pr = o.prune(0, 0, 0, w.stages)
        got = blocks[b * w.Hkv + g].cpu().numpy()
        assert np.array_equal(got[got >= 0], pr.block_starts), (b, g)
        ref, _ = o.attend(0, 0, 0, pr.block_starts, pr.block_lens)
        assert np.abs(out[b, g * G:(g + 1) * G, 0].float().cpu().numpy() - ref[:, 0]).max() <= 2e-2, (b, g)
    # the same rows contiguous (no pages): the large first stage takes the RoPE kernel's three-chunks-per-
    # lane-group variant; same arithmetic, so the same bits
    del pg
    torch.cuda.empty_cache()
    blocks2 = torch.empty_like(blocks)
    out2 = L.decode_layer(q, k8, v8, chunks, keeps, out_blocks=blocks2, rope=rp, kv_scales=scales)
    torch.cuda.synchronize()
    assert torch.equal(blocks2, blocks) and torch.equal(out2, out)
    del k8, v8
    torch.cuda.empty_cache()


def test_cfg4_prefill_full_size_rope_fp8_pages(ihip, orc):
    """The same variants on the full chunked-prefill workload through ihip_prefill_layer_ex."""
    w, dev = configs.CFG4, torch.device("cuda:0")
    q, k8, v8, sl, scales, pg, rp, spec = serving_variant(ihip, orc, w, dev)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    L = ihip.Layer(q, k8, sl, w.b_q, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device=dev)
    out = L.prefill_layer(q, None, None, chunks, keeps, out_blocks=blocks, rope=rp, kv_scales=scales, paged=pg)
    torch.cuda.synchronize()
    G = w.G
    for (g, m) in [(1, 0), (6, 63)]:
        print("cfg4 serving", g, m, flush=True)
        o = orc.Oracle(q[:, g * G:(g + 1) * G].cpu(), k8[:, g:g + 1].cpu(), v8[:, g:g + 1].cpu(), [w.T], w.b_q,
                       w.n_sink, w.n_stream, rope=spec, kv_scales=scales)
        pr = o.prune(0, 0, m, w.stages)
        got = blocks[g * w.Mq + m].cpu().numpy()
        assert np.array_equal(got[got >= 0], pr.block_starts), (g, m)
        ref, _ = o.attend(0, 0, m, pr.block_starts, pr.block_lens)
        err = np.abs(out[0, g * G:(g + 1) * G, m * w.b_q:(m + 1) * w.b_q].float().cpu().numpy() - ref).max()
        assert err <= 2e-2, (g, m, err)
