"""GPU parity of the decode layer with several variants at once (dynamic RoPE,
FP8 K/V, paged K/V, all-heads pooling, mask caching) through
ihip_decode_layer_ex, against the CPU oracle.

Integer-valued inputs, the quarter-turn rotary table and power-of-two FP8
scales keep every score an exact integer multiple on both sides: kept block
lists are compared bit for bit, outputs within 2e-2."""
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


def scatter_to_pages(k, v, page, seed, fill, spare=5):
    """[B,Hkv,T,d] -> pools [n_pages,Hkv,page,d] with a seeded random page order + block table."""
    B, Hkv, T, d = k.shape
    per_seq = (T + page - 1) // page
    n_pages = B * per_seq + spare
    order = gen.distinct_ints(seed, 77, B * per_seq, n_pages).view(B, per_seq)
    k_pool = torch.full((n_pages, Hkv, page, d), fill, dtype=k.dtype)      # unused rows hold junk
    v_pool = torch.full((n_pages, Hkv, page, d), fill, dtype=v.dtype)
    pad = per_seq * page - T
    kp = torch.nn.functional.pad(k, (0, 0, 0, pad)).view(B, Hkv, per_seq, page, d)
    vp = torch.nn.functional.pad(v, (0, 0, 0, pad)).view(B, Hkv, per_seq, page, d)
    for b in range(B):
        k_pool[order[b]] = kp[b].permute(1, 0, 2, 3)
        v_pool[order[b]] = vp[b].permute(1, 0, 2, 3)
    return k_pool, v_pool, order.to(torch.int32)


class Case:
    """Inputs of one workload in every representation the variants need."""

    def __init__(self, ihip, orc, w, sl, rope, fp8, paged, prune_style="relative", seed=0):
        self.w = w
        q, k, v, _, _ = configs.make_inputs(w, seed, kind="int")
        self.q, self.sl = q, sl
        self.scales = (0.5, 0.25) if fp8 else None
        if fp8:       # values -2..2 over a power-of-two scale are E4M3 numbers: lossless
            k, v = gen.to_e4m3(k, self.scales[0]), gen.to_e4m3(v, self.scales[1])
        self.k, self.v = k, v
        self.cos, self.sin = gen.quarter_turn_table(w.T, w.d)
        self.rope_spec = orc.RopeSpec(self.cos.numpy(), self.sin.numpy(), prune=prune_style, attn="streaming") \
            if rope else None
        style = {"relative": ihip.ROPE_RELATIVE, "chunk": ihip.ROPE_CHUNK_INDEXED}[prune_style]
        self.rope = ihip.Rope(self.cos.cuda(), self.sin.cuda(), style, ihip.ROPE_STREAMING) if rope else None
        self.kd, self.vd = k.cuda(), v.cuda()
        self.paged = None
        if paged:
            k_pool, v_pool, table = scatter_to_pages(k, v, paged, seed=3, fill=7)
            self.paged = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
        self.chunks = [s[0] for s in w.stages]
        self.keeps = [s[1] for s in w.stages]

    def oracle(self, orc, q=None, sl=None):
        return orc.Oracle(self.q if q is None else q, self.k, self.v, (self.sl if sl is None else sl).tolist(), 1,
                          self.w.n_sink, self.w.n_stream, rope=self.rope_spec, kv_scales=self.scales)

    def layer_kwargs(self):
        return dict(rope=self.rope, kv_scales=self.scales, paged=self.paged)


COMBOS = [
    dict(rope=True, fp8=True, paged=0),
    dict(rope=True, fp8=False, paged=16),
    dict(rope=False, fp8=True, paged=16),
    dict(rope=True, fp8=True, paged=64),
    dict(rope=True, fp8=True, paged=16, prune_style="chunk"),
]


@pytest.mark.parametrize("combo", COMBOS, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
@pytest.mark.parametrize("T,B", [(8192, 1), (4096 + 37, 2)])
def test_combined_variants_match_the_oracle(ihip, orc, combo, T, B):
    w = configs.shrink(configs.CFG1, T=T, B=B, n_needles=0)
    sl = torch.tensor([T, T - 1001][:B], dtype=torch.int32)
    c = Case(ihip, orc, w, sl, **combo)
    qd, sld = c.q.cuda(), sl.cuda()
    L = ihip.Layer(qd, c.kd, sld, 1, w.n_sink, w.n_stream)
    P = w.B * w.Hkv
    blocks = torch.empty((P, c.keeps[-1]), dtype=torch.int32, device="cuda")
    out = L.decode_layer(qd, c.kd, c.vd, c.chunks, c.keeps, out_blocks=blocks, **c.layer_kwargs())
    torch.cuda.synchronize()
    o = c.oracle(orc)
    for b in range(B):
        for g in range(w.Hkv):
            pr = o.prune(b, g, 0, w.stages)
            kp = blocks[b * w.Hkv + g].cpu().numpy()
            assert np.array_equal(kp[kp >= 0], pr.block_starts), (b, g)
            ref, _ = o.attend(b, g, 0, pr.block_starts, pr.block_lens)
            got = out[b, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy()
            assert np.abs(got - ref[:, 0]).max() <= 2e-2, (b, g)


def test_all_heads_pooling_with_rope_and_pages(ihip, orc):
    w = configs.shrink(configs.CFG1, T=4096, n_needles=0)
    sl = torch.tensor([4096], dtype=torch.int32)
    c = Case(ihip, orc, w, sl, rope=True, fp8=False, paged=16)
    qd = c.q.cuda()
    L = ihip.Layer(qd, c.kd, sl.cuda(), 1, w.n_sink, w.n_stream)
    blocks = torch.empty((w.Hkv, c.keeps[-1]), dtype=torch.int32, device="cuda")
    out = L.decode_layer(qd, None, None, c.chunks, c.keeps, out_blocks=blocks, pooling=ihip.POOL_ALL_HEADS,
                         **c.layer_kwargs())
    torch.cuda.synchronize()
    o = c.oracle(orc)
    prs = o.prune_all_heads(0, 0, w.stages)
    for g in range(w.Hkv):
        kp = blocks[g].cpu().numpy()
        assert np.array_equal(kp[kp >= 0], prs[g].block_starts), g
        ref, _ = o.attend(0, g, 0, prs[g].block_starts, prs[g].block_lens)
        got = out[0, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy()
        assert np.abs(got - ref[:, 0]).max() <= 2e-2


@pytest.mark.parametrize("combo", [dict(rope=True, fp8=False, paged=0), dict(rope=True, fp8=True, paged=16)],
                         ids=["rope", "rope-fp8-paged"])
def test_mask_caching_with_variants_follows_oracle(ihip, orc, combo):
    # Alg. 4's refresh schedule on top of the variants: sequences grow, queries change every step
    refresh = (4, 2, 1)
    w = configs.shrink(configs.CFG1, B=2, Hq=8, Hkv=2, T=3000, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    lens0 = [2900, 2200]
    c = Case(ihip, orc, w, torch.tensor(lens0, dtype=torch.int32), **combo)
    state = None
    cached = {(b, g): [np.zeros(0, np.int64)] * 3 for b in range(w.B) for g in range(w.Hkv)}
    P = w.B * w.Hkv
    for step in range(9):
        sl = torch.tensor([lens0[0] + step, lens0[1] + 3 * step], dtype=torch.int32)
        q = configs.make_q(w, 100 + step, kind="int")
        qd, sld = q.cuda(), sl.cuda()
        L = ihip.Layer(qd, c.kd, sld, 1, w.n_sink, w.n_stream)
        if state is None:
            state = L.mask_state(c.keeps)
        first = ihip.first_stage_due(step, refresh)
        out = L.decode_layer(qd, c.kd, c.vd, c.chunks, c.keeps, stage_starts=state, first_stage=first,
                             **c.layer_kwargs())
        torch.cuda.synchronize()
        o = c.oracle(orc, q=q, sl=sl)
        off, st_gpu = 0, []
        for keep in c.keeps:
            st_gpu.append(state[off:off + P * keep].view(P, keep).cpu().numpy())
            off += P * keep
        for b in range(w.B):
            for g in range(w.Hkv):
                kept, bs, bl = o.prune_from(b, g, 0, w.stages, first, cached[(b, g)])
                cached[(b, g)] = kept
                p = b * w.Hkv + g
                for i in range(3):
                    got = st_gpu[i][p]
                    assert got[got >= 0].tolist() == kept[i].tolist(), (step, b, g, i)
                ref, _ = o.attend(b, g, 0, bs, bl)
                err = np.abs(out[b, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy() - ref[:, 0]).max()
                assert err <= 2e-2, (step, b, g, err)


@pytest.mark.parametrize("T", [2048, 4096 + 37])
def test_keep_everything_with_all_variants_is_rotary_attention(ihip, T):
    # Every chunk kept: the decode layer with streaming RoPE over FP8 pages must be ordinary rotary
    # attention of the last token over the dequantised K and V (torch, fp64; no oracle involved).
    w = configs.shrink(configs.CFG1, T=T, B=2, n_needles=0)
    n1 = (T - w.n_sink - w.n_stream + 63) // 64
    stages = ((64, n1), (16, 4 * n1), (4, 16 * n1))
    q, k, v, _, _ = configs.make_inputs(w, 4)
    sl = torch.tensor([T, T - 300], dtype=torch.int32)
    scales = (1.0 / 32, 1.0 / 16)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    kf = k8.view(torch.float8_e4m3fn).double() * scales[0]
    vf = v8.view(torch.float8_e4m3fn).double() * scales[1]
    cos, sin = gen.rope_table(T + 64, w.d)
    k_pool, v_pool, table = scatter_to_pages(k8, v8, 16, seed=11, fill=3)
    pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    rp = ihip.Rope(cos.cuda(), sin.cuda(), ihip.ROPE_RELATIVE, ihip.ROPE_STREAMING)
    qd = q.cuda()
    L = ihip.Layer(qd, k8.cuda(), sl.cuda(), 1, w.n_sink, w.n_stream)
    out = L.decode_layer(qd, None, None, [s[0] for s in stages], [s[1] for s in stages], rope=rp, kv_scales=scales,
                         paged=pg)
    torch.cuda.synchronize()
    G, d = w.G, w.d
    for b in range(w.B):
        n = int(sl[b])
        pos = torch.arange(n)
        c, s_ = cos[pos].double(), sin[pos].double()
        ke, ko = kf[b, :, :n, 0::2], kf[b, :, :n, 1::2]
        kr = torch.empty((w.Hkv, n, d), dtype=torch.float64)
        kr[..., 0::2], kr[..., 1::2] = ke * c - ko * s_, ke * s_ + ko * c
        qe, qo = q[b, :, 0, 0::2].double(), q[b, :, 0, 1::2].double()
        qr = torch.empty((w.Hq, d), dtype=torch.float64)
        qr[:, 0::2] = qe * c[n - 1] - qo * s_[n - 1]
        qr[:, 1::2] = qe * s_[n - 1] + qo * c[n - 1]
        logits = torch.einsum("hd,hnd->hn", qr, kr.repeat_interleave(G, 0)) / d ** 0.5
        ref = torch.einsum("hn,hnd->hd", torch.softmax(logits, -1), vf[b, :, :n].repeat_interleave(G, 0))
        assert (out[b, :, 0].cpu().double() - ref).abs().max().item() <= 2e-2, b
