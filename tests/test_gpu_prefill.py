"""GPU parity of the chunked-prefill path (MFMA pruning scores, MFMA
block-sparse attention) against the CPU oracle, through the C ABI.

Bar as for decode: bit-exact scores / representatives / kept sets on
integer-valued inputs; block recall >= 0.99 and outputs within 2e-2 on
Gaussian inputs.
"""
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


def small(Tq=256, prefix=2048, b_q=64, B=1, Hq=32, Hkv=8, n_stream=256, stages=((64, 8), (16, 16)), **kw):
    return configs.shrink(configs.CFG4, B=B, Hq=Hq, Hkv=Hkv, T=prefix + Tq, Tq=Tq, b_q=b_q,
                          n_stream=n_stream, stages=stages, **kw)


def gpu_prefill(ihip, w, q, k, v, sl, want_rep=True):
    L = ihip.Layer(q, k, sl, w.b_q, w.n_sink, w.n_stream)
    stages, parents, pchunk = [], None, 0
    for (l_c, keep) in w.stages:
        scores, rep = L.prune_stage(q, k, l_c, parents, pchunk, want_rep=want_rep)
        kept = L.select_blocks(scores, l_c, keep, parents, pchunk)
        stages.append((scores, rep, kept))
        parents, pchunk = kept, l_c
    out, lse = L.sparse_attn_prefill(q, k, v, parents, pchunk, want_lse=True)
    torch.cuda.synchronize()
    return L, stages, out, lse


def compare(w, o, stages, out, lse, exact, problems=None):
    G, Mq = w.G, w.Mq
    worst, min_recall = 0.0, 1.0
    if problems is None:
        problems = [(b, g, m) for b in range(w.B) for g in range(w.Hkv) for m in range(Mq)]
    for (b, g, m) in problems:
        p = (b * w.Hkv + g) * Mq + m
        pr = o.prune(b, g, m, w.stages)
        for i, st in enumerate(pr.stages):
            scores, rep, kept = stages[i]
            n = len(st.starts)
            sc = scores[p].cpu().numpy()
            kp = kept[p].cpu().numpy()
            if exact:
                assert np.array_equal(sc[:n], st.scores), (b, g, m, i)
                assert np.isneginf(sc[n:]).all(), (b, g, m, i)
                if rep is not None:
                    rp = rep[b, g * G:(g + 1) * G, m].cpu().numpy()
                    assert np.array_equal(rp[:, :n], st.reps), (b, g, m, i)
                    assert (rp[:, n:] == -1).all()
                ks = st.kept_starts
                assert np.array_equal(kp[:len(ks)], ks), (b, g, m, i)
                assert (kp[len(ks):] == -1).all()
            else:
                np.testing.assert_allclose(sc[:n], st.scores, rtol=1e-5, atol=1e-4)
                want = set(st.kept_starts.tolist())
                got = set(kp[kp >= 0].tolist())
                assert len(got) == len(want)
                min_recall = min(min_recall, len(got & want) / max(1, len(want)))
        if not pr.stages:
            for scores, rep, kept in stages:
                assert (kept[p].cpu().numpy() == -1).all()
        ref, ref_lse = o.attend(b, g, m, pr.block_starts, pr.block_lens)       # [G, b_q, d]
        got = out[b, g * G:(g + 1) * G, m * w.b_q:(m + 1) * w.b_q].float().cpu().numpy()
        worst = max(worst, np.abs(got - ref).max())
        if exact:
            np.testing.assert_allclose(lse[b, g * G:(g + 1) * G, m * w.b_q:(m + 1) * w.b_q].cpu().numpy(),
                                       ref_lse, rtol=2e-5, atol=2e-5)
    return worst, min_recall


def dev(*ts):
    return [t.cuda() for t in ts]


@pytest.mark.parametrize("w", [
    small(),                                              # Llama shape, 4 query blocks
    small(prefix=2048 + 37, B=2, Hq=8, Hkv=2),            # ragged middle, two sequences
    small(b_q=32, Tq=128, Hq=8, Hkv=2),
    small(b_q=16, Tq=64, Hq=4, Hkv=2, stages=((32, 8), (8, 16), (2, 40))),
    small(Hq=8, Hkv=8, Tq=128),                           # G = 1
    small(Hq=16, Hkv=2, Tq=64),                           # G = 8
], ids=["llama", "ragged-b2", "bq32", "bq16-3stage", "g1", "g8"])
def test_integer_inputs_bit_exact(ihip, orc, w):
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if w.B == 2:
        sl = torch.tensor([w.T, w.T - 517], dtype=torch.int32)
    o = orc.Oracle(q, k, v, sl.tolist(), w.b_q, w.n_sink, w.n_stream)
    L, stages, out, lse = gpu_prefill(ihip, w, *dev(q, k, v, sl))
    worst, _ = compare(w, o, stages, out, lse, exact=True)
    assert worst <= 2e-2


@pytest.mark.parametrize("seed", [0, 1])
def test_gaussian_recall_and_output(ihip, orc, seed):
    w = small(Tq=256, prefix=4096, stages=((64, 16), (16, 32)))
    q, k, v, sl, _ = configs.make_inputs(w, seed)
    o = orc.Oracle(q, k, v, sl.tolist(), w.b_q, w.n_sink, w.n_stream)
    L, stages, out, lse = gpu_prefill(ihip, w, *dev(q, k, v, sl), want_rep=False)
    worst, recall = compare(w, o, stages, out, lse, exact=False)
    assert recall >= 0.99
    assert worst <= 2e-2


@pytest.mark.parametrize("prefix", [0, 100, 1000, 26000, 27584, 30000])
def test_keep_everything_is_dense_causal(ihip, orc, prefix):
    # prefix 0: prefill from scratch -- early blocks see only (part of) the sink, causally;
    # prefix 27584: 28,416 key slots, exactly what the 32x32 kernel can keep in LDS (26000: a little less);
    # prefix 30000: more than that -> the 16x16 kernel runs
    keep = max(100, (prefix + 512) // 64 + 1)
    w = small(Tq=512, prefix=prefix, n_stream=128, stages=((64, keep), (16, 4 * keep)))
    q, k, v, sl, _ = configs.make_inputs(w, 5)
    L, stages, out, lse = gpu_prefill(ihip, w, *dev(q, k, v, sl), want_rep=False)
    G, T, Tq = w.G, w.T, w.Tq
    mask = torch.arange(T).view(1, -1) <= torch.arange(T - Tq, T).view(-1, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(G, 1), v.double().repeat_interleave(G, 1), attn_mask=mask)
    assert (out.cpu().double() - ref).abs().max().item() <= 2e-2


@pytest.mark.parametrize("gain", [6.0, 24.0])
def test_softmax_reference_moves(ihip, orc, gain):
    # Keys grow louder along the sequence, so the running softmax reference of the kernel has to
    # move many times (and far: scores reach a few hundred in log2 units at gain 24); everything
    # is kept, so the result is dense causal attention.
    prefix = 3000
    keep = (prefix + 512) // 64 + 1
    w = small(Tq=512, prefix=prefix, n_stream=128, stages=((64, keep), (16, 4 * keep)))
    q, k, v, sl, _ = configs.make_inputs(w, 11)
    ramp = torch.linspace(0.05, 1.0, w.T).view(1, 1, -1, 1) * gain
    k = (k.float() * ramp).to(torch.bfloat16)
    L, stages, out, lse = gpu_prefill(ihip, w, *dev(q, k, v, sl), want_rep=False)
    G, T, Tq = w.G, w.T, w.Tq
    mask = torch.arange(T).view(1, -1) <= torch.arange(T - Tq, T).view(-1, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(G, 1), v.double().repeat_interleave(G, 1), attn_mask=mask)
    assert (out.cpu().double() - ref).abs().max().item() <= 2e-2
    logits = torch.einsum("bhqd,bhkd->bhqk", q.double(), k.double().repeat_interleave(G, 1)) / 128 ** 0.5
    ref_lse = torch.logsumexp(logits.masked_fill(~mask, float("-inf")), -1)
    assert torch.allclose(lse.cpu().double(), ref_lse, rtol=1e-4, atol=1e-3)


def test_attention_alone_on_oracle_indices(ihip, orc):
    w = small(Tq=128, prefix=3000, Hq=8, Hkv=2, stages=((64, 16), (16, 24)))
    q, k, v, sl, _ = configs.make_inputs(w, 3)
    o = orc.Oracle(q, k, v, sl.tolist(), w.b_q, w.n_sink, w.n_stream)
    P = w.Hkv * w.Mq
    starts = np.full((P, w.stages[-1][1]), -1, np.int32)
    refs = {}
    for g in range(w.Hkv):
        for m in range(w.Mq):
            pr = o.prune(0, g, m, w.stages)
            starts[g * w.Mq + m, :len(pr.block_starts)] = pr.block_starts
            refs[(g, m)] = o.attend(0, g, m, pr.block_starts, pr.block_lens)
    qd, kd, vd, sld = dev(q, k, v, sl)
    L = ihip.Layer(qd, kd, sld, w.b_q, w.n_sink, w.n_stream)
    out, lse = L.sparse_attn_prefill(qd, kd, vd, torch.from_numpy(starts).cuda(), w.stages[-1][0], want_lse=True)
    for (g, m), (ref, ref_lse) in refs.items():
        got = out[0, g * w.G:(g + 1) * w.G, m * 64:(m + 1) * 64].float().cpu().numpy()
        # P is rounded to bf16 before the second product: a few 1e-3 on |O| <~ 1
        assert np.abs(got - ref).max() <= 1e-2
        np.testing.assert_allclose(lse[0, g * w.G:(g + 1) * w.G, m * 64:(m + 1) * 64].cpu().numpy(), ref_lse,
                                   rtol=2e-5, atol=2e-5)


def test_rows_two_megabytes_apart_take_the_64_bit_offsets(ihip, orc):
    # K and V rows 2^20 elements apart: row offsets pass 2^31 elements, so the pruning and attention kernels
    # built for 64-bit offsets run (prefill and decode); same values, so the same results as the dense layout
    w = small(Tq=256, prefix=2048, Hq=4, Hkv=1)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    stride = 1 << 20
    qd, sld = q.cuda(), sl.cuda()
    kbuf = torch.empty(w.T * stride, dtype=torch.bfloat16, device="cuda")
    vbuf = torch.empty(w.T * stride, dtype=torch.bfloat16, device="cuda")
    kw = kbuf.as_strided((1, 1, w.T, w.d), (0, 0, stride, 1))
    vw = vbuf.as_strided((1, 1, w.T, w.d), (0, 0, stride, 1))
    kw.copy_(k.cuda())
    vw.copy_(v.cuda())
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    L = ihip.Layer(qd, kw, sld, w.b_q, w.n_sink, w.n_stream)
    b1 = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
    b2 = torch.empty_like(b1)
    got = L.prefill_layer(qd, kw, vw, chunks, keeps, out_blocks=b1)
    ref = L.prefill_layer(qd, k.cuda(), v.cuda(), chunks, keeps, out_blocks=b2)
    torch.cuda.synchronize()
    assert torch.equal(b1, b2) and torch.equal(got, ref)
    o = orc.Oracle(q, k, v, sl.tolist(), w.b_q, w.n_sink, w.n_stream)
    for m in (0, w.Mq - 1):
        pr = o.prune(0, 0, m, w.stages)
        kp = b1[m].cpu().numpy()
        assert np.array_equal(kp[kp >= 0], pr.block_starts)
    # the decode kernels on the same buffers
    qdec = q[:, :, -1:].contiguous().cuda()
    Ld = ihip.Layer(qdec, kw, sld, 1, w.n_sink, w.n_stream)
    d1 = Ld.decode_layer(qdec, kw, vw, chunks, keeps)
    d2 = Ld.decode_layer(qdec, k.cuda(), v.cuda(), chunks, keeps)
    torch.cuda.synchronize()
    assert torch.equal(d1, d2)
    del kbuf, vbuf
    torch.cuda.empty_cache()
