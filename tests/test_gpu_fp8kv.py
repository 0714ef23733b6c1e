"""GPU parity of the decode path with an FP8 (E4M3) KV cache against the
oracle's FP8 option, through the C ABI.  Integer-valued inputs with
power-of-two scales are exact on both sides; Gaussian inputs quantised to
E4M3 are held to the same recall / tolerance as the bf16 path."""
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


def run_gpu(ihip, w, q, k8, v8, sl, scales):
    qd, kd, vd, sld = [t.cuda() for t in (q, k8, v8, sl)]
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    stages, parents, pchunk = [], None, 0
    for (l_c, keep) in w.stages:
        scores, rep = L.prune_stage(qd, kd, l_c, parents, pchunk, want_rep=True, k_scale=scales[0])
        kept = L.select_blocks(scores, l_c, keep, parents, pchunk)
        stages.append((scores, rep, kept))
        parents, pchunk = kept, l_c
    out, lse = L.sparse_attn_decode(qd, kd, vd, parents, pchunk, want_lse=True, kv_scales=scales)
    fused = L.decode_layer(qd, kd, vd, [s[0] for s in w.stages], [s[1] for s in w.stages], kv_scales=scales)
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


@pytest.mark.parametrize("scales", [(1.0, 1.0), (0.5, 0.25)])
@pytest.mark.parametrize("T,B", [(8192, 1), (4096 + 37, 2)])
def test_integer_inputs_bit_exact(ihip, orc, scales, T, B):
    w = configs.shrink(configs.CFG1, T=T, B=B, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if B == 2:
        sl = torch.tensor([T, T - 1001], dtype=torch.int32)
    # values -2..2 divided by a power-of-two scale are E4M3 numbers: quantisation is lossless
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    assert torch.equal(k8.view(torch.float8_e4m3fn).float() * scales[0], k.float())
    o = orc.Oracle(q, k8, v8, sl.tolist(), 1, w.n_sink, w.n_stream, kv_scales=scales)
    stages, out, lse, fused = run_gpu(ihip, w, q, k8, v8, sl, scales)
    worst, _ = compare(w, o, stages, out, lse, exact=True)
    assert worst <= 2e-2
    assert torch.equal(fused, out)


def test_fp8_result_equals_bf16_kernels_on_dequantised_values(ihip):
    # the byte order inside a row and the scale handling, against the library's own bf16 path
    w = configs.shrink(configs.CFG1, T=4096, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 2)
    scales = (0.0625, 0.125)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    kd = (k8.view(torch.float8_e4m3fn).float() * scales[0]).to(torch.bfloat16)
    vd = (v8.view(torch.float8_e4m3fn).float() * scales[1]).to(torch.bfloat16)
    L = ihip.Layer(q.cuda(), kd.cuda(), sl.cuda(), 1, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    b1 = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
    b2 = torch.empty_like(b1)
    ref = L.decode_layer(q.cuda(), kd.cuda(), vd.cuda(), chunks, keeps, out_blocks=b1)
    got = L.decode_layer(q.cuda(), k8.cuda(), v8.cuda(), chunks, keeps, kv_scales=scales, out_blocks=b2)
    assert torch.equal(b1, b2)
    assert (ref.float() - got.float()).abs().max().item() <= 8e-3      # one bf16 ulp of the output


def test_gaussian_recall_and_output(ihip, orc):
    w = configs.CFG1
    q, k, v, sl, _ = configs.make_inputs(w, 1)
    scales = (1.0 / 64, 1.0 / 64)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    o = orc.Oracle(q, k8, v8, sl.tolist(), 1, w.n_sink, w.n_stream, kv_scales=scales)
    stages, out, lse, fused = run_gpu(ihip, w, q, k8, v8, sl, scales)
    worst, recall = compare(w, o, stages, out, lse, exact=False)
    assert recall >= 0.99
    assert worst <= 2e-2


def test_bad_scale_is_refused(ihip):
    w = configs.shrink(configs.CFG1, T=2048, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    k8 = gen.to_e4m3(k, 1.0).cuda()
    L = ihip.Layer(q.cuda(), k8, sl.cuda(), 1, w.n_sink, w.n_stream)
    with pytest.raises(ihip.IhipError):
        L.prune_stage(q.cuda(), k8, 64, k_scale=0.0)
