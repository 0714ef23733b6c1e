"""GPU parity of the chunked-prefill path over an FP8 (E4M3) KV cache against
the oracle's FP8 option, through the C ABI.  Integer-valued inputs with
power-of-two scales (and the quarter-turn rotary table) are exact on both
sides: scores, representatives and kept lists bit for bit.  Gaussian inputs
quantised to E4M3: block recall >= 0.99, outputs within 2e-2."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import configs, gen  # noqa: E402
from test_gpu_prefill import compare, small  # noqa: E402
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


def gpu_prefill_fp8(ihip, w, q, k8, v8, sl, scales, want_rep=True):
    qd, kd, vd, sld = [t.cuda() for t in (q, k8, v8, sl)]
    L = ihip.Layer(qd, kd, sld, w.b_q, w.n_sink, w.n_stream)
    stages, parents, pchunk = [], None, 0
    for (l_c, keep) in w.stages:
        scores, rep = L.prune_stage(qd, kd, l_c, parents, pchunk, want_rep=want_rep, k_scale=scales[0])
        kept = L.select_blocks(scores, l_c, keep, parents, pchunk)
        stages.append((scores, rep, kept))
        parents, pchunk = kept, l_c
    out, lse = L.sparse_attn_prefill(qd, kd, vd, parents, pchunk, want_lse=True, kv_scales=scales)
    blocks = torch.empty_like(parents)
    fused = L.prefill_layer(qd, kd, vd, [s[0] for s in w.stages], [s[1] for s in w.stages], kv_scales=scales,
                            out_blocks=blocks)
    torch.cuda.synchronize()
    assert torch.equal(blocks, parents) and torch.equal(fused, out)
    return stages, out, lse


@pytest.mark.parametrize("scales", [(1.0, 1.0), (0.5, 0.25)])
@pytest.mark.parametrize("w", [
    small(),                                              # Llama shape, 4 query blocks
    small(prefix=2048 + 37, B=2, Hq=8, Hkv=2),            # ragged middle, two sequences
    small(b_q=32, Tq=128, Hq=8, Hkv=2),
    small(b_q=16, Tq=64, Hq=4, Hkv=2, stages=((32, 8), (8, 16), (2, 40))),
    small(Hq=8, Hkv=8, Tq=128),                           # G = 1
    small(Hq=16, Hkv=2, Tq=64),                           # G = 8
], ids=["llama", "ragged-b2", "bq32", "bq16-3stage", "g1", "g8"])
def test_integer_inputs_bit_exact(ihip, orc, w, scales):
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if w.B == 2:
        sl = torch.tensor([w.T, w.T - 517], dtype=torch.int32)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    assert torch.equal(k8.view(torch.float8_e4m3fn).float() * scales[0], k.float())     # lossless here
    o = orc.Oracle(q, k8, v8, sl.tolist(), w.b_q, w.n_sink, w.n_stream, kv_scales=scales)
    stages, out, lse = gpu_prefill_fp8(ihip, w, q, k8, v8, sl, scales)
    worst, _ = compare(w, o, stages, out, lse, exact=True)
    assert worst <= 2e-2


def test_fp8_result_equals_bf16_kernels_on_dequantised_values(ihip):
    # byte order inside a row and the scale handling, against the library's own bf16 path
    w = small(Tq=256, prefix=4096, stages=((64, 16), (16, 32)))
    q, k, v, sl, _ = configs.make_inputs(w, 2)
    scales = (0.0625, 0.125)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    kd = (k8.view(torch.float8_e4m3fn).float() * scales[0]).to(torch.bfloat16)
    vd = (v8.view(torch.float8_e4m3fn).float() * scales[1]).to(torch.bfloat16)
    L = ihip.Layer(q.cuda(), kd.cuda(), sl.cuda(), w.b_q, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    s_ref, r_ref = L.prune_stage(q.cuda(), kd.cuda(), chunks[0], want_rep=True)
    s_got, r_got = L.prune_stage(q.cuda(), k8.cuda(), chunks[0], want_rep=True, k_scale=scales[0])
    assert torch.equal(s_ref, s_got) and torch.equal(r_ref, r_got)
    b1 = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
    b2 = torch.empty_like(b1)
    ref = L.prefill_layer(q.cuda(), kd.cuda(), vd.cuda(), chunks, keeps, out_blocks=b1)
    got = L.prefill_layer(q.cuda(), k8.cuda(), v8.cuda(), chunks, keeps, kv_scales=scales, out_blocks=b2)
    assert torch.equal(b1, b2)
    assert (ref.float() - got.float()).abs().max().item() <= 1.6e-2      # other kernel, other summation order


def test_every_e4m3_byte_is_widened_exactly(ihip):
    # K rows that hold all 254 finite E4M3 bytes (subnormals, both zeros, the largest values): the
    # pruning scores over the bytes must equal, bit for bit, the bf16 kernel's scores over the decoded
    # values -- the widening in the kernels is exact for every byte
    w = small(Tq=128, prefix=4096, stages=((64, 16), (16, 32)))
    q, k, v, sl, _ = configs.make_inputs(w, 2)
    codes = torch.arange(256, dtype=torch.int64)
    codes = codes[(codes & 0x7f) != 0x7f]                               # no NaN
    idx = (torch.arange(k.numel()) * 37 + 11) % codes.numel()            # every byte, in every lane position
    k8 = codes[idx].to(torch.uint8).view(k.shape)
    scale = 2.0 ** -6                                                    # a power of two: products stay exact
    kd = (k8.view(torch.float8_e4m3fn).float() * scale).to(torch.bfloat16)
    assert torch.equal(kd.float(), k8.view(torch.float8_e4m3fn).float() * scale)
    L = ihip.Layer(q.cuda(), kd.cuda(), sl.cuda(), w.b_q, w.n_sink, w.n_stream)
    s_ref, r_ref = L.prune_stage(q.cuda(), kd.cuda(), 64, want_rep=True)
    s_got, r_got = L.prune_stage(q.cuda(), k8.cuda(), 64, want_rep=True, k_scale=scale)
    assert torch.equal(s_ref, s_got) and torch.equal(r_ref, r_got)


@pytest.mark.parametrize("scales", [(1.0 / 64, 1.0 / 64), (0.013, 0.021)])
def test_gaussian_recall_and_output(ihip, orc, scales):
    w = small(Tq=256, prefix=4096, stages=((64, 16), (16, 32)))
    q, k, v, sl, _ = configs.make_inputs(w, 1)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    o = orc.Oracle(q, k8, v8, sl.tolist(), w.b_q, w.n_sink, w.n_stream, kv_scales=scales)
    stages, out, lse = gpu_prefill_fp8(ihip, w, q, k8, v8, sl, scales, want_rep=False)
    worst, recall = compare(w, o, stages, out, lse, exact=False)
    assert recall >= 0.99
    assert worst <= 2e-2


@pytest.mark.parametrize("rope", [None, "relative", "chunk"])
@pytest.mark.parametrize("page", [0, 16])
@pytest.mark.parametrize("w", [small(), small(b_q=16, Tq=64, Hq=4, Hkv=2, stages=((32, 8), (8, 16), (2, 40))),
                               small(Hq=16, Hkv=2, Tq=64), small(b_q=32, Tq=128, Hq=2, Hkv=2)],
                         ids=["llama", "bq16-3stage", "g8", "bq32-g1"])
def test_fp8_with_rope_pages_and_pooling_bit_exact(ihip, orc, w, page, rope):
    """The combined entry point: E4M3 rows with dynamic RoPE, page pools and either pooling rule."""
    scales = (0.5, 2.0)
    q, k, v, sl, _ = configs.make_inputs(w, 3, kind="int")
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    cos, sin = gen.quarter_turn_table(w.T + 64, w.d)
    spec = orc.RopeSpec(cos.numpy(), sin.numpy(), prune=rope, attn="streaming") if rope else None
    rp = None
    if rope:
        style = ihip.ROPE_RELATIVE if rope == "relative" else ihip.ROPE_CHUNK_INDEXED
        rp = ihip.Rope(cos.cuda(), sin.cuda(), style, ihip.ROPE_STREAMING)
    pg = None
    if page:
        k_pool, v_pool, table = scatter_to_pages(k8, v8, page, 11, 7)
        pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    qd, kd, vd = q.cuda(), k8.cuda(), v8.cuda()
    L = ihip.Layer(qd, kd, sl.cuda(), w.b_q, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    o = orc.Oracle(q, k8, v8, sl.tolist(), w.b_q, w.n_sink, w.n_stream, rope=spec, kv_scales=scales)
    for pooling in (None, ihip.POOL_ALL_HEADS):
        blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
        out = L.prefill_layer(qd, kd, vd, chunks, keeps, rope=rp, paged=pg, pooling=pooling, kv_scales=scales,
                              out_blocks=blocks)
        torch.cuda.synchronize()
        for b in range(w.B):
            for m in range(w.Mq):
                prs = o.prune_all_heads(b, m, w.stages) if pooling else [o.prune(b, g, m, w.stages) for g in range(w.Hkv)]
                for g in (0, w.Hkv - 1):
                    p = (b * w.Hkv + g) * w.Mq + m
                    kp = blocks[p].cpu().numpy()
                    assert np.array_equal(kp[kp >= 0], prs[g].block_starts), (pooling, b, g, m)
                    ref, _ = o.attend(b, g, m, prs[g].block_starts, prs[g].block_lens)
                    got = out[b, g * w.G:(g + 1) * w.G, m * w.b_q:(m + 1) * w.b_q].float().cpu().numpy()
                    assert np.abs(got - ref).max() <= 2e-2, (pooling, b, g, m)


@pytest.mark.parametrize("prefix,page", [(3000, 0), (21760, 0), (23000, 0), (10624, 16), (11000, 16)],
                         ids=["32x32-kernel", "32x32-kernel-at-its-limit", "16x16-kernel", "32x32-kernel-paged-at-its-limit",
                              "16x16-kernel-paged"])
def test_keep_everything_is_dense_causal_on_dequantised_values(ihip, prefix, page):
    # nothing pruned -> dense causal attention over scale * decoded bytes (torch, fp64).  The 32x32
    # kernel keeps up to 22,336 key slots in LDS (11,200 with page ids): prefixes 21760 / 10624 give
    # exactly that many, the longer key lists go to the 16x16 kernel.
    keep = (prefix + 256) // 64 + 1
    w = small(Tq=256, prefix=prefix, n_stream=128, Hq=8, Hkv=2, stages=((64, keep), (16, 4 * keep)))
    q, k, v, sl, _ = configs.make_inputs(w, 5)
    scales = (0.017, 0.009)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    pg = None
    if page:
        k_pool, v_pool, table = scatter_to_pages(k8, v8, page, 9, 7)
        pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    L = ihip.Layer(q.cuda(), k8.cuda(), sl.cuda(), w.b_q, w.n_sink, w.n_stream)
    out = L.prefill_layer(q.cuda(), k8.cuda(), v8.cuda(), [s[0] for s in w.stages], [s[1] for s in w.stages],
                          kv_scales=scales, paged=pg)
    torch.cuda.synchronize()
    kd = k8.view(torch.float8_e4m3fn).double() * scales[0]
    vd = v8.view(torch.float8_e4m3fn).double() * scales[1]
    G, T, Tq = w.G, w.T, w.Tq
    mask = torch.arange(T).view(1, -1) <= torch.arange(T - Tq, T).view(-1, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.double(), kd.repeat_interleave(G, 1), vd.repeat_interleave(G, 1), attn_mask=mask)
    assert (out.cpu().double() - ref).abs().max().item() <= 2e-2
