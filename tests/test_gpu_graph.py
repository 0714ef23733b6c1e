"""The layer calls neither allocate nor synchronise, so they can be captured into a HIP graph.
Each graph is replayed several times with new queries written into the captured input buffer and
eager work of the same library in between; every replay must equal the eager call bit for bit."""
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


def replay_against_eager(make_q, q_buf, run, out_buf, n=4):
    """run(): enqueues the layer call reading q_buf and writing out_buf on the current stream."""
    q_buf.copy_(make_q(0))
    run()                                   # warm-up outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for i in range(1, n + 1):
        q = make_q(i)
        q_buf.copy_(q)
        run()                               # eager
        torch.cuda.synchronize()
        want = out_buf.clone()
        out_buf.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_buf, want), i


def test_decode_layer_variants_in_a_graph(ihip):
    w = configs.shrink(configs.CFG1, T=4096 + 37, B=2, n_needles=0)
    _, k, v, _, _ = configs.make_inputs(w, 0)
    sl = torch.tensor([w.T, w.T - 1001], dtype=torch.int32).cuda()
    kd, vd = k.cuda(), v.cuda()
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    q_buf = configs.make_q(w, 0).cuda()
    L = ihip.Layer(q_buf, kd, sl, 1, w.n_sink, w.n_stream)
    ws = L.workspace(ihip.OP_DECODE_LAYER, chunks, keeps)
    out = torch.empty((w.B, w.Hq, 1, w.d), dtype=torch.bfloat16, device="cuda")
    make_q = lambda i: configs.make_q(w, 10 + i).cuda()      # noqa: E731

    replay_against_eager(make_q, q_buf, lambda: L.decode_layer(q_buf, kd, vd, chunks, keeps, ws=ws, out=out), out)

    cos, sin = gen.rope_table(w.T, w.d)
    rp = ihip.Rope(cos.cuda(), sin.cuda(), ihip.ROPE_RELATIVE, ihip.ROPE_STREAMING)
    scales = (1.0 / 32, 1.0 / 32)
    k8, v8 = gen.to_e4m3(k, scales[0]).cuda(), gen.to_e4m3(v, scales[1]).cuda()
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
    replay_against_eager(make_q, q_buf,
                         lambda: L.decode_layer(q_buf, k8, v8, chunks, keeps, ws=ws, out=out, rope=rp,
                                                kv_scales=scales, out_blocks=blocks), out)

    # mask caching: the captured call recomputes the last two stages from the lists the first left
    state = L.mask_state(keeps)
    L.decode_layer(q_buf, kd, vd, chunks, keeps, ws=ws, out=out, stage_starts=state, first_stage=0)
    replay_against_eager(make_q, q_buf,
                         lambda: L.decode_layer(q_buf, kd, vd, chunks, keeps, ws=ws, out=out, stage_starts=state,
                                                first_stage=len(chunks) - 2), out)


def test_prefill_layer_in_a_graph(ihip):
    w = configs.shrink(configs.CFG4, B=1, Hq=8, Hkv=2, T=2048 + 256, Tq=256, b_q=64, n_stream=256,
                       stages=((64, 8), (16, 16)))
    _, k, v, sl, _ = configs.make_inputs(w, 0)
    kd, vd, sld = k.cuda(), v.cuda(), sl.cuda()
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    q_buf = configs.make_q(w, 0).cuda()
    L = ihip.Layer(q_buf, kd, sld, w.b_q, w.n_sink, w.n_stream)
    ws = L.workspace(ihip.OP_PREFILL_LAYER, chunks, keeps)
    out = torch.empty((w.B, w.Hq, w.Tq, w.d), dtype=torch.bfloat16, device="cuda")
    make_q = lambda i: configs.make_q(w, 20 + i).cuda()      # noqa: E731
    replay_against_eager(make_q, q_buf, lambda: L.prefill_layer(q_buf, kd, vd, chunks, keeps, ws=ws, out=out), out)
    cos, sin = gen.rope_table(w.T, w.d)
    rp = ihip.Rope(cos.cuda(), sin.cuda(), ihip.ROPE_CHUNK_INDEXED, ihip.ROPE_STREAMING)
    replay_against_eager(make_q, q_buf,
                         lambda: L.prefill_layer(q_buf, kd, vd, chunks, keeps, ws=ws, out=out, rope=rp), out)
