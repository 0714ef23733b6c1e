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


def test_static_scratch_decode_layer_in_a_graph(ihip):
    """ihip_decode_layer_static is meant for callers that cannot allocate, a captured graph among them."""
    w = configs.shrink(configs.CFG1, T=4096 + 37, B=2, n_needles=0)
    _, k, v, _, _ = configs.make_inputs(w, 0)
    sl = torch.tensor([w.T, w.T - 1001], dtype=torch.int32).cuda()
    kd, vd = k.cuda(), v.cuda()
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    q_buf = configs.make_q(w, 0).cuda()
    L = ihip.Layer(q_buf, kd, sl, 1, w.n_sink, w.n_stream)
    out = torch.empty((w.B, w.Hq, 1, w.d), dtype=torch.bfloat16, device="cuda")
    make_q = lambda i: configs.make_q(w, 30 + i).cuda()      # noqa: E731
    replay_against_eager(make_q, q_buf, lambda: L.decode_layer_static(q_buf, kd, vd, chunks, keeps, out), out)
    # and the replays equal the workspace variant
    ref = L.decode_layer(q_buf, kd, vd, chunks, keeps)
    torch.cuda.synchronize()
    assert torch.equal(ref, out)


def test_host_tier_refuses_a_stream_under_capture(ihip):
    """The host tier's call counter lives on the host (a captured call would replay a frozen stamp), so
    its calls return IHIP_ERR_UNSUPPORTED on a capturing stream and enqueue nothing; the capture itself
    goes on, and the cache works as before afterwards."""
    w = configs.shrink(configs.CFG1, B=1, Hq=4, Hkv=1, T=2048, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    q, k, v, sl, _ = configs.make_inputs(w, 1)
    hk = torch.empty(k.shape, dtype=torch.bfloat16, pin_memory=True).copy_(k)
    hv = torch.empty(v.shape, dtype=torch.bfloat16, pin_memory=True).copy_(v)
    cache = ihip.HostKVCache(hk, hv, 64, 16, 16)
    try:
        qd, kd, vd, sld = q.cuda(), k.cuda(), v.cuda(), sl.cuda()
        L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
        ws = L.workspace(ihip.OP_DECODE_LAYER, chunks, keeps)
        out = torch.zeros((w.B, w.Hq, 1, w.d), dtype=torch.bfloat16, device="cuda")
        ref = L.decode_layer(qd, kd, vd, chunks, keeps)
        torch.cuda.synchronize()
        errors = []
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            out.zero_()
            for call in (lambda: ihip.decode_layer_cached(L, qd, cache, chunks, keeps, ws=ws, out=out),
                         lambda: cache.update()):
                try:
                    call()
                except ihip.IhipError as e:
                    errors.append(str(e))
        assert len(errors) == 2 and all("-4" in e and "graph" in e for e in errors), errors
        g.replay()
        torch.cuda.synchronize()
        assert not out.any()                                  # nothing of the refused calls was captured
        got = ihip.decode_layer_cached(L, qd, cache, chunks, keeps, ws=ws, out=out)
        cache.update()
        torch.cuda.synchronize()
        assert torch.equal(got, ref)
    finally:
        cache.close()
