"""GPU parity of the decode path against the CPU oracle, through the C ABI.

Bar: selected index sets, representatives and scores bit-exact on
integer-valued inputs (fp32 dot products are exact in any order); on Gaussian
inputs block recall >= 0.99 per problem and outputs within 2e-2 max-abs.
"""
import ctypes
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from workloads import configs, gen  # noqa: E402


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


@pytest.fixture(scope="module")
def ihip():
    _need_gpu()
    import paper_2502_08910_amd as pkg
    pkg.lib()                       # raises if the HIP library is not built
    return pkg


@pytest.fixture(scope="module")
def orc():
    import oracle
    oracle.build(force=False)
    return oracle


def gpu_stagewise(ihip, w, q, k, v, seq_lens, want_rep=True):
    """Runs stage by stage through the separate entry points."""
    L = ihip.Layer(q, k, seq_lens, w.b_q, w.n_sink, w.n_stream)
    stages, parents, pchunk = [], None, 0
    for (l_c, keep) in w.stages:
        scores, rep = L.prune_stage(q, k, l_c, parents, pchunk, want_rep=want_rep)
        kept = L.select_blocks(scores, l_c, keep, parents, pchunk)
        stages.append((scores, rep, kept))
        parents, pchunk = kept, l_c
    out, lse = L.sparse_attn_decode(q, k, v, parents, pchunk, want_lse=True)
    torch.cuda.synchronize()
    return L, stages, out, lse


def compare_stagewise(w, o, stages, out, lse, exact, problems=None):
    """Element-by-element comparison with the oracle, problem by problem."""
    G = w.G
    worst, min_recall = 0.0, 1.0
    if problems is None:
        problems = [(b, g) for b in range(w.B) for g in range(w.Hkv)]
    for (b, g) in problems:
        p = b * w.Hkv + g
        pr = o.prune(b, g, 0, w.stages)
        for i, st in enumerate(pr.stages):
            scores, rep, kept = stages[i]
            n = len(st.starts)
            sc = scores[p].cpu().numpy()
            kp = kept[p].cpu().numpy()
            if exact:
                assert np.array_equal(sc[:n], st.scores), (b, g, i)
                assert np.isneginf(sc[n:]).all()
                if rep is not None:
                    rp = rep[b, g * G:(g + 1) * G, 0].cpu().numpy()
                    assert np.array_equal(rp[:, :n], st.reps), (b, g, i)
                    assert (rp[:, n:] == -1).all()
                ks = st.kept_starts
                assert np.array_equal(kp[:len(ks)], ks), (b, g, i)
                assert (kp[len(ks):] == -1).all()
            else:
                np.testing.assert_allclose(sc[:n], st.scores, rtol=1e-5, atol=1e-4)
                want = set(st.kept_starts.tolist())
                got = set(kp[kp >= 0].tolist())
                assert len(got) == len(want)
                min_recall = min(min_recall, len(got & want) / max(1, len(want)))
                assert (np.diff(kp[kp >= 0]) > 0).all()
        # attention over the oracle's own final blocks
        ref, ref_lse = o.attend(b, g, 0, pr.block_starts, pr.block_lens)
        got = out[b, g * G:(g + 1) * G, 0].float().cpu().numpy()
        worst = max(worst, np.abs(got - ref[:, 0]).max())
        if exact:
            np.testing.assert_allclose(lse[b, g * G:(g + 1) * G, 0].cpu().numpy(), ref_lse[:, 0],
                                       rtol=1e-5, atol=1e-5)
    return worst, min_recall


def dev(*ts):
    return [t.cuda() for t in ts]


# ---------------------------------------------------------------------------
@pytest.mark.parametrize("T,B", [(8192, 1), (8192 + 37, 2), (1500, 1)])
def test_integer_inputs_bit_exact(ihip, orc, T, B):
    w = configs.shrink(configs.CFG1, T=T, B=B, n_needles=0)
    q, k, v, sl, _ = configs.make_inputs(w, 0, kind="int")
    if B == 2:
        sl = torch.tensor([T, T - 1001], dtype=torch.int32)
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
    L, stages, out, lse = gpu_stagewise(ihip, w, *dev(q, k, v, sl))
    worst, _ = compare_stagewise(w, o, stages, out, lse, exact=True)
    assert worst <= 2e-2


@pytest.mark.parametrize("seed", [0, 1])
def test_gaussian_cfg1_recall_and_output(ihip, orc, seed):
    w = configs.CFG1
    q, k, v, sl, pos = configs.make_inputs(w, seed)
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
    L, stages, out, lse = gpu_stagewise(ihip, w, *dev(q, k, v, sl))
    # attention checked in isolation on the oracle's indices as well
    worst, recall = compare_stagewise(w, o, stages, out, lse, exact=False)
    assert recall >= 0.99
    assert worst <= 2e-2
    # needles survive on the GPU too
    final = stages[-1][2].cpu().numpy()
    l_n = w.stages[-1][0]
    for g in range(w.Hkv):
        kept = set((final[g][:, None] + np.arange(l_n)[None]).ravel().tolist())
        assert all(int(x) in kept for x in pos[0, g])


def test_attention_alone_on_oracle_indices(ihip, orc):
    w = configs.CFG1
    q, k, v, sl, _ = configs.make_inputs(w, 3)
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
    starts = np.full((w.Hkv, w.stages[-1][1]), -1, np.int32)
    refs = []
    for g in range(w.Hkv):
        pr = o.prune(0, g, 0, w.stages)
        starts[g, :len(pr.block_starts)] = pr.block_starts
        refs.append(o.attend(0, g, 0, pr.block_starts, pr.block_lens))
    qd, kd, vd, sld = dev(q, k, v, sl)
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    out, lse = L.sparse_attn_decode(qd, kd, vd, torch.from_numpy(starts).cuda(), w.stages[-1][0], want_lse=True)
    for g in range(w.Hkv):
        got = out[0, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy()
        assert np.abs(got - refs[g][0][:, 0]).max() <= 4e-3
        np.testing.assert_allclose(lse[0, g * w.G:(g + 1) * w.G, 0].cpu().numpy(), refs[g][1][:, 0],
                                   rtol=2e-5, atol=2e-5)


@pytest.mark.parametrize("T", [1, 5, 128, 129, 700, 1152, 1153, 1300])
def test_short_sequences(ihip, orc, T):
    # shorter than the sink, inside the window, a middle range of one ragged chunk, ...
    w = configs.shrink(configs.CFG1, T=max(T, 8), n_needles=0, stages=((64, 4), (16, 8), (4, 16)))
    q, k, v, _, _ = configs.make_inputs(w, 2, kind="int")
    sl = torch.tensor([T], dtype=torch.int32)
    o = orc.Oracle(q, k, v, [T], 1, w.n_sink, w.n_stream)
    L, stages, out, lse = gpu_stagewise(ihip, w, *dev(q, k, v, sl))
    worst, _ = compare_stagewise(w, o, stages, out, lse, exact=True)
    assert worst <= 2e-2


def test_keep_everything_is_dense(ihip, orc):
    w = configs.shrink(configs.CFG1, T=2048 + 5, n_stream=256, n_needles=0,
                       stages=((64, 1000), (16, 4000), (4, 16000)))
    q, k, v, sl, _ = configs.make_inputs(w, 5)
    qd, kd, vd, sld = dev(q, k, v, sl)
    L, stages, out, lse = gpu_stagewise(ihip, w, qd, kd, vd, sld, want_rep=False)
    G = w.G
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(G, 1), v.double().repeat_interleave(G, 1))
    assert (out.cpu().double() - ref).abs().max().item() <= 2e-2


def test_fused_entry_points_equal_stagewise(ihip, orc):
    w = configs.shrink(configs.CFG1, B=2, T=4096 + 11)
    q, k, v, sl, _ = configs.make_inputs(w, 4)
    sl = torch.tensor([w.T, w.T - 333], dtype=torch.int32)
    qd, kd, vd, sld = dev(q, k, v, sl)
    L, stages, out, lse = gpu_stagewise(ihip, w, qd, kd, vd, sld, want_rep=False)
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    blocks = L.prune_all(qd, kd, chunks, keeps)
    assert torch.equal(blocks, stages[-1][2])
    blocks2 = torch.empty_like(blocks)
    out2 = L.decode_layer(qd, kd, vd, chunks, keeps, out_blocks=blocks2)
    torch.cuda.synchronize()
    assert torch.equal(blocks2, blocks)
    assert torch.equal(out2, out)
    # twice the same: deterministic
    out3 = L.decode_layer(qd, kd, vd, chunks, keeps)
    assert torch.equal(out3, out)


def test_strided_kv_layout(ihip, orc):
    # token-major storage [B,T,Hkv,d] viewed as [B,Hkv,T,d]
    w = configs.shrink(configs.CFG1, T=2048, n_stream=256, n_needles=0, stages=((64, 8), (16, 8), (4, 16)))
    q, k, v, sl, _ = configs.make_inputs(w, 6, kind="int")
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
    kd = k.cuda().permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    vd = v.cuda().permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert not kd.is_contiguous()
    L, stages, out, lse = gpu_stagewise(ihip, w, q.cuda(), kd, vd, sl.cuda())
    worst, _ = compare_stagewise(w, o, stages, out, lse, exact=True)
    assert worst <= 2e-2


def select_case(ihip, orc, P, n, keep, ties):
    rng = np.random.default_rng(n + keep + P)
    chunk, n_sink, n_stream = 4, 8, 16
    s = rng.standard_normal((P, n)).astype(np.float32)
    if ties:
        s = np.round(s * 2) / 2
        s[:, ::7] = -0.0
        s[:, 3::7] = 0.0
    n_valid = [(n, max(1, n - 5), max(1, n // 2))[p % 3] for p in range(P)]
    T = n_sink + n * chunk + n_stream
    seq = []
    for p in range(P):
        s[p, n_valid[p]:] = -np.inf
        seq.append(n_sink + n_valid[p] * chunk - (1 if n_valid[p] > 1 else 0) + n_stream)   # last chunk ragged
    q = torch.zeros((P, 1, 1, 128), dtype=torch.bfloat16).cuda()
    k = torch.zeros((1, 1, T, 128), dtype=torch.bfloat16).cuda().expand(P, 1, T, 128)      # never read
    L = ihip.Layer(q, k, torch.tensor(seq, dtype=torch.int32).cuda(), 1, n_sink, n_stream)
    got = L.select_blocks(torch.from_numpy(s).cuda(), chunk, keep).cpu().numpy()
    lib = orc.lib()
    for p in range(P):
        ids = np.empty(max(1, min(keep, n)), np.int32)
        cnt = lib.orc_topk(n_valid[p], s[p].ctypes.data_as(ctypes.c_void_p), keep,
                           ids.ctypes.data_as(ctypes.c_void_p))
        want = n_sink + ids[:cnt].astype(np.int64) * chunk
        assert np.array_equal(got[p, :cnt], want), p
        assert (got[p, cnt:] == -1).all()


@pytest.mark.parametrize("n,keep,ties", [(1, 1, False), (110, 64, False), (257, 64, True), (1000, 1000, True),
                                         (50, 80, True), (1500, 300, False), (2048, 512, True),
                                         (4092, 256, False), (4092, 256, True),
                                         (4143, 256, False), (6000, 2500, True), (8192, 300, True),
                                         (12288, 300, True), (20000, 777, True), (300, 1, True)])
def test_select_blocks_alone(ihip, orc, n, keep, ties):
    """Three problems: every workgroup shape of the selection that few problems get (4 slots per thread in
    256, 512 or 1024 threads, then 8 and 16 in 1024), the radix fallback beyond, heavy ties."""
    select_case(ihip, orc, 3, n, keep, ties)


@pytest.mark.parametrize("n,keep,ties", [(900, 100, False), (1500, 300, True), (3000, 256, False), (6000, 700, True),
                                         (12000, 300, False), (20000, 500, True)])
def test_select_blocks_many_problems(ihip, orc, n, keep, ties):
    """More problems than CUs: the smallest workgroup that holds the slots (256 threads with 4, 8 or 16
    slots each, 512 and 1024 threads with 16), and the radix select beyond."""
    select_case(ihip, orc, 260, n, keep, ties)


def test_decode_layer_under_graph_capture(ihip, orc):
    """The fused layer call allocates nothing and never synchronises, so it can be captured into a
    HIP graph; every replay (with eager work in between, new queries written in place) must give
    the eager result."""
    w = configs.shrink(configs.CFG1, B=2, T=4096 + 7)
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    q, k, v, sl, _ = configs.make_inputs(w, 7)
    qd, kd, vd, sld = dev(q, k, v, sl)
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    ws = L.workspace(ihip.OP_DECODE_LAYER, chunks, keeps)
    out = torch.empty((w.B, w.Hq, 1, w.d), dtype=torch.bfloat16, device="cuda")
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside capture
        L.decode_layer(qd, kd, vd, chunks, keeps, ws=ws, out=out, out_blocks=blocks)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        L.decode_layer(qd, kd, vd, chunks, keeps, ws=ws, out=out, out_blocks=blocks)
    for seed in (11, 12, 13):
        qn = configs.make_q(w, seed).cuda()
        ref_blocks = torch.empty_like(blocks)
        ref = L.decode_layer(qn, kd, vd, chunks, keeps, out_blocks=ref_blocks)     # eager, own buffers
        qd.copy_(qn)                                    # new input written in place
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(blocks, ref_blocks), seed
        assert torch.equal(out, ref), seed


def test_empty_batch_is_a_no_op(ihip):
    # B = 0: every entry point returns without enqueuing anything or touching a pointer
    w = configs.shrink(configs.CFG1, T=2048, n_needles=0)
    q = torch.empty((0, w.Hq, 1, w.d), dtype=torch.bfloat16, device="cuda")
    k = torch.empty((0, w.Hkv, w.T, w.d), dtype=torch.bfloat16, device="cuda")
    sl = torch.empty((0,), dtype=torch.int32, device="cuda")
    L = ihip.Layer(q, k, sl, 1, w.n_sink, w.n_stream)
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    scores, _ = L.prune_stage(q, k, chunks[0])
    assert scores.shape[0] == 0
    kept = L.select_blocks(scores, chunks[0], keeps[0])
    assert kept.shape == (0, keeps[0])
    out = L.decode_layer(q, k, k, chunks, keeps)
    assert out.shape == (0, w.Hq, 1, w.d)
    Lp = ihip.Layer(torch.empty((0, w.Hq, 64, w.d), dtype=torch.bfloat16, device="cuda"), k, sl, 64, w.n_sink, 1024)
    outp = Lp.prefill_layer(torch.empty((0, w.Hq, 64, w.d), dtype=torch.bfloat16, device="cuda"), k, k, chunks, keeps)
    torch.cuda.synchronize()
    assert outp.shape == (0, w.Hq, 64, w.d)
