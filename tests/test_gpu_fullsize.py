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
    """The headline workload through the fused call bench.py times: all 64 (sequence, KV head) problems
    against the oracle, one sequence's K/V on the host at a time; and the first stage alone through
    ihip_prune_stage (at this size it takes the three-chunks-per-lane-group variant of the kernel):
    scores and representatives of sampled problems element by element."""
    w, dev = configs.CFG3, torch.device("cuda:0")
    q, k, v, sl, pos = configs.make_inputs(w, 0, device=dev, kind=kind)
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    L = ihip.Layer(q, k, sl, 1, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device=dev)
    out = L.decode_layer(q, k, v, chunks, keeps, out_blocks=blocks)
    scores1, rep1 = L.prune_stage(q, k, chunks[0], want_rep=True)
    torch.cuda.synchronize()
    blocks, out = blocks.cpu().numpy(), out.float().cpu().numpy()
    G, l_n = w.G, chunks[-1]
    stage_samples = {(0, 0), (3, 5), (7, 7)}
    for b in range(w.B):
        print("cfg3", kind, "sequence", b, flush=True)
        o = orc.Oracle(q[b:b + 1].cpu(), k[b:b + 1].cpu(), v[b:b + 1].cpu(), [w.T], 1, w.n_sink, w.n_stream)
        for g in range(w.Hkv):
            pr = o.prune(0, g, 0, w.stages)
            got = blocks[b * w.Hkv + g]
            got = got[got >= 0]
            assert (np.diff(got) > 0).all()
            want = pr.block_starts
            if kind == "int":
                assert np.array_equal(got, want), (b, g)
            else:
                recall = len(set(got.tolist()) & set(want.tolist())) / len(want)
                assert recall >= 0.99, (b, g, recall)
                kept = set((got[:, None] + np.arange(l_n)[None]).ravel().tolist())
                assert all(int(x) in kept for x in pos[b, g]), "a planted needle was dropped"
            ref, _ = o.attend(0, g, 0, pr.block_starts, pr.block_lens)
            err = np.abs(out[b, g * G:(g + 1) * G, 0] - ref[:, 0]).max()
            assert err <= 2e-2, (b, g, err)
            assert len(got) == keeps[-1]
            assert got.min() >= w.n_sink and got.max() + l_n <= w.T - w.n_stream
            if (b, g) in stage_samples:
                st = pr.stages[0]
                n = len(st.starts)
                sc = scores1[b * w.Hkv + g].cpu().numpy()
                rp = rep1[b, g * G:(g + 1) * G, 0].cpu().numpy()
                assert np.isneginf(sc[n:]).all() and (rp[:, n:] == -1).all()
                if kind == "int":
                    assert np.array_equal(sc[:n], st.scores), (b, g)
                    assert np.array_equal(rp[:, :n], st.reps), (b, g)
                else:
                    np.testing.assert_allclose(sc[:n], st.scores, rtol=1e-5, atol=1e-4)
                    assert (rp[:, :n] == st.reps).mean() >= 0.999, (b, g)
        del o
    del q, k, v
    torch.cuda.empty_cache()


@pytest.mark.parametrize("kind", ["normal", "int"])
def test_cfg4_prefill_4k_on_256k(ihip, orc, kind):
    """Chunked prefill at full size through the fused ihip_prefill_layer call: all 512 (KV head, query
    block) problems against the oracle, whose problems are dealt to 16 host threads (its C routines run
    outside the interpreter lock; the arithmetic of a problem is untouched)."""
    from concurrent.futures import ThreadPoolExecutor
    w = configs.CFG4
    dev = torch.device("cuda:0")
    q, k, v, sl, _ = configs.make_inputs(w, 0, device=dev, kind=kind)
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    L = ihip.Layer(q, k, sl, w.b_q, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device=dev)
    out = L.prefill_layer(q, k, v, chunks, keeps, out_blocks=blocks)
    torch.cuda.synchronize()
    blocks_h, out_h = blocks.cpu().numpy(), out.float().cpu().numpy()
    G = w.G
    o = orc.Oracle(q.cpu(), k.cpu(), v.cpu(), [w.T], w.b_q, w.n_sink, w.n_stream)

    def one(gm):
        g, m = gm
        pr = o.prune(0, g, m, w.stages)
        got = blocks_h[g * w.Mq + m]
        got = got[got >= 0]
        want = pr.block_starts
        assert len(got) == len(want) == keeps[-1], (g, m)
        if kind == "int":
            assert np.array_equal(got, want), (g, m)
        else:
            recall = len(set(got.tolist()) & set(want.tolist())) / len(want)
            assert recall >= 0.99, (g, m, recall)
        ref, _ = o.attend(0, g, m, pr.block_starts, pr.block_lens)
        err = np.abs(out_h[0, g * G:(g + 1) * G, m * w.b_q:(m + 1) * w.b_q] - ref).max()
        assert err <= 2e-2, (g, m, err)
        return err

    problems = [(g, m) for m in range(w.Mq) for g in range(w.Hkv)]
    with ThreadPoolExecutor(max_workers=16) as pool:
        for i0 in range(0, len(problems), 64):
            errs = list(pool.map(one, problems[i0:i0 + 64]))
            print("cfg4", kind, "problems", i0, "..", i0 + len(errs) - 1, "max err", max(errs), flush=True)


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


# ---- cfg5: 3,145,728 keys in pinned host memory behind the hot-block cache ---------------------------
@pytest.fixture(scope="module")
def cfg5_host_kv(ihip):
    """Integer-valued K and V of the 3M-key layer in pinned host memory (6 + 6 GiB), generated slab by
    slab on the GPU.  KV head 7's slab starts 2.8e9 elements into the tensor."""
    from workloads import gen
    w, dev = configs.CFG5, torch.device("cuda:0")
    shape = (w.B, w.Hkv, w.T, w.d)
    hk = torch.empty(shape, dtype=torch.bfloat16, pin_memory=True)
    hv = torch.empty(shape, dtype=torch.bfloat16, pin_memory=True)
    step_t = 1 << 18
    for tid_, host in ((configs.TID_K, hk), (configs.TID_V, hv)):
        for t_lo in range(0, w.T, step_t):
            t_hi = min(w.T, t_lo + step_t)
            host[:, :, t_lo:t_hi].copy_(gen.small_int_bf16(0, tid_, shape, dev, (0, w.B, 0, w.Hkv, t_lo, t_hi)))
        print("cfg5: host tensor filled", flush=True)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return hk, hv


@pytest.fixture(scope="module")
def cfg5_oracle_calls(orc, cfg5_host_kv):
    """What the oracle computes for the query sets of the test, on the same pinned tensors: per seed,
    per KV head, the kept blocks, the attention output and the 64-token blocks each bank touches."""
    w, bt = configs.CFG5, 64
    hk, hv = cfg5_host_kv
    blocks_per_head = (w.T + bt - 1) // bt
    cache = {}

    def run(seed):
        if seed not in cache:
            q = configs.make_q(w, seed, kind="int")
            o = orc.Oracle(q, hk, hv, [w.T], 1, w.n_sink, w.n_stream)
            per_head, touched = [], [set(), set()]
            for g in range(w.Hkv):
                print("cfg5 oracle: query set", seed, "KV head", g, flush=True)
                pr = o.prune(0, g, 0, w.stages)
                ref, _ = o.attend(0, g, 0, pr.block_starts, pr.block_lens)
                per_head.append((pr.block_starts.copy(), ref[:, 0].copy()))
                base = g * blocks_per_head
                for st in pr.stages:
                    touched[0].update((base + st.touched_pos // bt).tolist())
                touched[1].update((base + o.attended_positions(0, 0, pr.block_starts, pr.block_lens) // bt).tolist())
            cache[seed] = (q, per_head, touched)
        return cache[seed]
    return run


@pytest.mark.parametrize("mask_slots,sa_slots", [(16384, 8192), (300000, 270000)],
                         ids=["banks-512MiB", "banks-beyond-2^31-elements"])
def test_cfg5_3m_host_tier(ihip, orc, cfg5_host_kv, cfg5_oracle_calls, mask_slots, sa_slots):
    """Config 5 at full size through the fused call with K/V behind the host tier, three calls with the
    LRU update in between (the third repeats the first query set, now partly served from the banks):
    kept lists of all 8 KV heads bit-exact against the oracle on the same pinned tensors (head 7's rows
    lie beyond 2^31 elements), outputs within 2e-2, page tables, slot tables and hit/miss counts of both
    banks equal to the LRU simulation fed with the blocks the oracle touches.  The second
    parametrisation makes the banks so large that slot offsets exceed 2^31 elements too."""
    w, bt, dev = configs.CFG5, 64, torch.device("cuda:0")
    hk, hv = cfg5_host_kv
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    assert mask_slots * bt * w.d > 2 ** 31 or mask_slots == 16384
    cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots)
    sim = [orc.LruBank(cache.n_blocks_total, mask_slots), orc.LruBank(cache.n_blocks_total, sa_slots)]
    sl = torch.full((w.B,), w.T, dtype=torch.int32, device=dev)
    kview = torch.empty((w.B, w.Hkv, w.T, 0), dtype=torch.bfloat16, device=dev)     # shape carrier only
    G = w.G
    try:
        for call, seed in enumerate([0, 1, 0]):
            q, per_head, touched = cfg5_oracle_calls(seed)
            qd = q.to(dev)
            L = ihip.Layer(qd, kview, sl, 1, w.n_sink, w.n_stream)
            blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device=dev)
            print("cfg5", mask_slots, "call", call, flush=True)
            out = ihip.decode_layer_cached(L, qd, cache, chunks, keeps, out_blocks=blocks)
            cache.update()
            torch.cuda.synchronize()
            for g in range(w.Hkv):
                want, ref = per_head[g]
                got = blocks[g].cpu().numpy()
                assert np.array_equal(got[got >= 0], want), (call, g)
                err = np.abs(out[0, g * G:(g + 1) * G, 0].float().cpu().numpy() - ref).max()
                assert err <= 2e-2, (call, g, err)
            stats = cache.stats()
            for bank, name in ((0, "mask"), (1, "sa")):
                sim[bank].call(touched[bank])
                assert stats[name]["last_touched"] == sim[bank].last_touched, (call, name)
                assert stats[name]["last_misses"] == sim[bank].last_misses, (call, name)
                assert (stats[name]["hits"], stats[name]["misses"]) == (sim[bank].hits, sim[bank].misses), (call, name)
                pt, sb = cache.tables(bank)
                assert np.array_equal(pt, np.asarray(sim[bank].page_table, np.int32)), (call, name)
                assert np.array_equal(sb, np.asarray(sim[bank].slot_block, np.int32)), (call, name)
        s = cache.stats()
        assert s["mask"]["hits"] > 0 and s["sa"]["hits"] > 0          # the later calls were partly served from the banks
    finally:
        cache.close()
        torch.cuda.empty_cache()
