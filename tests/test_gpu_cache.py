"""Host-memory KV tier + on-GPU hot-block cache: outputs are bit-identical to
the HBM-resident path whatever the cache holds, and the page tables, slot
tables and hit/miss counts follow the CPU simulation of the LRU policy
exactly (integer-valued inputs, so both sides touch the same rows)."""
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


def touched_blocks(o, w, stages_res, bt, blocks_per_head, bank):
    """Global block ids the oracle touches in one layer call: bank 0 = pruning
    stages (keys), bank 1 = attention (keys and values)."""
    out = set()
    for (b, g, m), (pr, _, _) in stages_res.items():
        base = (b * w.Hkv + g) * blocks_per_head
        if bank == 0:
            for st in pr.stages:
                out.update((base + st.touched_pos // bt).tolist())
        else:
            pos = o.attended_positions(b, m, pr.block_starts, pr.block_lens)
            out.update((base + pos // bt).tolist())
    return out


@pytest.mark.parametrize("mask_slots,sa_slots", [(40, 24), (1000, 1000), (3, 2)])
def test_cached_layer_equals_resident_and_follows_lru(ihip, orc, mask_slots, sa_slots):
    w = configs.shrink(configs.CFG1, B=2, Hq=8, Hkv=2, T=4096 + 29, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    bt = 64
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    _, k, v, _, _ = configs.make_inputs(w, 0, kind="int")
    sl = torch.tensor([w.T, w.T - 700], dtype=torch.int32)
    hk = torch.empty(k.shape, dtype=torch.bfloat16, pin_memory=True).copy_(k)
    hv = torch.empty(v.shape, dtype=torch.bfloat16, pin_memory=True).copy_(v)
    kd, vd, sld = k.cuda(), v.cuda(), sl.cuda()
    cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots)
    blocks_per_head = (w.T + bt - 1) // bt
    sim = [orc.LruBank(cache.n_blocks_total, mask_slots), orc.LruBank(cache.n_blocks_total, sa_slots)]
    try:
        for call, seed in enumerate([0, 1, 0, 2, 1, 0, 3]):
            q = configs.make_q(w, seed, kind="int")
            qd = q.cuda()
            L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
            ref_blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
            ref = L.decode_layer(qd, kd, vd, chunks, keeps, out_blocks=ref_blocks)
            got_blocks = torch.empty_like(ref_blocks)
            got = ihip.decode_layer_cached(L, qd, cache, chunks, keeps, out_blocks=got_blocks)
            cache.update()
            torch.cuda.synchronize()
            assert torch.equal(got_blocks, ref_blocks), call
            assert torch.equal(got, ref), call          # bit-identical whatever the cache holds

            o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
            res = o.layer(w.stages)
            stats = cache.stats()
            for bank, name in ((0, "mask"), (1, "sa")):
                sim[bank].call(touched_blocks(o, w, res, bt, blocks_per_head, bank))
                pt, sb = cache.tables(bank)
                assert stats[name]["last_touched"] == sim[bank].last_touched, (call, name)
                assert stats[name]["last_misses"] == sim[bank].last_misses, (call, name)
                assert (stats[name]["hits"], stats[name]["misses"]) == (sim[bank].hits, sim[bank].misses)
                assert pt.tolist() == sim[bank].page_table, (call, name)
                assert sb.tolist() == sim[bank].slot_block, (call, name)
        # a reset empties it again
        cache.reset()
        pt, sb = cache.tables(0)
        assert (pt == -1).all() and (sb == -1).all()
    finally:
        cache.close()


def test_bank_contents_are_the_host_rows(ihip, orc):
    # after warming, a layer call served from the banks gives the same bits (checked above);
    # here: everything resident => second call has no misses at all
    w = configs.shrink(configs.CFG1, B=1, Hq=4, Hkv=1, T=2048, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    q, k, v, sl, _ = configs.make_inputs(w, 1)
    hk = torch.empty(k.shape, dtype=torch.bfloat16, pin_memory=True).copy_(k)
    hv = torch.empty(v.shape, dtype=torch.bfloat16, pin_memory=True).copy_(v)
    cache = ihip.HostKVCache(hk, hv, 64, 32, 32)          # 32 blocks = the whole sequence
    try:
        qd, kd, vd, sld = q.cuda(), k.cuda(), v.cuda(), sl.cuda()
        L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
        ref = L.decode_layer(qd, kd, vd, chunks, keeps)
        for call in range(2):
            got = ihip.decode_layer_cached(L, qd, cache, chunks, keeps)
            cache.update()
            assert torch.equal(got, ref)
        s = cache.stats()
        assert s["mask"]["last_misses"] == 0 and s["sa"]["last_misses"] == 0
        assert s["mask"]["last_touched"] > 0 and s["sa"]["last_touched"] > 0
    finally:
        cache.close()


@pytest.mark.parametrize("pooling", [None, "all_heads"])
def test_host_tier_with_mask_caching_equals_resident(ihip, pooling):
    # Alg. 4's refresh schedule on top of the host tier (one options struct): bit-identical to the
    # same schedule on resident K/V, and a step that reuses every cached list does not touch the
    # key bank of the pruning stages at all.
    w = configs.shrink(configs.CFG1, B=2, Hq=8, Hkv=2, T=3000, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    refresh = (4, 2, 2)
    pool = None if pooling is None else ihip.POOL_ALL_HEADS
    _, k, v, _, _ = configs.make_inputs(w, 0, kind="int")
    hk = torch.empty(k.shape, dtype=torch.bfloat16, pin_memory=True).copy_(k)
    hv = torch.empty(v.shape, dtype=torch.bfloat16, pin_memory=True).copy_(v)
    kd, vd = k.cuda(), v.cuda()
    cache = ihip.HostKVCache(hk, hv, 64, 24, 16)
    try:
        state_c = state_r = None
        for step in range(9):
            sl = torch.tensor([2900 + step, 2200 + 3 * step], dtype=torch.int32).cuda()
            qd = configs.make_q(w, 200 + step, kind="int").cuda()
            L = ihip.Layer(qd, kd, sl, 1, w.n_sink, w.n_stream)
            if state_c is None:
                state_c, state_r = L.mask_state(keeps), L.mask_state(keeps)
            first = ihip.first_stage_due(step, refresh)
            got = L.decode_layer(qd, None, None, chunks, keeps, cache=cache, stage_starts=state_c,
                                 first_stage=first, pooling=pool)
            cache.update()
            ref = L.decode_layer(qd, kd, vd, chunks, keeps, stage_starts=state_r, first_stage=first,
                                 pooling=pool if pool is not None else ihip.POOL_KV_HEAD)
            torch.cuda.synchronize()
            assert torch.equal(state_c, state_r), step
            assert torch.equal(got, ref), step
            s = cache.stats()
            if first == len(chunks):
                assert s["mask"]["last_touched"] == 0, step
            else:
                assert s["mask"]["last_touched"] > 0, step
            assert s["sa"]["last_touched"] > 0, step
    finally:
        cache.close()


@pytest.mark.parametrize("style", ["relative", "chunk"])
def test_host_tier_with_dynamic_rope(ihip, orc, style):
    # Dynamic RoPE over K/V behind the host tier: same bits as the resident RoPE path whatever the
    # banks hold, and the banks follow the blocks the oracle (run with the same RoPE) touches.
    from workloads import gen
    w = configs.shrink(configs.CFG1, B=2, Hq=8, Hkv=2, T=4096 + 29, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    bt, mask_slots, sa_slots = 64, 40, 24
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    _, k, v, _, _ = configs.make_inputs(w, 0, kind="int")
    sl = torch.tensor([w.T, w.T - 700], dtype=torch.int32)
    cos, sin = gen.quarter_turn_table(w.T, w.d)
    rp = ihip.Rope(cos.cuda(), sin.cuda(), {"relative": ihip.ROPE_RELATIVE, "chunk": ihip.ROPE_CHUNK_INDEXED}[style],
                   ihip.ROPE_STREAMING)
    spec = orc.RopeSpec(cos.numpy(), sin.numpy(), prune=style, attn="streaming")
    hk = torch.empty(k.shape, dtype=torch.bfloat16, pin_memory=True).copy_(k)
    hv = torch.empty(v.shape, dtype=torch.bfloat16, pin_memory=True).copy_(v)
    kd, vd, sld = k.cuda(), v.cuda(), sl.cuda()
    cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots)
    blocks_per_head = (w.T + bt - 1) // bt
    sim = [orc.LruBank(cache.n_blocks_total, mask_slots), orc.LruBank(cache.n_blocks_total, sa_slots)]
    try:
        for call, seed in enumerate([0, 1, 0, 2]):
            q = configs.make_q(w, seed, kind="int")
            qd = q.cuda()
            L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
            ref_blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
            ref = L.decode_layer(qd, kd, vd, chunks, keeps, out_blocks=ref_blocks, rope=rp)
            got_blocks = torch.empty_like(ref_blocks)
            got = L.decode_layer(qd, None, None, chunks, keeps, out_blocks=got_blocks, rope=rp, cache=cache)
            cache.update()
            torch.cuda.synchronize()
            assert torch.equal(got_blocks, ref_blocks), call
            assert torch.equal(got, ref), call
            o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream, rope=spec)
            res = o.layer(w.stages)
            stats = cache.stats()
            for bank, name in ((0, "mask"), (1, "sa")):
                sim[bank].call(touched_blocks(o, w, res, bt, blocks_per_head, bank))
                pt, sb = cache.tables(bank)
                assert stats[name]["last_touched"] == sim[bank].last_touched, (call, name)
                assert stats[name]["last_misses"] == sim[bank].last_misses, (call, name)
                assert pt.tolist() == sim[bank].page_table, (call, name)
    finally:
        cache.close()


@pytest.mark.parametrize("rope", [False, True])
def test_host_tier_with_fp8_rows(ihip, orc, rope):
    # FP8 KV cache behind the host tier (128-byte rows in host memory and in the banks), with and
    # without dynamic RoPE: same bits as the resident FP8 path, banks follow the oracle's touches.
    from workloads import gen
    w = configs.shrink(configs.CFG1, B=2, Hq=8, Hkv=2, T=4096 + 29, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    bt, mask_slots, sa_slots = 64, 40, 24
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    _, k, v, _, _ = configs.make_inputs(w, 0, kind="int")
    scales = (0.5, 0.25)
    k8, v8 = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    sl = torch.tensor([w.T, w.T - 700], dtype=torch.int32)
    cos, sin = gen.quarter_turn_table(w.T, w.d)
    rp = ihip.Rope(cos.cuda(), sin.cuda(), ihip.ROPE_RELATIVE, ihip.ROPE_STREAMING) if rope else None
    spec = orc.RopeSpec(cos.numpy(), sin.numpy(), prune="relative", attn="streaming") if rope else None
    hk = torch.empty(k8.shape, dtype=torch.uint8, pin_memory=True).copy_(k8)
    hv = torch.empty(v8.shape, dtype=torch.uint8, pin_memory=True).copy_(v8)
    kd, vd, sld = k8.cuda(), v8.cuda(), sl.cuda()
    cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots)
    blocks_per_head = (w.T + bt - 1) // bt
    sim = [orc.LruBank(cache.n_blocks_total, mask_slots), orc.LruBank(cache.n_blocks_total, sa_slots)]
    try:
        for call, seed in enumerate([0, 1, 0, 2]):
            q = configs.make_q(w, seed, kind="int")
            qd = q.cuda()
            L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
            ref_blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
            ref = L.decode_layer(qd, kd, vd, chunks, keeps, out_blocks=ref_blocks, rope=rp, kv_scales=scales,
                                 pooling=ihip.POOL_KV_HEAD)
            got_blocks = torch.empty_like(ref_blocks)
            got = L.decode_layer(qd, None, None, chunks, keeps, out_blocks=got_blocks, rope=rp, kv_scales=scales,
                                 cache=cache)
            cache.update()
            torch.cuda.synchronize()
            assert torch.equal(got_blocks, ref_blocks), call
            assert torch.equal(got, ref), call
            o = orc.Oracle(q, k8, v8, sl.tolist(), 1, w.n_sink, w.n_stream, rope=spec, kv_scales=scales)
            res = o.layer(w.stages)
            stats = cache.stats()
            for bank, name in ((0, "mask"), (1, "sa")):
                sim[bank].call(touched_blocks(o, w, res, bt, blocks_per_head, bank))
                pt, sb = cache.tables(bank)
                assert stats[name]["last_touched"] == sim[bank].last_touched, (call, name)
                assert stats[name]["last_misses"] == sim[bank].last_misses, (call, name)
                assert pt.tolist() == sim[bank].page_table, (call, name)
        # a bf16 request against this cache is refused
        with pytest.raises(ihip.IhipError):
            L.decode_layer(qd, None, None, chunks, keeps, cache=cache)
    finally:
        cache.close()


@pytest.mark.parametrize("fp8", [False, True])
def test_stage_by_stage_calls_through_the_host_tier(ihip, orc, fp8):
    """ihip_prune_stage_cached / ihip_sparse_attn_decode_cached: every stage bit-identical to the resident
    stage calls, the recorded touches and misses those of the layer call (same LRU simulation)."""
    from workloads import gen
    w = configs.shrink(configs.CFG1, B=2, Hq=8, Hkv=2, T=4096 + 29, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    bt, mask_slots, sa_slots = 64, 40, 24
    _, k, v, _, _ = configs.make_inputs(w, 0, kind="int")
    sl = torch.tensor([w.T, w.T - 700], dtype=torch.int32)
    scales = (0.5, 0.25) if fp8 else None
    if fp8:
        k, v = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    hk = torch.empty(k.shape, dtype=k.dtype, pin_memory=True).copy_(k)
    hv = torch.empty(v.shape, dtype=v.dtype, pin_memory=True).copy_(v)
    kd, vd, sld = k.cuda(), v.cuda(), sl.cuda()
    cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots)
    blocks_per_head = (w.T + bt - 1) // bt
    sim = [orc.LruBank(cache.n_blocks_total, mask_slots), orc.LruBank(cache.n_blocks_total, sa_slots)]
    try:
        for call, seed in enumerate([0, 1, 0, 2]):
            q = configs.make_q(w, seed, kind="int")
            qd = q.cuda()
            L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
            parents, pchunk = None, 0
            for (l_c, keep) in w.stages:
                ref_s, ref_r = L.prune_stage(qd, kd, l_c, parents, pchunk, want_rep=True,
                                             k_scale=scales[0] if fp8 else None)
                got_s, got_r = ihip.prune_stage_cached(L, qd, cache, l_c, parents, pchunk, want_rep=True,
                                                       k_scale=scales[0] if fp8 else 1.0)
                assert torch.equal(ref_s, got_s) and torch.equal(ref_r, got_r), (call, l_c)
                parents, pchunk = L.select_blocks(got_s, l_c, keep, parents, pchunk), l_c
            ref_o, ref_l = L.sparse_attn_decode(qd, kd, vd, parents, pchunk, want_lse=True, kv_scales=scales)
            got_o, got_l = ihip.sparse_attn_decode_cached(L, qd, cache, parents, pchunk, want_lse=True,
                                                          kv_scales=scales if fp8 else (1.0, 1.0))
            cache.update()
            torch.cuda.synchronize()
            assert torch.equal(ref_o, got_o) and torch.equal(ref_l, got_l), call
            o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream, kv_scales=scales)
            res = o.layer(w.stages)
            stats = cache.stats()
            for bank, name in ((0, "mask"), (1, "sa")):
                sim[bank].call(touched_blocks(o, w, res, bt, blocks_per_head, bank))
                pt, sb = cache.tables(bank)
                assert stats[name]["last_touched"] == sim[bank].last_touched, (call, name)
                assert stats[name]["last_misses"] == sim[bank].last_misses, (call, name)
                assert pt.tolist() == sim[bank].page_table, (call, name)
                assert sb.tolist() == sim[bank].slot_block, (call, name)
    finally:
        cache.close()


@pytest.mark.parametrize("fp8", [False, True])
@pytest.mark.parametrize("page", [16, 256])
def test_paged_host_tier_equals_resident_and_follows_lru(ihip, orc, page, fp8):
    """ihip_cache_create_paged: the host memory is a page pool in a seeded random page order (pages smaller
    and larger than a cache block); outputs bit-identical to the resident path, tables as the simulation."""
    from workloads import gen
    from test_gpu_random_shapes import scatter_to_pages
    w = configs.shrink(configs.CFG1, B=2, Hq=8, Hkv=2, T=4096, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    bt, mask_slots, sa_slots = 64, 40, 24
    chunks, keeps = [s[0] for s in w.stages], [s[1] for s in w.stages]
    _, k, v, _, _ = configs.make_inputs(w, 0, kind="int")
    sl = torch.tensor([w.T, w.T - 700], dtype=torch.int32)
    scales = (0.5, 0.25) if fp8 else None
    if fp8:
        k, v = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    k_pool, v_pool, table = scatter_to_pages(k, v, page, 21, 7)
    hk = torch.empty(k_pool.shape, dtype=k.dtype, pin_memory=True).copy_(k_pool)
    hv = torch.empty(v_pool.shape, dtype=v.dtype, pin_memory=True).copy_(v_pool)
    kd, vd, sld = k.cuda(), v.cuda(), sl.cuda()
    cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots, block_table=table.cuda(), seq_tokens=w.T)
    blocks_per_head = (w.T + bt - 1) // bt
    sim = [orc.LruBank(cache.n_blocks_total, mask_slots), orc.LruBank(cache.n_blocks_total, sa_slots)]
    try:
        for call, seed in enumerate([0, 1, 0, 2, 1]):
            q = configs.make_q(w, seed, kind="int")
            qd = q.cuda()
            L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
            ref_blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
            ref = L.decode_layer(qd, kd, vd, chunks, keeps, out_blocks=ref_blocks, kv_scales=scales)
            got_blocks = torch.empty_like(ref_blocks)
            got = L.decode_layer(qd, None, None, chunks, keeps, out_blocks=got_blocks, cache=cache, kv_scales=scales)
            cache.update()
            torch.cuda.synchronize()
            assert torch.equal(got_blocks, ref_blocks) and torch.equal(got, ref), call
            o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream, kv_scales=scales)
            res = o.layer(w.stages)
            stats = cache.stats()
            for bank, name in ((0, "mask"), (1, "sa")):
                sim[bank].call(touched_blocks(o, w, res, bt, blocks_per_head, bank))
                pt, sb = cache.tables(bank)
                assert stats[name]["last_misses"] == sim[bank].last_misses, (call, name)
                assert pt.tolist() == sim[bank].page_table and sb.tolist() == sim[bank].slot_block, (call, name)
    finally:
        cache.close()
