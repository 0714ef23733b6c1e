"""Seeded random shapes and plans, every variant switched on at random: the layer
calls against the oracle run with the same options.  Integer-valued inputs, the
quarter-turn rotary table and power-of-two FP8 scales make every score exact, so
the kept block lists must agree bit for bit; outputs within 2e-2.

The draws stay inside what the entry points document (shape and plan checks);
they aim at what the fixed cases do not hit together: odd sequence lengths,
sequences shorter than sink + window, sinks and windows that are no multiple of
anything, budgets larger than the number of chunks, chunk sizes down to 1, pages
down to one token, three KV heads, every group size; for prefill also E4M3 rows
and a query-block size per stage."""
import os

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


# IHIP_RANDOM_SEEDS=n widens the sweep to n draws per test (default: 14 decode, 10 prefill)
N_DECODE = int(os.environ.get("IHIP_RANDOM_SEEDS", "14"))
N_PREFILL = int(os.environ.get("IHIP_RANDOM_SEEDS", "10"))


def scatter_to_pages(k, v, page, seed, fill):
    B, Hkv, T, d = k.shape
    per_seq = (T + page - 1) // page
    n_pages = B * per_seq + 3
    order = gen.distinct_ints(seed, 77, B * per_seq, n_pages).view(B, per_seq)
    k_pool = torch.full((n_pages, Hkv, page, d), fill, dtype=k.dtype)
    v_pool = torch.full((n_pages, Hkv, page, d), fill, dtype=v.dtype)
    pad = per_seq * page - T
    kp = torch.nn.functional.pad(k, (0, 0, 0, pad)).view(B, Hkv, per_seq, page, d)
    vp = torch.nn.functional.pad(v, (0, 0, 0, pad)).view(B, Hkv, per_seq, page, d)
    for b in range(B):
        k_pool[order[b]] = kp[b].permute(1, 0, 2, 3)
        v_pool[order[b]] = vp[b].permute(1, 0, 2, 3)
    return k_pool, v_pool, order.to(torch.int32)


def draw_plan(rng, first_choices):
    chunks = [int(rng.choice(first_choices))]
    while chunks[-1] > 1 and len(chunks) < 4 and rng.random() < 0.75:
        chunks.append(chunks[-1] // int(rng.choice([2, 4] if chunks[-1] >= 4 else [2])))
    keeps = [int(rng.integers(1, 40)) for _ in chunks]
    return list(zip(chunks, keeps))


def check_against_oracle(w, o, sl, blocks, out, b_q, pooled):
    for b in range(w.B):
        for m in range(w.Tq // b_q):
            prs = o.prune_all_heads(b, m, w.stages) if pooled else [o.prune(b, g, m, w.stages) for g in range(w.Hkv)]
            for g in range(w.Hkv):
                pr = prs[g]
                p = (b * w.Hkv + g) * (w.Tq // b_q) + m
                kp = blocks[p].cpu().numpy()
                assert np.array_equal(kp[kp >= 0], pr.block_starts), (b, g, m)
                ref, _ = o.attend(b, g, m, pr.block_starts, pr.block_lens)
                got = out[b, g * w.G:(g + 1) * w.G, m * b_q:(m + 1) * b_q].float().cpu().numpy()
                assert np.abs(got - ref).max() <= 2e-2, (b, g, m)


def draw_large_plan(rng):
    """Thousands of slots per problem: the wide selection kernels, several attention splits."""
    chunks = [int(rng.choice([16, 8, 4]))]
    while chunks[-1] > 1 and len(chunks) < 3 and rng.random() < 0.7:
        chunks.append(chunks[-1] // 2)
    keeps = [int(rng.integers(200, 1500)) for _ in chunks]
    return list(zip(chunks, keeps))


@pytest.mark.parametrize("seed", [pytest.param(s, id=f"large{s}") for s in range(100, 100 + max(4, N_DECODE // 3))]
                         + list(range(N_DECODE)))
def test_random_decode_layer(ihip, orc, seed):
    rng = np.random.default_rng(1000 + seed)
    large = seed >= 100
    B, Hkv, G = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.choice([1, 2, 4, 8]))
    T = int(rng.integers(300, 3000)) if not large else int(rng.integers(20000, 70000))
    n_sink, n_stream = int(rng.choice([0, 4, 100, 128])), int(rng.choice([1, 17, 256]))
    stages = tuple(draw_plan(rng, [256, 64, 32, 8]) if not large else draw_large_plan(rng))
    if large:
        B, Hkv = min(B, 2), min(Hkv, 2)
    w = configs.shrink(configs.CFG1, B=B, Hq=Hkv * G, Hkv=Hkv, T=T, n_sink=n_sink, n_stream=n_stream,
                       n_needles=0, stages=stages)
    sl = torch.tensor([T if b == 0 else int(rng.integers(1, T + 1)) for b in range(B)], dtype=torch.int32)
    rope = rng.choice([None, "relative", "chunk"])
    fp8, page = bool(rng.integers(0, 2)), int(rng.choice([0, 0, 1, 4, 16, 64]))
    pooled = bool(rng.integers(0, 4) == 0)
    q, k, v, _, _ = configs.make_inputs(w, seed, kind="int")
    scales = (0.5, 0.25) if fp8 else None
    if fp8:
        k, v = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    cos, sin = gen.quarter_turn_table(20000 if not large else 60000, w.d)   # a row for every position or id a draw can ask for
    spec = orc.RopeSpec(cos.numpy(), sin.numpy(), prune=str(rope), attn="streaming") if rope is not None else None
    rp = None
    if rope is not None:
        style = ihip.ROPE_RELATIVE if rope == "relative" else ihip.ROPE_CHUNK_INDEXED
        rp = ihip.Rope(cos.cuda(), sin.cuda(), style, ihip.ROPE_STREAMING)
    pg = None
    if page:
        k_pool, v_pool, table = scatter_to_pages(k, v, page, seed, 7)
        pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    L = ihip.Layer(qd, kd, sl.cuda(), 1, n_sink, n_stream)
    chunks, keeps = [s[0] for s in stages], [s[1] for s in stages]
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
    out = L.decode_layer(qd, kd, vd, chunks, keeps, out_blocks=blocks, rope=rp, kv_scales=scales, paged=pg,
                         pooling=ihip.POOL_ALL_HEADS if pooled else None)
    torch.cuda.synchronize()
    o = orc.Oracle(q, k, v, sl.tolist(), 1, n_sink, n_stream, rope=spec, kv_scales=scales)
    check_against_oracle(w, o, sl, blocks, out, 1, pooled)


@pytest.mark.parametrize("seed", list(range(max(8, N_DECODE // 2))))
def test_random_decode_layer_behind_the_host_tier(ihip, orc, seed):
    """The same draws with K/V in pinned host memory (contiguous or a page pool) behind hot-block banks of
    random size: two calls with an update in between (the second is served partly from the banks), both
    against the oracle; RoPE, E4M3 rows and all-heads pooling at random."""
    rng = np.random.default_rng(4000 + seed)
    B, Hkv, G = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.choice([1, 2, 4, 8]))
    T = int(rng.integers(300, 3000))
    n_sink, n_stream = int(rng.choice([0, 4, 100, 128])), int(rng.choice([1, 17, 256]))
    stages = tuple(draw_plan(rng, [256, 64, 32, 8]))
    w = configs.shrink(configs.CFG1, B=B, Hq=Hkv * G, Hkv=Hkv, T=T, n_sink=n_sink, n_stream=n_stream,
                       n_needles=0, stages=stages)
    sl = torch.tensor([T if b == 0 else int(rng.integers(1, T + 1)) for b in range(B)], dtype=torch.int32)
    rope = rng.choice([None, "relative", "chunk"])
    fp8, page = bool(rng.integers(0, 2)), int(rng.choice([0, 0, 4, 16, 128]))
    pooled = bool(rng.integers(0, 4) == 0)
    bt = int(rng.choice([16, 64]))
    mask_slots, sa_slots = int(rng.integers(1, 60)), int(rng.integers(1, 60))
    q, k, v, _, _ = configs.make_inputs(w, seed, kind="int")
    scales = (0.5, 0.25) if fp8 else None
    if fp8:
        k, v = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    cos, sin = gen.quarter_turn_table(20000, w.d)
    spec = orc.RopeSpec(cos.numpy(), sin.numpy(), prune=str(rope), attn="streaming") if rope is not None else None
    rp = None
    if rope is not None:
        style = ihip.ROPE_RELATIVE if rope == "relative" else ihip.ROPE_CHUNK_INDEXED
        rp = ihip.Rope(cos.cuda(), sin.cuda(), style, ihip.ROPE_STREAMING)
    if page:
        k_pool, v_pool, table = scatter_to_pages(k, v, page, seed, 7)
        hk = torch.empty(k_pool.shape, dtype=k.dtype, pin_memory=True).copy_(k_pool)
        hv = torch.empty(v_pool.shape, dtype=v.dtype, pin_memory=True).copy_(v_pool)
        cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots, block_table=table.cuda(), seq_tokens=T)
    else:
        hk = torch.empty(k.shape, dtype=k.dtype, pin_memory=True).copy_(k)
        hv = torch.empty(v.shape, dtype=v.dtype, pin_memory=True).copy_(v)
        cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots)
    try:
        chunks, keeps = [s[0] for s in stages], [s[1] for s in stages]
        for call in range(2):
            q = configs.make_q(w, seed + call, kind="int")
            qd = q.cuda()
            L = ihip.Layer(qd, torch.empty((B, Hkv, T, 0), dtype=torch.bfloat16, device="cuda"), sl.cuda(), 1,
                           n_sink, n_stream)
            blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
            out = L.decode_layer(qd, None, None, chunks, keeps, out_blocks=blocks, rope=rp, kv_scales=scales,
                                 cache=cache, pooling=ihip.POOL_ALL_HEADS if pooled else None)
            cache.update()
            torch.cuda.synchronize()
            o = orc.Oracle(q, k, v, sl.tolist(), 1, n_sink, n_stream, rope=spec, kv_scales=scales)
            check_against_oracle(w, o, sl, blocks, out, 1, pooled)
        st = cache.stats()
        assert st["mask"]["last_touched"] >= 0 and st["sa"]["last_touched"] > 0
    finally:
        cache.close()


@pytest.mark.parametrize("seed", [pytest.param(s, id=f"large{s}") for s in range(100, 100 + max(3, N_PREFILL // 3))]
                         + list(range(N_PREFILL)))
def test_random_prefill_layer(ihip, orc, seed):
    rng = np.random.default_rng(2000 + seed)
    large = seed >= 100         # hundreds of kept chunks: long key lists, either attention kernel
    B, Hkv, G = int(rng.integers(1, 3)), int(rng.integers(1, 3)), int(rng.choice([1, 2, 4, 8]))
    b_q = int(rng.choice([16, 32, 64]))
    Tq = b_q * int(rng.integers(1, 4))
    T = Tq + (int(rng.integers(0, 1500)) if not large else int(rng.integers(4000, 14000)))
    n_sink, n_stream = int(rng.choice([0, 4, 100, 128])), b_q + int(rng.choice([0, 1, 70, 192]))
    stages = tuple(draw_plan(rng, [64, 32, 16]))
    if large:
        B, Hkv = 1, min(Hkv, 2)
        stages = tuple((c, int(rng.integers(100, 400))) for c, _ in stages)
    # a query-block size per stage (a stream of its own, so that the other draws stay as they were):
    # built from the last stage (b_q) backwards, doubling at random; the new tokens are then a whole
    # number of first-stage blocks and the window holds one
    rng_b = np.random.default_rng(3000 + seed)
    stage_b_q = [b_q]
    for _ in stages[1:]:
        stage_b_q.insert(0, min(64, stage_b_q[0] * int(rng_b.choice([1, 2]))))
    if stage_b_q[0] == b_q:
        stage_b_q = None
    else:
        first = stage_b_q[0]
        T += -Tq % first
        Tq += -Tq % first
        n_stream = max(n_stream, first)
    w = configs.shrink(configs.CFG4, B=B, Hq=Hkv * G, Hkv=Hkv, T=T, Tq=Tq, b_q=b_q, n_sink=n_sink,
                       n_stream=n_stream, stages=stages)
    sl = torch.tensor([T if b == 0 else int(rng.integers(Tq, T + 1)) for b in range(B)], dtype=torch.int32)
    rope = rng.choice([None, "relative", "chunk"])
    page = int(rng.choice([0, 0, 1, 4, 16, 64]))
    pooled = bool(rng.integers(0, 4) == 0)
    fp8 = bool(rng.integers(0, 2))
    q, k, v, _, _ = configs.make_inputs(w, seed, kind="int")
    scales = (0.25, 0.5) if fp8 else None
    if fp8:
        k, v = gen.to_e4m3(k, scales[0]), gen.to_e4m3(v, scales[1])
    cos, sin = gen.quarter_turn_table(20000 if not large else 60000, w.d)
    spec = orc.RopeSpec(cos.numpy(), sin.numpy(), prune=str(rope), attn="streaming") if rope is not None else None
    rp = None
    if rope is not None:
        style = ihip.ROPE_RELATIVE if rope == "relative" else ihip.ROPE_CHUNK_INDEXED
        rp = ihip.Rope(cos.cuda(), sin.cuda(), style, ihip.ROPE_STREAMING)
    pg = None
    if page:
        k_pool, v_pool, table = scatter_to_pages(k, v, page, seed, 7)
        pg = ihip.PagedKV(k_pool.cuda(), v_pool.cuda(), table.cuda())
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    L = ihip.Layer(qd, kd, sl.cuda(), b_q, n_sink, n_stream)
    chunks, keeps = [s[0] for s in stages], [s[1] for s in stages]
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device="cuda")
    out = L.prefill_layer(qd, kd, vd, chunks, keeps, out_blocks=blocks, rope=rp, paged=pg, kv_scales=scales,
                          pooling=ihip.POOL_ALL_HEADS if pooled else None, stage_b_q=stage_b_q)
    torch.cuda.synchronize()
    o = orc.Oracle(q, k, v, sl.tolist(), b_q, n_sink, n_stream, rope=spec, kv_scales=scales, stage_b_q=stage_b_q)
    check_against_oracle(w, o, sl, blocks, out, b_q, pooled)
