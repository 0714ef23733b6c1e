#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.  One step = one layer call: all
pruning stages + arg-top-K selects + block-sparse attention, every stage
refreshed, over one batch of synthetic input resident in HBM.

Default workload (the headline metric): cfg3 -- decode, batch 8, 1,048,576
keys per sequence, 32 query / 8 KV heads, d = 128, bf16, 4 stages
(256 -> 64 -> 16 -> 4), 4,096-token budget.  One layer's K/V (32 GiB) stays in
HBM and is reused by 32 different query sets, so consecutive steps touch
different rows.  `--workload cfg4-prefill-4k-on-256k` times the chunked
prefill layer instead (4,096 new tokens on a 262,144-token prefix).

Prints one JSON line.  `value` is microseconds per layer call for the whole
batch.  `roofline` is for the kernel with the largest share of the step:
 - decode: algorithmic bytes per launch (distinct K rows the search must
   score, counted by the CPU oracle on a sample of problems, x 256 B, plus the
   scores it writes) / mean launch duration, against 8 TB/s of HBM;
 - prefill: matrix-core flops per launch (2*d per query-key pair actually
   multiplied) / mean launch duration, against 2.5 PFLOP/s dense bf16.
The mean launch duration comes from HIP events recorded around every launch
on its stream in a second pass over the same steps.  `cpu_baseline` is the
CPU oracle timed on a bounded sample of the same workload in the same run.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
N_QUERY_SETS = 32

# HBM traffic per launch from rocprofv3 --pmc runs of this same command (FETCH_SIZE, then WRITE_SIZE, KiB
# per dispatch, each scaled by what the counter reads for a device copy of known size: FETCH_SIZE x 2.0,
# WRITE_SIZE x 1.0).  Counters cannot be read inside this process, so the figure is carried from the
# summary named in `traffic_source`, which also gives the date and commit it was taken at; a kernel that
# has no current summary reports traffic null.
TRAFFIC_SOURCE = "profiles/decode_cfg3_and_prefill_cfg4_kernel_trace_and_hbm_counters.txt"
MEASURED_TRAFFIC_BYTES = {
    ("cfg3-decode-1m-b8", "prune_decode.first.l256"): (781758.3 * 2.0 + 1225.5) * 1024.0,
    ("cfg4-prefill-4k-on-256k", "prune_prefill.first.l64"): (765662.2 * 2.0 + 10655.5) * 1024.0,
    ("cfg4-prefill-4k-on-256k", "prune_prefill.l16"): (469639.2 * 2.0 + 2048.0) * 1024.0,
    ("cfg4-prefill-4k-on-256k", "attn_prefill"): (636708.9 * 2.0 + 32769.9) * 1024.0,
}


def measured_traffic(workload, kernel):
    t = MEASURED_TRAFFIC_BYTES.get((workload, kernel))
    if t is None:
        return {"traffic": None}
    return {"traffic": t, "traffic_source": TRAFFIC_SOURCE}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="cfg3-decode-1m-b8")
    ap.add_argument("--kv-dtype", default="bf16", choices=["bf16", "fp8"],
                    help="fp8 = K and V quantised to E4M3 bytes (scale 1/64 each), a separate metric")
    ap.add_argument("--paged", type=int, default=0, metavar="PAGE_TOKENS",
                    help="decode and prefill workloads: K and V scattered into pages of this many tokens in a seeded random "
                         "order, read through a block table (a separate metric)")
    ap.add_argument("--paged-order", default="random", choices=["random", "sequential"],
                    help="with --paged: page ids in a seeded random order (default) or in token order")
    ap.add_argument("--kv-layout", default="bhtd", choices=["bhtd", "bthd"],
                    help="decode workloads: memory order of K and V (the same logical [B,Hkv,T,d] tensors; bthd = "
                         "token-major, the KV heads of a token adjacent)")
    ap.add_argument("--rope", default=None, choices=["relative", "chunk"],
                    help="decode and prefill workloads: dynamic RoPE in the pruning stages (this style) and the attention "
                         "(streaming style); a separate metric, no roofline / cpu_baseline objects")
    ap.add_argument("--graph", action="store_true",
                    help="decode and prefill workloads: capture the timed steps into one HIP graph and time its replay "
                         "(a separate metric)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="CPU time budget of the oracle baseline (0 = skip)")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--refresh", default=None,
                    help="decode only: comma-separated mask refresh intervals per stage (e.g. 16,8,4,2); "
                         "stage i is recomputed only at steps that are multiples of its interval and the "
                         "cached masks are reused otherwise (the reported value is then the amortised time)")
    ap.add_argument("--bank-mib", type=int, default=512,
                    help="cfg5 only: on-GPU bytes of the hot-block banks (default 512 MiB: a 16 GB budget over 32 layers)")
    ap.add_argument("--no-extras", action="store_true",
                    help="default workload only: do not append the `prefill` (cfg4) and `offload` (cfg5) objects")
    ap.add_argument("--extras-budget-s", type=float, default=150.0,
                    help="an extra workload is started only while the run is younger than this")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run 10 device copies of 1 GiB (a kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters) and exit")
    return ap.parse_args()


def progress(msg):
    """One line per finished phase on stderr (a long profiled run is not silent)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def timed_passes(step, steps, warmup, ihip, torch, profile, graph=False):
    """W warm-up steps, K timed steps between synchronisations, then (optionally)
    the same K steps again with HIP events around every kernel launch.
    graph: the K steps are captured into one HIP graph (the library neither allocates nor
    synchronises) and one replay of it is timed, after one untimed replay."""
    progress("inputs ready")
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    progress("warm-up done")
    if graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(steps):
                step(i)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.replay()
    else:
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / steps * 1e6
    progress(f"{steps} timed steps done")
    kernels = {}
    if profile:
        ihip.profile_enable(True)
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        ihip.profile_enable(False)
        for name, (ms, n) in ihip.profile_read().items():
            kernels[name] = {"us": ms / n * 1e3, "launches_per_step": n / steps}
    return us, kernels, step_spread(step, steps, torch) if not graph else None


def step_spread(step, steps, torch, first=0):
    """The same steps once more with an event pair around each (the library enqueues on torch's current
    stream): p10 / median / p90 of the per-step times, which the mean over the timed region hides."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i in range(steps):
        ev[i][0].record()
        step(first + i)
        ev[i][1].record()
    torch.cuda.synchronize()
    t = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    pick = lambda f: t[min(len(t) - 1, int(f * len(t)))]      # noqa: E731
    progress("per-step spread done")
    return {"p10": pick(0.1), "median": pick(0.5), "p90": pick(0.9), "n": len(t), "unit": "us"}


def dominant(kernels):
    return max(kernels, key=lambda n: kernels[n]["us"] * kernels[n]["launches_per_step"])


# ---------------------------------------------------------------------------
def host_threads():
    """Worker threads of the CPU baseline: the host cores this process may use (the box's share,
    OMP_NUM_THREADS where it is set), at most 16.  The oracle's C routines run outside the
    interpreter lock, so threads scale like processes and nothing is forked after the GPU is up."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return max(1, min(16, n))


def decode_oracle_sample(w, qs, kvs, seq_lens, budget_s, kv_scales=None):
    """Times the CPU oracle, as it stands, on sequence 0: its (query set, KV head) problems are dealt
    to host_threads() threads -- the arithmetic of a problem is untouched --, a wave of whole layer
    calls at a time until the budget is used.  Also returns the mean number of distinct K rows each
    stage scores per problem and the attended tokens."""
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    oracle.build(force=False)
    threads = host_threads()
    host = {}
    rows = [0.0] * len(w.stages)
    tokens, problems, calls, t_used = 0.0, 0, 0, 0.0
    sets_per_wave = max(1, threads // w.Hkv)

    def one(task):
        o, g = task
        pr = o.prune(0, g, 0, w.stages)
        o.attend(0, g, 0, pr.block_starts, pr.block_lens)
        return [st.rows_touched for st in pr.stages], o.attended_tokens(0, 0, pr.block_lens)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        for i0 in range(0, len(qs), sets_per_wave):
            tasks = []
            for i in range(i0, min(len(qs), i0 + sets_per_wave)):
                layer = i % len(kvs)
                if layer not in host:
                    host = {layer: (kvs[layer][0][0:1].cpu(), kvs[layer][1][0:1].cpu())}
                k0, v0 = host[layer]
                o = oracle.Oracle(qs[i][0:1].cpu(), k0, v0, [int(seq_lens[0])], w.b_q, w.n_sink, w.n_stream,
                                  kv_scales=kv_scales)
                tasks += [(o, g) for g in range(w.Hkv)]
                calls += 1
            t0 = time.perf_counter()
            done = list(pool.map(one, tasks))
            t_used += time.perf_counter() - t0
            for stage_rows, toks in done:
                for s_, r in enumerate(stage_rows):
                    rows[s_] += r
                tokens += toks
                problems += 1
            if t_used >= budget_s:
                break
    return {"seconds": t_used, "layer_calls_one_sequence": calls, "problems": problems, "threads": threads,
            "rows_per_problem": [r / problems for r in rows], "tokens_per_problem": tokens / problems}


def bench_decode(args, w, torch, ihip, configs):
    dev = torch.device("cuda:0")
    steps = 200 if args.steps is None else args.steps
    warmup = 20 if args.warmup is None else args.warmup
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]

    t0 = time.perf_counter()
    # one layer's K/V when it is far larger than the 256 MB last-level cache; otherwise as many
    # distinct layers as query sets (32), rotated, so that steps never find their rows cached
    layer_bytes = 2 * w.B * w.Hkv * w.T * w.d * 2
    n_layers = 1 if layer_bytes >= (4 << 30) else N_QUERY_SETS
    kvs = [configs.make_kv(w, layer, dev) for layer in range(n_layers)]
    qs = []
    for i in range(N_QUERY_SETS):
        q = configs.make_q(w, i, dev)
        configs.plant_needles(w, kvs[i % n_layers][0], q, i)
        qs.append(q)
    kv_scales = None
    if args.kv_dtype == "fp8":
        # the same Gaussian K/V, quantised one sequence at a time (needles included)
        from workloads import gen
        kv_scales = (1.0 / 64, 1.0 / 64)
        kvs8 = []
        for (kb, vb) in kvs:
            k8 = torch.empty(kb.shape, dtype=torch.uint8, device=dev)
            v8 = torch.empty(vb.shape, dtype=torch.uint8, device=dev)
            for b in range(w.B):
                k8[b] = gen.to_e4m3(kb[b], kv_scales[0])
                v8[b] = gen.to_e4m3(vb[b], kv_scales[1])
            kvs8.append((k8, v8))
        kvs = kvs8
        del kvs8, kb, vb
        torch.cuda.empty_cache()
    paged = None
    if args.paged:
        assert n_layers == 1, "paged: one layer"
        page = args.paged
        per_seq = (w.T + page - 1) // page
        assert per_seq * page == w.T, "context must be a whole number of pages"
        gen_ = torch.Generator(device=dev)
        gen_.manual_seed(1234)
        if args.paged_order == "random":
            order = torch.randperm(w.B * per_seq, generator=gen_, device=dev).view(w.B, per_seq)
        else:
            order = torch.arange(w.B * per_seq, device=dev).view(w.B, per_seq)
        kb, vb = kvs[0]
        k_pool = torch.empty((w.B * per_seq, w.Hkv, page, w.d), dtype=kb.dtype, device=dev)
        v_pool = torch.empty_like(k_pool)
        for b in range(w.B):
            k_pool[order[b]] = kb[b].view(w.Hkv, per_seq, page, w.d).permute(1, 0, 2, 3)
            v_pool[order[b]] = vb[b].view(w.Hkv, per_seq, page, w.d).permute(1, 0, 2, 3)
        paged = ihip.PagedKV(k_pool, v_pool, order.to(torch.int32).contiguous())
    if args.kv_layout == "bthd":
        # same values, token-major in memory: [B,T,Hkv,d] storage viewed as [B,Hkv,T,d]
        re = []
        for (kb, vb) in kvs:
            k2 = torch.empty((w.B, w.T, w.Hkv, w.d), dtype=kb.dtype, device=dev)
            v2 = torch.empty_like(k2)
            for b in range(w.B):
                k2[b] = kb[b].transpose(0, 1)
                v2[b] = vb[b].transpose(0, 1)
            re.append((k2.transpose(1, 2), v2.transpose(1, 2)))
        kvs = re
        del re, kb, vb
        torch.cuda.empty_cache()
    k, v = kvs[0]
    seq_lens = torch.full((w.B,), w.T, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t0

    L = ihip.Layer(qs[0], k, seq_lens, w.b_q, w.n_sink, w.n_stream)
    ws = L.workspace(ihip.OP_DECODE_LAYER, chunks, keeps)
    out = torch.empty((w.B, w.Hq, 1, w.d), dtype=torch.bfloat16, device=dev)
    # any combination of the variants goes through the one call (ihip_decode_layer_ex underneath)
    rope = None
    if args.rope:
        from workloads import gen
        n_pos = max(L.stage1_slots(chunks[0]), max(keeps)) + w.n_sink + w.n_stream + keeps[-1] * chunks[-1] + 8
        cos, sin = gen.rope_table(n_pos, w.d, device=dev)
        rope = ihip.Rope(cos, sin, ihip.ROPE_RELATIVE if args.rope == "relative" else ihip.ROPE_CHUNK_INDEXED,
                         ihip.ROPE_STREAMING)
    refresh = state = None
    if args.refresh:
        refresh = [int(x) for x in args.refresh.split(",")]
        assert len(refresh) == len(chunks), "one refresh interval per stage"
        assert n_layers == 1, "mask caching follows one layer's decode steps"
        state = L.mask_state(keeps)

    def step(i):
        kl, vl = kvs[i % n_layers]
        L.decode_layer(qs[i % N_QUERY_SETS], kl, vl, chunks, keeps, ws=ws, out=out, rope=rope, kv_scales=kv_scales,
                       paged=paged, stage_starts=state,
                       first_stage=ihip.first_stage_due(i, refresh) if refresh else None)

    us_per_layer, kernels, spread = timed_passes(step, steps, warmup, ihip, torch, not args.no_profile_pass, args.graph)

    cpu = sample = None
    if args.cpu_seconds > 0 and not args.rope:
        sample = decode_oracle_sample(w, qs, kvs, seq_lens.cpu().tolist(), args.cpu_seconds, kv_scales)
        per_seq_call = sample["seconds"] / sample["layer_calls_one_sequence"]
        cpu = {"value": per_seq_call * w.B * 1e6, "unit": "us/layer", "cores": sample["threads"], "kind": "oracle",
               "sample": f"sequence 0 of {w.B} (its {w.Hkv} KV heads), {sample['layer_calls_one_sequence']} "
                         f"layer calls with different queries, their (query set, KV head) problems dealt to "
                         f"{sample['threads']} threads, {sample['seconds']:.1f} s of wall time; scaled x{w.B} to the batch"}

    P = w.B * w.Hkv
    row_bytes = w.d * (1 if kv_scales else 2)
    roofline = whole = None
    if sample is not None and refresh is None:
        alg = {}
        slots = [L.stage1_slots(chunks[0])] + [keeps[i - 1] * (chunks[i - 1] // chunks[i])
                                                 for i in range(1, len(chunks))]
        for i, c in enumerate(chunks):
            first = ".first" if i == 0 else ""
            alg[f"prune_decode{first}.l{c}"] = P * (sample["rows_per_problem"][i] * row_bytes + slots[i] * 4)
            alg[f"select_blocks{first}.l{c}"] = P * (slots[i] * 4 + keeps[i] * 4)
        alg["attn_decode_split"] = P * sample["tokens_per_problem"] * 2 * row_bytes
        total_alg = sum(alg.values())
        gbs = total_alg / (us_per_layer * 1e-6) / 1e9
        whole = {"algorithmic_bytes_per_layer": total_alg, "achieved_GBps": gbs,
                 "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
        for n in kernels:
            if n in alg:
                kernels[n]["alg_GBps"] = alg[n] / (kernels[n]["us"] * 1e-6) / 1e9
        if kernels and dominant(kernels) in alg:
            dom = dominant(kernels)
            ach = kernels[dom]["alg_GBps"]
            roofline = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": ach / HBM_PEAK_GBS,
                        "algorithmic_bytes_per_launch": alg[dom], "us_per_launch": kernels[dom]["us"]}
            plain = not (kv_scales or paged or rope or args.kv_layout != "bhtd")
            roofline.update(measured_traffic(w.name if plain else None, dom))
    return {
        "metric": ("sparse_attn_decode_us_per_layer_1m_ctx" if w.T == 1048576 else "sparse_attn_decode_us_per_layer")
        + ("_amortised_mask_cache" if refresh else "") + (f"_dynamic_rope_{args.rope}" if args.rope else "") + ("_fp8_kv" if kv_scales else "") + (f"_paged{args.paged}_{args.paged_order}" if args.paged else "")
        + ("_hip_graph" if args.graph else ""),
        "value": us_per_layer, "unit": "us/layer", "steps": steps, "warmup": warmup,
        "config": {"workload": w.name, "batch": w.B, "context": w.T, "q_heads": w.Hq, "kv_heads": w.Hkv,
                   "head_dim": w.d, "stages_chunk_keep": list(map(list, w.stages)), "n_sink": w.n_sink,
                   "n_stream": w.n_stream, "query_sets": N_QUERY_SETS, "distinct_kv_layers": n_layers,
                   "mask_refresh": refresh, "kv_layout": args.kv_layout},
        "roofline": roofline, "cpu_baseline": cpu, "whole_path": whole, "kernels": kernels, "step_us": spread,
        "setup_s": t_setup,
    }


# ---------------------------------------------------------------------------
def bench_prefill(args, w, torch, ihip, configs):
    dev = torch.device("cuda:0")
    steps = 20 if args.steps is None else args.steps
    warmup = 3 if args.warmup is None else args.warmup
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]

    t0 = time.perf_counter()
    q, k, v, seq_lens, _ = configs.make_inputs(w, 0, dev)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t0

    kv_scales = None
    if args.kv_dtype == "fp8":
        from workloads import gen
        kv_scales = (1.0 / 64, 1.0 / 64)
        k, v = gen.to_e4m3(k, kv_scales[0]), gen.to_e4m3(v, kv_scales[1])
    L = ihip.Layer(q, k, seq_lens, w.b_q, w.n_sink, w.n_stream)
    ws = L.workspace(ihip.OP_PREFILL_LAYER, chunks, keeps)
    out = torch.empty((w.B, w.Hq, w.Tq, w.d), dtype=torch.bfloat16, device=dev)

    rope = None
    if args.rope:
        from workloads import gen
        n_pos = max(L.stage1_slots(chunks[0]), max(keeps)) + w.n_sink + w.n_stream + keeps[-1] * chunks[-1] + 8
        cos, sin = gen.rope_table(n_pos, w.d, device=dev)
        rope = ihip.Rope(cos, sin, ihip.ROPE_RELATIVE if args.rope == "relative" else ihip.ROPE_CHUNK_INDEXED,
                         ihip.ROPE_STREAMING)

    paged = None
    if args.paged:
        page = args.paged
        per_seq = (w.T + page - 1) // page
        assert per_seq * page == w.T, "context must be a whole number of pages"
        gen_ = torch.Generator(device=dev)
        gen_.manual_seed(1234)
        if args.paged_order == "random":
            order = torch.randperm(w.B * per_seq, generator=gen_, device=dev).view(w.B, per_seq)
        else:
            order = torch.arange(w.B * per_seq, device=dev).view(w.B, per_seq)
        k_pool = torch.empty((w.B * per_seq, w.Hkv, page, w.d), dtype=k.dtype, device=dev)
        v_pool = torch.empty_like(k_pool)
        for b in range(w.B):
            k_pool[order[b]] = k[b].view(w.Hkv, per_seq, page, w.d).permute(1, 0, 2, 3)
            v_pool[order[b]] = v[b].view(w.Hkv, per_seq, page, w.d).permute(1, 0, 2, 3)
        paged = ihip.PagedKV(k_pool, v_pool, order.to(torch.int32).contiguous())

    def step(i):
        L.prefill_layer(q, k, v, chunks, keeps, ws=ws, out=out, rope=rope, paged=paged, kv_scales=kv_scales)

    us_per_layer, kernels, spread = timed_passes(step, steps, warmup, ihip, torch, not args.no_profile_pass, args.graph)

    # matrix-core flops actually multiplied, from the geometry alone
    flops = {}
    n_valid_prev = None
    for i, (c, keep) in enumerate(w.stages):
        pairs = 0          # candidate rows scored x queries
        kept_valid = []
        for m in range(w.Mq):
            E = (w.T - w.Tq) + (m + 1) * w.b_q
            mid = max(0, E - w.n_stream - w.n_sink)
            if i == 0:
                n = math.ceil(mid / c)
            else:
                n = n_valid_prev[m] * (w.stages[i - 1][0] // c)     # ragged tails ignored (<= 1 chunk)
            kept_valid.append(min(keep, n))
            pairs += n * (1 + int(math.log2(c))) * w.b_q
        n_valid_prev = kept_valid
        first = ".first" if i == 0 else ""
        # relative-style RoPE: every candidate row against two rotated copies of the queries
        flops[f"prune_prefill{first}.l{c}"] = w.B * w.Hq * pairs * w.d * 2 * (2 if args.rope == "relative" else 1)
    keys = 0
    for m in range(w.Mq):
        E = (w.T - w.Tq) + (m + 1) * w.b_q
        hi = E - w.n_stream
        keys += min(w.n_sink, E) + n_valid_prev[m] * chunks[-1] + (E - max(hi, w.n_sink))
    flops["attn_prefill"] = w.B * w.Hq * w.b_q * keys * w.d * 4
    for n in kernels:
        if n in flops:
            kernels[n]["TFLOPs"] = flops[n] / (kernels[n]["us"] * 1e-6) / 1e12
    # what the matrix cores of this GPU sustain on independent chains of the two MFMA shapes the
    # kernels use (no memory traffic), next to the vendor's peak
    measured = {"attn_prefill": ihip.mfma_rate(0), "prune_prefill": ihip.mfma_rate(1)}
    for n in kernels:
        if "TFLOPs" in kernels[n]:
            kernels[n]["frac_of_peak"] = kernels[n]["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
            kernels[n]["frac_of_measured_mfma_rate"] = kernels[n]["TFLOPs"] / measured[n.split(".")[0]]
    def mfma_roofline(name):
        ach = kernels[name]["TFLOPs"]
        r = {"kernel": name, "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
             "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
             "flops_per_launch": flops[name], "us_per_launch": kernels[name]["us"],
             "measured_mfma_rate": measured[name.split(".")[0]],
             "frac_of_measured_mfma_rate": ach / measured[name.split(".")[0]]}
        r.update(measured_traffic(None if rope or paged or kv_scales else w.name, name))
        return r

    roofline = None
    if kernels and dominant(kernels) in flops:
        roofline = mfma_roofline(dominant(kernels))
    rooflines = {n: mfma_roofline(n) for n in kernels if n in flops}

    cpu = None
    if args.cpu_seconds > 0 and not rope:
        from concurrent.futures import ThreadPoolExecutor
        import oracle
        oracle.build(force=False)
        threads = host_threads()
        blocks = [0, w.Mq // 3, (2 * w.Mq) // 3, w.Mq - 1]
        o = oracle.Oracle(q.cpu(), k.cpu(), v.cpu(), [w.T] * w.B, w.b_q, w.n_sink, w.n_stream, kv_scales=kv_scales)
        t0 = time.perf_counter()
        done = 0
        # the oracle as it stands, its (KV head, query block) problems dealt to the threads, one query
        # block (all KV heads) at a time
        with ThreadPoolExecutor(max_workers=threads) as pool:
            for m in blocks:
                list(pool.map(lambda g: o.layer(w.stages, problems=[(0, g, m)]), range(w.Hkv)))
                done += w.Hkv
                if time.perf_counter() - t0 > args.cpu_seconds:
                    break
        secs = time.perf_counter() - t0
        P = w.B * w.Hkv * w.Mq
        cpu = {"value": secs / done * P * 1e6, "unit": "us/layer", "cores": threads, "kind": "oracle",
               "sample": f"{done} of {P} (KV head, query block) problems (all KV heads of blocks "
                         f"{blocks[:done // w.Hkv]}) on {threads} threads, {secs:.1f} s of wall time; scaled x{P}/{done}"}
    return {
        "metric": "sparse_attn_prefill_us_per_layer" + ("_fp8_kv" if kv_scales else "") + ("_hip_graph" if args.graph else ""),
        "value": us_per_layer, "unit": "us/layer", "steps": steps, "warmup": warmup,
        "config": {"workload": w.name + (f"_dynamic_rope_{args.rope}" if rope else "")
                   + (f"_paged{args.paged}_{args.paged_order}" if paged else ""), "batch": w.B, "context": w.T, "new_tokens": w.Tq, "query_block": w.b_q,
                   "q_heads": w.Hq, "kv_heads": w.Hkv, "head_dim": w.d,
                   "stages_chunk_keep": list(map(list, w.stages)), "n_sink": w.n_sink, "n_stream": w.n_stream},
        "roofline": roofline, "rooflines": rooflines, "cpu_baseline": cpu,
        "whole_path": {"mfma_flops_per_layer": sum(flops.values()),
                       "achieved_TFLOPs": sum(flops.values()) / (us_per_layer * 1e-6) / 1e12,
                       "measured_mfma_rate_TFLOPs": {"32x32x16_bf16": measured["attn_prefill"],
                                                     "16x16x32_bf16": measured["prune_prefill"]}},
        "kernels": kernels, "step_us": spread, "setup_s": t_setup,
    }


# ---------------------------------------------------------------------------
def bench_offload(args, w, torch, ihip, configs):
    """cfg5: K/V of the layer in pinned host memory, 512 MiB of on-GPU banks
    (256 MiB of keys for the pruning stages, 256 MiB of keys+values for the
    attention), one decode call after another with Zipf(1.1)-placed needles.
    The bound here is the host link, not HBM; no roofline object is claimed."""
    from workloads import gen
    dev = torch.device("cuda:0")
    steps = 24 if args.steps is None else args.steps
    warmup = 4 if args.warmup is None else args.warmup
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    # --bank-mib: the on-GPU budget, half for the pruning stages' key bank, half for the attention's
    # key+value bank (64-token blocks of 256-byte rows); never more slots than the layer has blocks
    bt = 64
    n_blocks_total = w.B * w.Hkv * ((w.T + bt - 1) // bt)
    mask_slots = min(n_blocks_total, (args.bank_mib << 20) // 2 // (bt * 256))
    sa_slots = min(n_blocks_total, (args.bank_mib << 20) // 2 // (bt * 512))
    shape = (w.B, w.Hkv, w.T, w.d)

    t0 = time.perf_counter()
    hk = torch.empty(shape, dtype=torch.bfloat16, pin_memory=True)
    hv = torch.empty(shape, dtype=torch.bfloat16, pin_memory=True)
    step_t = 1 << 18
    for tid_, host in ((configs.TID_K, hk), (configs.TID_V, hv)):
        for t_lo in range(0, w.T, step_t):
            t_hi = min(w.T, t_lo + step_t)
            host[:, :, t_lo:t_hi].copy_(gen.normal_bf16(0, tid_, shape, dev, (0, w.B, 0, w.Hkv, t_lo, t_hi)))
    n_calls = steps + warmup
    l1 = chunks[0]
    n_chunks = (w.T - w.n_sink - w.n_stream) // l1
    qs = []
    for c in range(n_calls):
        q = configs.make_q(w, c, "cpu")
        ranks = gen.zipf_ranks(c, 77, w.Hkv * w.n_needles, n_chunks).view(w.Hkv, w.n_needles)
        chunk_ids = (ranks * 7919 + 12345) % n_chunks            # fixed scramble of the ranks (7919 is prime)
        pos = w.n_sink + chunk_ids * l1
        noise = gen.normal_bf16(c, configs.TID_NEEDLE_NOISE, (1, w.Hkv, w.n_needles, w.d)).float()[0]
        for g in range(w.Hkv):
            for i in range(w.n_needles):
                qv = q[0, g * w.G + i % w.G, 0].float()
                hk[0, g, pos[g, i]] = (w.needle_gain * qv / qv.norm() + w.needle_noise * noise[g, i]).to(torch.bfloat16)
        qs.append(q.to(dev))
    seq_lens = torch.full((w.B,), w.T, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t0

    kv_scales = None
    row_bytes = 256
    if args.kv_dtype == "fp8":
        # the same K/V (needles included) as E4M3 bytes in pinned memory; the same bank bytes hold twice the blocks
        kv_scales = (1.0 / 64, 1.0 / 64)
        hk8 = torch.empty(shape, dtype=torch.uint8, pin_memory=True)
        hv8 = torch.empty(shape, dtype=torch.uint8, pin_memory=True)
        for src, dst, sc in ((hk, hk8, kv_scales[0]), (hv, hv8, kv_scales[1])):
            for t_lo in range(0, w.T, step_t):
                t_hi = min(w.T, t_lo + step_t)
                dst[:, :, t_lo:t_hi].copy_(gen.to_e4m3(src[:, :, t_lo:t_hi].to(dev), sc))
        hk, hv = hk8, hv8
        mask_slots, sa_slots, row_bytes = min(n_blocks_total, 2 * mask_slots), min(n_blocks_total, 2 * sa_slots), 128
    rope = None
    if args.rope:
        n_pos = max(n_chunks + 1, max(keeps)) + w.n_sink + w.n_stream + keeps[-1] * chunks[-1] + 8
        cos, sin = gen.rope_table(n_pos, w.d, device=dev)
        rope = ihip.Rope(cos, sin, ihip.ROPE_RELATIVE if args.rope == "relative" else ihip.ROPE_CHUNK_INDEXED,
                         ihip.ROPE_STREAMING)
    cache = ihip.HostKVCache(hk, hv, bt, mask_slots, sa_slots)
    kview = torch.empty((w.B, w.Hkv, w.T, 0), dtype=torch.bfloat16, device=dev)     # shape carrier only
    L = ihip.Layer(qs[0], kview, seq_lens, w.b_q, w.n_sink, w.n_stream)
    ws = L.workspace(ihip.OP_DECODE_LAYER, chunks, keeps)
    out = torch.empty((w.B, w.Hq, 1, w.d), dtype=torch.bfloat16, device=dev)

    def step(i):
        L.decode_layer(qs[i % n_calls], None, None, chunks, keeps, ws=ws, out=out, cache=cache, kv_scales=kv_scales,
                       rope=rope)
        cache.update()

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    s0 = cache.stats()
    t0 = time.perf_counter()
    for i in range(warmup, n_calls):
        step(i)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / steps * 1e6
    s1 = cache.stats()
    kernels = {}
    if not args.no_profile_pass:
        ihip.profile_enable(True)
        for i in range(warmup, n_calls):
            step(i)
        torch.cuda.synchronize()
        ihip.profile_enable(False)
        for name, (ms, n) in ihip.profile_read().items():
            kernels[name] = {"us": ms / n * 1e3, "launches_per_step": n / steps}
    hit = {}
    for bank in ("mask", "sa"):
        h = s1[bank]["hits"] - s0[bank]["hits"]
        m = s1[bank]["misses"] - s0[bank]["misses"]
        hit[bank] = {"block_hits": h, "block_misses": m, "hit_ratio": h / max(1, h + m)}
    cpu = None
    host_link = None
    if args.cpu_seconds > 0 and kv_scales is None and rope is None:
        sample = decode_oracle_sample(w, qs, [(hk, hv)], [w.T], args.cpu_seconds)
        cpu = {"value": sample["seconds"] / sample["layer_calls_one_sequence"] * 1e6, "unit": "us/layer",
               "cores": sample["threads"], "kind": "oracle",
               "sample": f"{sample['layer_calls_one_sequence']} whole layer calls (all {w.Hkv} KV heads) on "
                         f"{sample['threads']} threads, {sample['seconds']:.1f} s of wall time"}
        # bytes that cross the host link per layer call: the rows the kernels read from blocks that are not
        # resident (distinct rows scored, counted by the oracle, x the banks' miss ratios) and the blocks
        # the update copies in afterwards
        P = w.B * w.Hkv
        miss = {b: 1.0 - hit[b]["hit_ratio"] for b in hit}
        first = f"prune_decode.first.l{chunks[0]}"
        first_bytes = P * sample["rows_per_problem"][0] * row_bytes * miss["mask"]
        prune_bytes = P * sum(sample["rows_per_problem"]) * row_bytes * miss["mask"]
        attn_bytes = P * sample["tokens_per_problem"] * 2 * row_bytes * miss["sa"]
        insert_bytes = (min(mask_slots, hit["mask"]["block_misses"] / steps) * bt * row_bytes
                        + min(sa_slots, hit["sa"]["block_misses"] / steps) * bt * 2 * row_bytes)
        host_link = {"est_bytes_per_layer_read_on_misses": prune_bytes + attn_bytes,
                     "bytes_per_layer_inserted": insert_bytes,
                     "est_GBps_over_the_layer": (prune_bytes + attn_bytes + insert_bytes) / (us * 1e-6) / 1e9,
                     "note": "rows read on misses are estimated: oracle-counted distinct rows x block miss ratio"}
        if first in kernels:
            host_link["est_first_stage_GBps"] = first_bytes / (kernels[first]["us"] * 1e-6) / 1e9
    cache.close()
    return {
        "metric": "sparse_attn_decode_offload_us_per_layer" + (f"_dynamic_rope_{args.rope}" if rope else "")
        + ("_fp8_kv" if kv_scales else ""), "value": us, "unit": "us/layer", "steps": steps,
        "warmup": warmup,
        "config": {"workload": w.name, "batch": w.B, "context": w.T, "q_heads": w.Hq, "kv_heads": w.Hkv,
                   "head_dim": w.d, "stages_chunk_keep": list(map(list, w.stages)), "n_sink": w.n_sink,
                   "n_stream": w.n_stream, "block_tokens": bt, "mask_bank_MiB": mask_slots * bt * row_bytes >> 20,
                   "sa_bank_MiB": sa_slots * bt * 2 * row_bytes >> 20, "needles": "Zipf(1.1) over scrambled chunk ranks"},
        "roofline": None, "cpu_baseline": cpu, "cache": hit, "host_link": host_link, "kernels": kernels,
        "setup_s": t_setup,
    }


def extra_workloads(args, torch, ihip, configs, t_run):
    """The other two measured workloads, appended to the default line so that one recorded run carries
    them: `prefill` = one chunked-prefill layer of cfg4 (the second target: matrix-core rate of the
    block-sparse attention and of the first pruning stage), `offload` = the cfg5 decode layer with K/V
    in host memory.  Short runs of the same code `--workload` times; each starts only while the run is
    younger than --extras-budget-s."""
    import copy
    import gc
    out = {}

    def young():
        return time.perf_counter() - t_run < args.extras_budget_s

    gc.collect()
    torch.cuda.empty_cache()
    if young():
        a = copy.copy(args)
        a.steps, a.warmup, a.cpu_seconds, a.no_profile_pass = 10, 3, 0.0, False
        pf = bench_prefill(a, configs.CFG4, torch, ihip, configs)
        first = f"prune_prefill.first.l{configs.CFG4.stages[0][0]}"
        out["prefill"] = {"workload": configs.CFG4.name, "us_per_layer": pf["value"], "steps": pf["steps"],
                          "warmup": pf["warmup"],
                          "kernels_us": {n: kk["us"] for n, kk in pf["kernels"].items()},
                          "roofline": {"attn_prefill": pf["rooflines"].get("attn_prefill"),
                                       "prune_prefill_first_stage": pf["rooflines"].get(first)},
                          "whole_path": pf["whole_path"], "step_us": pf["step_us"]}
        progress("prefill workload done")
        del pf
        gc.collect()
        torch.cuda.empty_cache()
    if young():
        a = copy.copy(args)
        a.steps, a.warmup, a.cpu_seconds, a.no_profile_pass = 16, 4, min(args.cpu_seconds, 3.0), False
        off = bench_offload(a, configs.CFG5, torch, ihip, configs)
        out["offload"] = {"workload": configs.CFG5.name, "us_per_layer": off["value"], "steps": off["steps"],
                          "warmup": off["warmup"], "banks": {kk: off["config"][kk] for kk in ("block_tokens", "mask_bank_MiB", "sa_bank_MiB")},
                          "cache": off["cache"], "host_link": off["host_link"],
                          "kernels_us": {n: kk["us"] for n, kk in off["kernels"].items()}}
        progress("offload workload done")
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; --gpus must be 1 (nothing here shards or uses collectives)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4}))
        return
    import paper_2502_08910_amd as ihip
    from workloads import configs

    ihip.lib()
    w = configs.BY_NAME[args.workload]
    torch.cuda.set_device(0)
    t_run = time.perf_counter()
    if w.name.startswith("cfg5"):
        body = bench_offload(args, w, torch, ihip, configs)
    elif w.Tq == 1:
        body = bench_decode(args, w, torch, ihip, configs)
    else:
        body = bench_prefill(args, w, torch, ihip, configs)
    headline = (w.name == "cfg3-decode-1m-b8" and args.kv_dtype == "bf16" and not args.paged and not args.rope
                and not args.graph and not args.refresh and args.kv_layout == "bhtd")
    if headline and not args.no_extras:
        body.update(extra_workloads(args, torch, ihip, configs, t_run))
    line = {"metric": body.pop("metric"), "value": body.pop("value"), "unit": body.pop("unit"), "n_gpus": 1,
            "steps": body.pop("steps"), "warmup": body.pop("warmup")}
    line["ms_per_step"] = line["value"] / 1e3
    line.update({"higher_is_better": False, "scaling": "weak", "vs_baseline": None,
                 "dtype": "bf16 (K/V stored as fp8 e4m3)" if args.kv_dtype == "fp8" else "bf16",
                 "data": "synthetic"})
    line.update(body)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
