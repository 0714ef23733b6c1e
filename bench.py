#!/usr/bin/env python3
"""Benchmark of the decode hot path: one step = one layer call (all pruning
stages + arg-top-K selects + block-sparse decode attention, every stage
refreshed) over one batch of synthetic input resident in HBM.

Default workload: cfg3 -- batch 8, 1,048,576 keys per sequence, 32 query / 8
KV heads, d = 128, bf16, 4 stages (256 -> 64 -> 16 -> 4), 4,096-token budget.
One layer's K/V (32 GiB) stays in HBM and is reused by 32 different query
sets, so consecutive steps touch different rows.

Prints one JSON line.  `value` is microseconds per layer call for the whole
batch.  `roofline` is for the kernel with the largest share of the step:
algorithmic bytes per launch (distinct K rows the search must score, counted
by the CPU oracle on a sample of problems, plus the scores it writes) divided
by that kernel's mean duration, measured with HIP events around the launch on
its stream in a second pass over the same steps.  `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same workload in the same run.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
N_QUERY_SETS = 32

# HBM traffic per launch of the dominant kernel from rocprofv3 --pmc runs
# (FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size); see
# profiles/.  None until measured for a workload.
MEASURED_TRAFFIC_BYTES = {
    # FETCH_SIZE 781,266 KiB x 2.0 (copy-kernel scale) + WRITE_SIZE 1,220 KiB x 1.0 per launch
    ("cfg3-decode-1m-b8", "prune_decode.first.l256"): (781265.9 * 2.0 + 1220.0) * 1024.0,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3-decode-1m-b8")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="CPU time budget of the oracle baseline (0 = skip)")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run 10 device copies of 1 GiB (a kernel of known traffic, to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters) and exit")
    return ap.parse_args()


def oracle_sample(w, qs, k, v, seq_lens, budget_s):
    """Times the CPU oracle on sequence 0 (all its KV heads), one query set
    after another until the budget is used; also returns the mean number of
    distinct K rows each stage scores per problem and the attended tokens."""
    import numpy as np
    import oracle
    oracle.build(force=False)
    k0 = k[0:1].cpu()
    v0 = v[0:1].cpu()
    rows = [0.0] * len(w.stages)
    tokens, problems, calls = 0.0, 0, 0
    t_used = 0.0
    for i, q in enumerate(qs):
        o = oracle.Oracle(q[0:1].cpu(), k0, v0, [int(seq_lens[0])], w.b_q, w.n_sink, w.n_stream)
        t0 = time.perf_counter()
        res = o.layer(w.stages)
        t_used += time.perf_counter() - t0
        calls += 1
        for (b, g, m), (pr, out, lse) in res.items():
            for s, st in enumerate(pr.stages):
                rows[s] += st.rows_touched
            tokens += o.attended_tokens(b, m, pr.block_lens)
            problems += 1
        if t_used >= budget_s:
            break
    return {
        "seconds": t_used, "layer_calls_one_sequence": calls, "problems": problems,
        "rows_per_problem": [r / problems for r in rows], "tokens_per_problem": tokens / problems,
    }


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
    if w.Tq != 1:
        print("bench.py: only decode workloads are timed here", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]

    t0 = time.perf_counter()
    k, v = configs.make_kv(w, 0, dev)
    qs = []
    for i in range(N_QUERY_SETS):
        q = configs.make_q(w, i, dev)
        configs.plant_needles(w, k, q, i)
        qs.append(q)
    seq_lens = torch.full((w.B,), w.T, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t0

    L = ihip.Layer(qs[0], k, seq_lens, w.b_q, w.n_sink, w.n_stream)
    ws = L.workspace(ihip.OP_DECODE_LAYER, chunks, keeps)
    out = torch.empty((w.B, w.Hq, 1, w.d), dtype=torch.bfloat16, device=dev)

    def step(i):
        L.decode_layer(qs[i % N_QUERY_SETS], k, v, chunks, keeps, ws=ws, out=out)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    us_per_layer = elapsed / args.steps * 1e6

    # second pass over the same steps with HIP events around every kernel launch
    kernels = {}
    if not args.no_profile_pass:
        ihip.profile_enable(True)
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        ihip.profile_enable(False)
        for name, (ms, n) in ihip.profile_read().items():
            kernels[name] = {"us": ms / n * 1e3, "launches_per_step": n / args.steps}

    # CPU oracle on a bounded sample: timing + algorithmic byte counts
    cpu = None
    sample = None
    if args.cpu_seconds > 0:
        sample = oracle_sample(w, qs, k, v, seq_lens.cpu().tolist(), args.cpu_seconds)
        per_seq_call = sample["seconds"] / sample["layer_calls_one_sequence"]
        cpu = {"value": per_seq_call * w.B * 1e6, "unit": "us/layer", "cores": 1, "kind": "oracle",
               "sample": f"sequence 0 of {w.B} (its {w.Hkv} KV heads), {sample['layer_calls_one_sequence']} "
                         f"layer calls with different queries, {sample['seconds']:.1f} s; scaled x{w.B} to the batch"}

    P = w.B * w.Hkv
    row_bytes = w.d * 2
    roofline = None
    alg = {}
    if sample is not None:
        slots = [L.stage1_slots(chunks[0])] + [keeps[i - 1] * (chunks[i - 1] // chunks[i])
                                                 for i in range(1, len(chunks))]
        for i, c in enumerate(chunks):
            name = f"prune_decode.first.l{c}" if i == 0 else f"prune_decode.l{c}"
            alg[name] = P * (sample["rows_per_problem"][i] * row_bytes + slots[i] * 4)
            sname = f"select_blocks.first.l{c}" if i == 0 else f"select_blocks.l{c}"
            alg[sname] = P * (slots[i] * 4 + keeps[i] * 4)
        alg["attn_decode_split"] = P * sample["tokens_per_problem"] * 2 * row_bytes
        total_alg = sum(alg.values())
        if kernels:
            dom = max(kernels, key=lambda n: kernels[n]["us"] * kernels[n]["launches_per_step"])
            if dom in alg:
                ach = alg[dom] / (kernels[dom]["us"] * 1e-6) / 1e9
                roofline = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                            "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                            "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, dom)),
                            "algorithmic_bytes_per_launch": alg[dom], "us_per_launch": kernels[dom]["us"]}
            for n in kernels:
                if n in alg:
                    kernels[n]["alg_GBps"] = alg[n] / (kernels[n]["us"] * 1e-6) / 1e9
    else:
        total_alg = None

    line = {
        "metric": "sparse_attn_decode_us_per_layer_1m_ctx",
        "value": us_per_layer, "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": us_per_layer / 1e3, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.B, "context": w.T, "q_heads": w.Hq, "kv_heads": w.Hkv,
                   "head_dim": w.d, "stages_chunk_keep": list(map(list, w.stages)), "n_sink": w.n_sink,
                   "n_stream": w.n_stream, "query_sets": N_QUERY_SETS},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "whole_path": None if total_alg is None else {
            "algorithmic_bytes_per_layer": total_alg,
            "achieved_GBps": total_alg / (us_per_layer * 1e-6) / 1e9,
            "frac_of_hbm_peak": total_alg / (us_per_layer * 1e-6) / 1e9 / HBM_PEAK_GBS},
        "kernels": kernels,
        "setup_s": t_setup,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
