"""The paper's printed presets (tests/golden/paper_presets.txt) against the oracle's structure and
the host logic of the refresh rule: the stage plan they imply runs through Alg. 1 with exactly the
chunk counts the printed budgets fix, the final window has the size the presets are named after,
and Alg. 4's counters re-run stage i exactly once per n_refresh^(i) steps."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import Oracle
from workloads import gen

pytestmark = pytest.mark.usefixtures("oracle_lib")


def presets():
    out = {}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_presets.txt")
    for line in open(path):
        line = line.split("#")[0].split()
        if line:
            out[line[0]] = [int(x) for x in line[1:]]
    return out


def test_preset_names_are_the_final_window_sizes():
    p = presets()
    assert p["k_3_default"][0] + p["n_stream"][0] == p["window_default"][0]      # the "3K" preset
    assert p["k_3_5k_preset"][0] + p["n_stream"][0] == p["window_5k"][0]         # the "5K" preset


@pytest.mark.parametrize("k3_key", ["k_3_default", "k_3_first_layers"])
def test_default_preset_runs_through_alg1_with_the_printed_budgets(k3_key):
    p = presets()
    l_c = p["l_c"]
    k = p["k_1_2"] + p[k3_key]
    stages = tuple((l, kk // l) for l, kk in zip(l_c, k))            # chunks kept = k^(i) / l_c^(i)
    assert [s[1] for s in stages][:2] == [128, 256]
    n_sink, n_stream = p["n_sink"][0], p["n_stream"][0]
    T, d = n_sink + n_stream + 152 * l_c[0], 16       # a middle range of whole first-stage chunks
    q = gen.normal_bf16(0, 1, (1, 2, 1, d))
    kk = gen.normal_bf16(0, 2, (1, 1, T, d))
    v = gen.normal_bf16(0, 3, (1, 1, T, d))
    o = Oracle(q, kk, v, [T], 1, n_sink, n_stream)
    pr = o.prune(0, 0, 0, stages)
    mid = T - n_sink - n_stream
    want_candidates = [math.ceil(mid / l_c[0]), stages[0][1] * (l_c[0] // l_c[1]), stages[1][1] * (l_c[1] // l_c[2])]
    assert [len(st.starts) for st in pr.stages] == want_candidates
    assert [len(st.kept_ids) for st in pr.stages] == [s[1] for s in stages]
    assert int(pr.block_lens.sum()) == p[k3_key][0]                   # k^(3) tokens survive
    assert o.attended_tokens(0, 0, pr.block_lens) == n_sink + p[k3_key][0] + n_stream
    # every stage's survivors lie inside the stage before's
    for a, b in zip(pr.stages[:-1], pr.stages[1:]):
        parents = set(a.kept_starts.tolist())
        assert all((int(s) - n_sink) // a.l_c * a.l_c + n_sink in parents for s in b.kept_starts)


@pytest.mark.parametrize("name", ["n_refresh_default", "n_refresh_fast", "n_refresh_flash"])
def test_refresh_rule_reruns_stage_i_once_per_interval(name):
    """Alg. 4 with the printed intervals: counters start at 0, stage i runs when c^(i) mod n^(i) = 0 and the
    counters advance by one per generated token.  The library has the rule in ihip_refresh_due (host
    arithmetic in the C library); simulate the counters literally and compare."""
    from paper_2502_08910_amd.binding import first_stage_due, refresh_due
    n = presets()[name]
    steps = 2 * math.lcm(*n)
    c = [0] * len(n)
    runs = [0] * len(n)
    for step in range(steps):
        due = [ci % ni == 0 for ci, ni in zip(c, n)]
        first = first_stage_due(step, n)
        # the intervals are nested (each a multiple of the next), so a due stage makes every later one due
        assert due == [i >= first for i in range(len(n))], (step, due, first)
        assert refresh_due(step, n) == (first, due)
        for i, d_ in enumerate(due):
            runs[i] += d_
        c = [(ci + 1) % ni for ci, ni in zip(c, n)]
    assert runs == [steps // ni for ni in n]


def test_alg4_stage_loop_with_intervals_that_are_not_nested():
    """Alg. 4's stage loop, simulated literally over decode steps with counters c^(i) and intervals
    (3, 4, 2) -- at step 3 the first stage is due and the second is not, at step 4 the second and third
    are due and the first is not --, against Oracle.prune_due driven by the library's ihip_refresh_due.
    The literal loop below keeps its own lists and calls only the single-stage routine."""
    from oracle.pipeline import stage1_chunks, child_chunks
    from paper_2502_08910_amd.binding import refresh_due
    from workloads import configs
    w = configs.shrink(configs.CFG1, T=2048 + 64, n_stream=256, n_needles=0, stages=((64, 8), (16, 8), (4, 16)))
    n_refresh = (3, 4, 2)
    _, k, v, _, _ = configs.make_inputs(w, 0, kind="int")
    N = len(w.stages)
    c = [0] * N                                                   # Alg. 4: c^(i) <- 0
    lists = [np.zeros(0, np.int64)] * N                           # I^(l,i) of the literal loop
    cached = [np.zeros(0, np.int64)] * N                          # the same, handed to prune_due
    patterns = set()
    for step in range(13):
        T = 2048 + 5 * step                                       # the sequence grows
        q = configs.make_q(w, 50 + step, kind="int")
        o = Oracle(q, k, v, [T], 1, w.n_sink, w.n_stream)
        lo, hi, _ = o.ranges(0, 0)
        for i, (l_c, keep) in enumerate(w.stages):                # for each stage i = 1..N
            if c[i] % n_refresh[i] == 0:                          #   if c^(i) mod n_refresh^(i) = 0: run stage i on I^(<i)
                if i == 0:
                    starts, lens = stage1_chunks(lo, hi, l_c)
                else:
                    plens = np.minimum(w.stages[i - 1][0], hi - lists[i - 1]).astype(np.int32)
                    starts, lens = child_chunks(lists[i - 1], plens, l_c)
                lists[i] = o.prune_stage(0, 1, 0, starts, lens, l_c, keep).kept_starts
        first, due = refresh_due(step, n_refresh)
        assert due == [ci % ni == 0 for ci, ni in zip(c, n_refresh)]
        patterns.add(tuple(due))
        cached, bs, bl = o.prune_due(0, 1, 0, w.stages, due, cached)
        assert [x.tolist() for x in cached] == [x.tolist() for x in lists], step
        assert bs.tolist() == lists[-1].tolist()
        assert (bs + bl <= hi).all() and (bl >= 1).all()
        c = [(ci + 1) % ni for ci, ni in zip(c, n_refresh)]       # c^(i) <- (c^(i) + 1) mod n_refresh^(i)
    assert (True, False, False) in patterns and (False, True, True) in patterns and (True, False, True) in patterns
