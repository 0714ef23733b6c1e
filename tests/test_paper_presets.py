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
    counters advance by one per generated token.  The library exposes the rule as 'first stage to
    recompute' (host logic in the binding); simulate the counters literally and compare."""
    from paper_2502_08910_amd.binding import first_stage_due
    n = presets()[name]
    steps = 2 * math.lcm(*n)
    c = [0] * len(n)
    runs = [0] * len(n)
    for step in range(steps):
        due = [ci % ni == 0 for ci, ni in zip(c, n)]
        first = first_stage_due(step, n)
        # the intervals are nested (each a multiple of the next), so a due stage makes every later one due
        assert due == [i >= first for i in range(len(n))], (step, due, first)
        for i, d_ in enumerate(due):
            runs[i] += d_
        c = [(ci + 1) % ni for ci, ni in zip(c, n)]
    assert runs == [steps // ni for ni in n]
