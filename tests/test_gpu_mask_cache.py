"""Decode with per-stage mask caching (refresh intervals) against the oracle's
cached-mask routine, step by step, while the sequences grow."""
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


@pytest.mark.parametrize("refresh", [(4, 2, 1), (1, 1, 1), (6, 3, 3), (3, 4, 2), (2, 5, 3)])
def test_masked_decode_follows_oracle(ihip, orc, refresh):
    """Nested intervals go through ihip_decode_layer_masked ("recompute from stage i on"); intervals
    that are not nested -- a stage due while the next one is not -- through the per-stage flags of
    ihip_decode_layer_ex, which ihip_refresh_due fills from Alg. 4's counters."""
    nested = all(refresh[i] % refresh[i + 1] == 0 for i in range(len(refresh) - 1))
    w = configs.shrink(configs.CFG1, B=2, Hq=8, Hkv=2, T=3000, n_stream=256, n_needles=0,
                       stages=((64, 8), (16, 8), (4, 16)))
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    _, k, v, _, _ = configs.make_inputs(w, 0, kind="int")
    kd, vd = k.cuda(), v.cuda()
    lens0 = [2900, 2200]
    state = None
    cached = {(b, g): [np.zeros(0, np.int64)] * 3 for b in range(w.B) for g in range(w.Hkv)}
    for step in range(13):
        sl = torch.tensor([lens0[0] + step, lens0[1] + 3 * step], dtype=torch.int32)     # sequences grow
        q = configs.make_q(w, 100 + step, kind="int")
        qd, sld = q.cuda(), sl.cuda()
        L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
        if state is None:
            state = L.mask_state(keeps)
        first, due = ihip.refresh_due(step, refresh)
        if nested:
            assert due == [i >= first for i in range(3)]
            out = L.decode_layer_masked(qd, kd, vd, chunks, keeps, first, state)
        else:
            out = L.decode_layer(qd, kd, vd, chunks, keeps, stage_starts=state, stage_due=due)
        torch.cuda.synchronize()
        o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
        P = w.B * w.Hkv
        off = 0
        st_gpu = []
        for keep in keeps:
            st_gpu.append(state[off:off + P * keep].view(P, keep).cpu().numpy())
            off += P * keep
        for b in range(w.B):
            for g in range(w.Hkv):
                kept, bs, bl = o.prune_due(b, g, 0, w.stages, due, cached[(b, g)])
                cached[(b, g)] = kept
                p = b * w.Hkv + g
                for i in range(3):
                    got = st_gpu[i][p]
                    assert got[got >= 0].tolist() == kept[i].tolist(), (step, b, g, i)
                ref, _ = o.attend(b, g, 0, bs, bl)
                err = np.abs(out[b, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy() - ref[:, 0]).max()
                assert err <= 2e-2, (step, b, g, err)
