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
    print("cfg3", kind, flush=True)
    check_samples(ihip, orc, configs.CFG3, kind, [(0, 0), (3, 5), (7, 7)])
    torch.cuda.empty_cache()


@pytest.mark.parametrize("kind", ["normal", "int"])
def test_cfg4_prefill_4k_on_256k(ihip, orc, kind):
    """Chunked prefill at full size through the fused ihip_prefill_layer call;
    three (KV head, query block) problems are checked against the oracle."""
    w = configs.CFG4
    dev = torch.device("cuda:0")
    q, k, v, sl, _ = configs.make_inputs(w, 0, device=dev, kind=kind)
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    L = ihip.Layer(q, k, sl, w.b_q, w.n_sink, w.n_stream)
    blocks = torch.empty((L.P, keeps[-1]), dtype=torch.int32, device=dev)
    out = L.prefill_layer(q, k, v, chunks, keeps, out_blocks=blocks)
    torch.cuda.synchronize()
    G = w.G
    for (g, m) in [(0, 0), (3, 31), (7, 63)]:
        print("cfg4", kind, g, m, flush=True)
        p = g * w.Mq + m
        o = orc.Oracle(q[:, g * G:(g + 1) * G].cpu(), k[:, g:g + 1].cpu(), v[:, g:g + 1].cpu(), [w.T],
                       w.b_q, w.n_sink, w.n_stream)
        pr = o.prune(0, 0, m, w.stages)
        got = blocks[p].cpu().numpy()
        got = got[got >= 0]
        want = pr.block_starts
        assert len(got) == len(want) == keeps[-1]
        if kind == "int":
            assert np.array_equal(got, want), (g, m)
        else:
            recall = len(set(got.tolist()) & set(want.tolist())) / len(want)
            assert recall >= 0.99, (g, m, recall)
        ref, _ = o.attend(0, 0, m, pr.block_starts, pr.block_lens)
        err = np.abs(out[0, g * G:(g + 1) * G, m * w.b_q:(m + 1) * w.b_q].float().cpu().numpy() - ref).max()
        assert err <= 2e-2, (g, m, err)
