"""The seeded generators: statistics, slice consistency, needle recipe."""
import torch

from workloads import configs, gen


def test_normal_statistics_and_slices():
    shape = (2, 3, 4096, 64)
    x = gen.normal_bf16(5, 2, shape).float()
    assert abs(x.mean().item()) < 5e-3 and abs(x.std().item() - 1.0) < 5e-3
    assert abs((x ** 4).mean().item() - 3.0) < 0.05
    assert abs((x[..., :-1] * x[..., 1:]).mean().item()) < 5e-3          # neighbours along d
    assert abs((x[:, :, :-1] * x[:, :, 1:]).mean().item()) < 5e-3        # neighbours along t
    s = gen.normal_bf16(5, 2, shape, sl=(1, 2, 2, 3, 100, 300))
    assert torch.equal(s[0, 0], gen.normal_bf16(5, 2, shape)[1, 2, 100:300])
    assert not torch.equal(gen.normal_bf16(6, 2, shape), gen.normal_bf16(5, 2, shape))
    assert not torch.equal(gen.normal_bf16(5, 3, shape), gen.normal_bf16(5, 2, shape))


def test_small_ints():
    y = gen.small_int_bf16(0, 2, (1, 2, 2048, 128)).float()
    assert set(y.unique().tolist()) == {-2.0, -1.0, 0.0, 1.0, 2.0}
    for val in range(-2, 3):
        assert abs((y == val).float().mean().item() - 0.2) < 0.01


def test_fill_matches_direct():
    out = torch.empty((2, 2, 300, 16), dtype=torch.bfloat16)
    gen.fill_(out, 9, 2, t_step=128)
    assert torch.equal(out, gen.normal_bf16(9, 2, (2, 2, 300, 16)))


def test_needle_recipe():
    w = configs.CFG1
    q, k, v, sl, pos = configs.make_inputs(w, 0)
    assert pos.shape == (1, 8, 16)
    l1 = w.stages[0][0]
    assert ((pos - w.n_sink) % l1 == 0).all()
    assert (pos >= w.n_sink).all() and (pos < w.T - w.n_stream).all()
    for g in range(w.Hkv):
        assert len(set(pos[0, g].tolist())) == 16
        for i in range(16):
            h = g * w.G + i % w.G
            qv = q[0, h, 0].float()
            s = (qv @ k[0, g, pos[0, g, i]].float()).item()
            assert abs(s - 4.0 * qv.norm().item()) < 0.5 * qv.norm().item()   # noise: 0.1|q| rms


def test_zipf_is_heavy_headed():
    r = gen.zipf_ranks(0, 9, 20000, 1000)
    assert (r == 0).float().mean() > 0.1 and (r < 10).float().mean() > 0.3
    assert r.max() > 500
