"""ihip_decode_layer_static (the decode layer on the library's static scratch, for callers that
cannot allocate) against ihip_decode_layer on a caller workspace: same kernels, so the outputs, the
log-sum-exp and the final block lists must be bit-identical -- on two calls in a row, the second
with a smaller input, so that whatever the first call left in the scratch is seen not to matter.
The kept lists are also held against the oracle (integer inputs: bit-exact)."""
import ctypes

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


def _one_call(ihip, orc, w, seed, kind):
    chunks = [s[0] for s in w.stages]
    keeps = [s[1] for s in w.stages]
    q, k, v, sl, _ = configs.make_inputs(w, seed, kind=kind)
    sl = sl.clone()
    sl[-1] -= 37                                   # a ragged last sequence
    qd, kd, vd, sld = (t.cuda() for t in (q, k, v, sl))
    L = ihip.Layer(qd, kd, sld, 1, w.n_sink, w.n_stream)
    P = L.P
    # the reference: the existing entry point on a workspace of the caller's
    ref_blocks = torch.empty((P, keeps[-1]), dtype=torch.int32, device="cuda")
    ref_lse = torch.empty((w.B, w.Hq), dtype=torch.float32, device="cuda")
    ref_out = L.decode_layer(qd, kd, vd, chunks, keeps, out_blocks=ref_blocks, lse=ref_lse)
    # the static variant: outputs allocated up front, then nothing but the call
    out = torch.full((w.B, w.Hq, 1, w.d), 7.0, dtype=torch.bfloat16, device="cuda")
    blocks = torch.full((P, keeps[-1]), -7, dtype=torch.int32, device="cuda")
    lse = torch.full((w.B, w.Hq), 7.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    L.decode_layer_static(qd, kd, vd, chunks, keeps, out, out_blocks=blocks, lse=lse)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(blocks, ref_blocks), (w.name, seed, kind)
    assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16)), (w.name, seed, kind)
    assert torch.equal(lse, ref_lse), (w.name, seed, kind)
    # and the oracle on the same inputs
    o = orc.Oracle(q, k, v, sl.tolist(), 1, w.n_sink, w.n_stream)
    for b in range(w.B):
        for g in range(w.Hkv):
            pr = o.prune(b, g, 0, w.stages)
            got = blocks[b * w.Hkv + g].cpu().numpy()
            got = got[got >= 0]
            if kind == "int":
                assert np.array_equal(got, pr.block_starts), (b, g)
            else:
                want = set(pr.block_starts.tolist())
                assert len(want & set(got.tolist())) >= 0.99 * len(want), (b, g)
            ref, _ = o.attend(b, g, 0, pr.block_starts, pr.block_lens)
            if kind == "int":
                err = np.abs(out[b, g * w.G:(g + 1) * w.G, 0].float().cpu().numpy() - ref[:, 0]).max()
                assert err <= 2e-2, (b, g, err)


def test_static_scratch_two_calls_in_a_row(ihip, orc):
    big = configs.shrink(configs.CFG1, B=2, T=20000 + 11, n_needles=0,
                         stages=((64, 48), (16, 64), (4, 96)))
    small = configs.shrink(configs.CFG1, B=1, Hq=8, Hkv=2, T=3000 + 5, n_stream=256, n_needles=0,
                           stages=((64, 8), (16, 8), (4, 16)))
    _one_call(ihip, orc, big, 3, "int")
    _one_call(ihip, orc, small, 4, "int")          # smaller: the scratch still holds the first call's data
    _one_call(ihip, orc, big, 5, "normal")
    _one_call(ihip, orc, small, 6, "normal")


def test_static_scratch_refuses_what_does_not_fit(ihip):
    from paper_2502_08910_amd.binding import Shape, Tensor
    L = ihip.lib()
    sl = torch.full((64,), 1 << 20, dtype=torch.int32, device="cuda")
    s = Shape(64, 32, 8, 128, 1, 1, sl.data_ptr(), 1 << 20, 128, 1024, 0)     # batch 64 x 1M keys: ~ 33 MiB of scores
    t = Tensor(256, 0, 0, 128)
    chunks = (ctypes.c_int32 * 2)(256, 16)
    keeps = (ctypes.c_int32 * 2)(256, 256)
    rc = L.ihip_decode_layer_static(ctypes.byref(s), t, t, t, 2, chunks, keeps, 1.0, 256, None, None, None)
    assert rc == -2 and b"static" in L.ihip_last_error()
