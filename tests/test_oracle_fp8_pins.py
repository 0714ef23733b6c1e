"""Pins of the oracle's FP8 (E4M3) KV-cache option: the byte decoder against
torch's float8_e4m3fn, and the whole path against the bf16 path run on the
dequantised values (which bf16 holds exactly when the scale is a power of two)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import Oracle
from workloads import gen


def test_e4m3_decoder_matches_torch_for_every_byte():
    L = oracle.lib()
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    got = np.array([L.orc_e4m3_to_f32(i) for i in range(256)], np.float32)
    nan = np.isnan(ref)
    assert nan.sum() == 2 and np.array_equal(np.isnan(got), nan)        # 0x7f and 0xff
    assert np.array_equal(got[~nan], ref[~nan])
    # landmarks of the format: largest finite 448, smallest subnormal 2^-9, one = 0x38
    assert got[0x7e] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x38] == 1.0 and got[0xb8] == -1.0


@pytest.mark.parametrize("scales", [(1.0, 1.0), (0.25, 2.0)])
def test_fp8_kv_equals_bf16_path_on_dequantised_values(scales):
    torch.manual_seed(0)
    B, Hq, Hkv, T, d = 1, 4, 2, 900, 128
    q = torch.randn(B, Hq, 1, d).to(torch.bfloat16)
    k8 = gen.to_e4m3(torch.randn(B, Hkv, T, d), scales[0])
    v8 = gen.to_e4m3(torch.randn(B, Hkv, T, d), scales[1])
    kd = (k8.view(torch.float8_e4m3fn).float() * scales[0])
    vd = (v8.view(torch.float8_e4m3fn).float() * scales[1])
    assert torch.equal(kd, kd.to(torch.bfloat16).float())               # bf16 holds them exactly
    o8 = Oracle(q, k8, v8, [T], 1, 16, 64, kv_scales=scales)
    ob = Oracle(q, kd.to(torch.bfloat16), vd.to(torch.bfloat16), [T], 1, 16, 64)
    stages = [(32, 8), (8, 12), (2, 20)]
    for g in range(Hkv):
        a, b = o8.prune(0, g, 0, stages), ob.prune(0, g, 0, stages)
        for sa, sb in zip(a.stages, b.stages):
            assert np.array_equal(sa.scores, sb.scores) and np.array_equal(sa.reps, sb.reps)
            assert np.array_equal(sa.kept_ids, sb.kept_ids)
        oa, la = o8.attend(0, g, 0, a.block_starts, a.block_lens)
        obb, lb = ob.attend(0, g, 0, b.block_starts, b.block_lens)
        assert np.array_equal(oa, obb) and np.array_equal(la, lb)


def test_quantiser_saturates_and_rounds_to_nearest():
    x = torch.tensor([0.0, 1.0, 1.0625, 1.07, 500.0, -1000.0, 2.0 ** -10])
    b = gen.to_e4m3(x, 1.0)
    back = b.view(torch.float8_e4m3fn).float()
    # 1.0625 and 2^-10 are exact ties: to the even mantissa
    assert back.tolist() == [0.0, 1.0, 1.0, 1.125, 448.0, -448.0, 0.0]
