"""The synthetic-input generator: determinism, distribution, rounding."""
import numpy as np
import torch

import asd_inputs as si


def test_deterministic_and_addressable():
    s = si.SHAPES["tiny"]
    a = si.tensor(s, 0, si.T_WG, 1)
    b = si.tensor(s, 0, si.T_WG, 1)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, si.tensor(s, 1, si.T_WG, 1))
    assert not np.array_equal(a, si.tensor(s, 0, si.T_WU, 1))
    assert not np.array_equal(a, si.tensor(s, 0, si.T_WG, 2))
    # any sub-range can be produced on its own (counter based)
    part = np.empty(100, dtype=np.float32)
    si.lib().synth_fill_f32(part.ctypes.data, 1000, 100, 0, si.T_WG, 1, si.tensor_constant(s, 0, si.T_WG, 1))
    assert np.array_equal(part, a.reshape(-1)[1000:1100])


def test_distribution_matches_recipe():
    s = si.SHAPES["tiny"].with_(d_model=1024, vocab=4096)
    w = si.tensor(s, 0, si.T_EMBED).astype(np.float64)
    assert abs(w.std() - 0.02) < 2e-4
    assert abs(w.mean()) < 1e-4
    assert np.abs(w).max() < 4.9 * 0.02 + 1e-6
    # roughly normal (sum of 8 uniforms is slightly flatter): ~68% within one sigma
    assert abs((np.abs(w) < 0.02).mean() - 0.6827) < 1e-2


def test_bf16_is_round_to_nearest_even_of_fp32_value():
    s32 = si.SHAPES["tiny"]
    s16 = s32.with_(dtype=si.DT_BF16)
    f = si.tensor(s32, 3, si.T_WD, 2)
    b = si.tensor(s16, 3, si.T_WD, 2)
    ref = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(b, ref)


def test_output_scales_and_prompt():
    sc = si.sublayer_scales(0, 32)
    assert sc.shape == (64,) and (sc >= 1e-3).all() and (sc <= 1.0).all()
    assert np.log10(sc).std() > 0.5          # spread over the three decades
    s = si.SHAPES["tiny"]
    wo = si.tensor(s, 0, si.T_WO, 1).astype(np.float64)
    assert abs(wo.std() / (0.02 * sc[2]) - 1.0) < 0.02
    p = si.prompt(0, 512, 32000)
    assert p.min() >= 0 and p.max() < 32000 and len(set(p.tolist())) > 400
    assert np.array_equal(p[:32], si.prompt(0, 32, 32000))


def test_fixed_keep_masks():
    m = si.fixed_keep_mask(32, 2)
    assert m.sum() == 32 and m[0] == 0 and m[1] == 0 and m[2] == 1
    assert si.fixed_keep_mask(32, 4).sum() == 48
