"""GPU checks of the loop extensions: adaptive draft exit, MLP-side CS thresholding, mask refresh.

The paper defines none of them, so what is compared is what any reading must satisfy (the output equals the
GPU's own plain greedy decode, bit for bit), the neutral corners against the fixed-length loop, and, on the fp32
shape where no decision sits near its threshold, the cycle-by-cycle statistics against the oracle's loop.
"""
import numpy as np
import pytest

import asd_inputs as si
import oracle
import paper_2410_01028_amd as asd
from test_gpu_parity import MID16, build_pair

pytestmark = pytest.mark.gpu

KEYS = ("cycles", "drafted", "accepted", "emitted")


@pytest.mark.parametrize("shape", [si.SHAPES["tiny"], MID16], ids=lambda s: s.name)
def test_adaptive_exit_corners_and_plain_equality(shape):
    eng = asd.Engine(asd.make_config(shape, 256)).init_synthetic(3)
    prompt = si.prompt(2, 40, shape.vocab)
    N = 40
    plain, _, _ = eng.generate(prompt, N, 0)
    fixed, st_f, _ = eng.generate(prompt, N, 4, alpha=0.9, m=2, n=1)
    assert np.array_equal(fixed, plain)
    for graphs in (False, True):
        # a threshold no probability falls below: the fixed-length loop
        out, st, _ = eng.generate(prompt, N, 4, alpha=0.9, m=2, n=1, exit_mode=1, gamma0=0.0, eps=0.0, use_graphs=graphs)
        assert np.array_equal(out, plain) and all(st[k] == st_f[k] for k in KEYS)
        # a threshold above every probability: one draft per cycle
        one, st_1, _ = eng.generate(prompt, N, 1, alpha=0.9, m=2, n=1, use_graphs=graphs)
        out, st, _ = eng.generate(prompt, N, 4, alpha=0.9, m=2, n=1, exit_mode=1, gamma0=1.5, eps=0.0, use_graphs=graphs)
        assert np.array_equal(out, plain) and all(st[k] == st_1[k] for k in KEYS)
        # moving thresholds, both graph modes
        for g0 in (0.01, 0.05, 0.3):
            out, st, _ = eng.generate(prompt, N, 5, alpha=0.9, m=2, n=1, exit_mode=1, gamma0=g0, ar0=1.0, ar_target=0.6,
                                      eps=0.02, beta1=0.5, beta2=0.8, use_graphs=graphs)
            assert np.array_equal(out, plain) and st["emitted"] == N and st["drafted"] <= 5 * st["cycles"]


def test_adaptive_exit_statistics_against_oracle():
    shape = si.SHAPES["tiny"]
    eng, orc = build_pair(shape, seed=6, max_seq=128)
    prompt = si.prompt(7, 24, shape.vocab)
    N = 32
    checked = 0
    for g0, target in ((0.02, 0.5), (0.05, 0.8), (0.1, 0.3), (0.004, 0.9)):
        kw = dict(alpha=0.9, m=2, n=1, exit_mode=1, gamma0=g0, ar0=1.0, ar_target=target, eps=0.01, beta1=0.5, beta2=0.9)
        want, wst, wmask, _, per = orc.generate_adaptive(prompt, N, 5, **kw)
        got, gst, gmask = eng.generate(prompt, N, 5, **kw)
        assert np.array_equal(got, want) and np.array_equal(gmask, wmask)
        assert all(gst[k] == wst[k] for k in KEYS), (g0, gst, wst)
        assert abs(gst["gamma"] - wst["gamma"]) < 1e-12 and abs(gst["ar"] - wst["ar"]) < 1e-12
        checked += int((per[:-1, 0] < 5).any())
    assert checked >= 2          # several of the settings do stop cycles early


def test_mask_refresh_and_mlp_thresholding():
    shape = si.SHAPES["tiny"]
    eng, orc = build_pair(shape, seed=9, max_seq=160)
    prompt = si.prompt(3, 20, shape.vocab)
    N = 40
    plain, _, _ = eng.generate(prompt, N, 0)
    # where the ACS of the prompt and of the whole sequence lie apart most: a threshold between the two must flip
    _, C_prompt, _ = eng.prefill(prompt)
    _, C_final, _ = eng.prefill(np.concatenate([prompt, plain[:N - 1]]))
    j = int(np.argmax(np.abs(C_prompt[0::2] - C_final[0::2])))
    alpha = float((C_prompt[2 * j] + C_final[2 * j]) / 2)
    assert abs(C_prompt[2 * j] - C_final[2 * j]) > 1e-4
    for graphs in (False, True):
        out, st, mask = eng.generate(prompt, N, 3, alpha=alpha, m=0, n=0, refresh=True, use_graphs=graphs)
        assert np.array_equal(out, plain)
        assert st["mask_changes"] >= 1
        assert np.array_equal(mask, asd.admg2(C_final, alpha, 0, 0))
        assert not np.array_equal(mask, asd.admg2(C_prompt, alpha, 0, 0))
    want, wst, wmask, _, _ = orc.generate_adaptive(prompt, N, 3, alpha=alpha, m=0, n=0, refresh=True)
    assert np.array_equal(want, plain) and np.array_equal(wmask, mask) and all(st[k] == wst[k] for k in KEYS)
    # MLP-side thresholding: the mask in effect is Algorithm 1's plus the MLPs whose ACS reaches the threshold
    amlp = float(np.sort(C_prompt[1::2])[-2])          # the two most similar MLP sublayers qualify (rule 2 may protect them)
    out, st, mask = eng.generate(prompt, N, 3, alpha=0.999, m=0, n=1, alpha_mlp=amlp, use_cs_mlp=True)
    assert np.array_equal(out, plain)
    assert np.array_equal(mask, asd.admg2(C_prompt, 0.999, 0, 1, True, amlp, True)) and mask[1::2].sum() >= 1


def test_generation_parameter_validation():
    shape = si.SHAPES["tiny"]
    eng = asd.Engine(asd.make_config(shape, 64)).init_synthetic(0)
    for kw in (dict(exit_mode=2), dict(exit_mode=1, beta1=1.5), dict(exit_mode=1, eps=-0.1), dict(exit_mode=1, gamma0=float("nan")),
               dict(use_cs_mlp=True, alpha_mlp=1.5)):
        with pytest.raises(asd.AsdError):
            eng.generate([1, 2, 3], 4, 2, **kw)
