"""Pins of the oracle's loop extensions: adaptive draft exit, MLP-side CS thresholding, mask refresh.

None of the three is defined by the paper's text (Section 4 cites the draft-exit mechanism of another paper
without printing it), so they are pinned by what must hold whatever the reading: closed forms of the small
functions, reduction to the already-pinned fixed-length loop in the neutral corner, token equality with plain
greedy decoding for any parameters, and the running ACS being the ACS of one teacher-forced pass.
"""
import itertools

import numpy as np
import pytest
from scipy.special import softmax

import asd_inputs as si
import oracle
from helpers import SMALL_GQA, SMALL_MHA, make_oracle


def test_top1_probability_closed_forms_and_softmax():
    assert oracle.top1_prob(np.zeros(7)) == pytest.approx(1 / 7, rel=1e-15)
    assert oracle.top1_prob([np.log(3.0), 0, 0, 0]) == pytest.approx(0.5, rel=1e-15)
    assert oracle.top1_prob([1000.0, 0.0]) == pytest.approx(1.0, rel=1e-15)          # no overflow
    assert oracle.top1_prob([-1000.0, -1000.0]) == pytest.approx(0.5, rel=1e-15)      # no underflow to 0/0
    rng = np.random.default_rng(0)
    for _ in range(50):
        lg = rng.normal(0, 3, int(rng.integers(2, 400)))
        assert oracle.top1_prob(lg) == pytest.approx(softmax(lg).max(), rel=1e-13)


def test_exit_update_closed_forms():
    # no smoothing: AR is this cycle's rate, gamma moves by exactly eps in the direction the rate dictates
    assert oracle.exit_update(0.3, 0.5, 3, 4, 0.9, 0.02, 0.0, 0.0) == pytest.approx((0.75, 0.52), rel=1e-15)
    assert oracle.exit_update(0.3, 0.5, 4, 4, 0.9, 0.02, 0.0, 0.0) == pytest.approx((1.0, 0.48), rel=1e-15)
    # AR exactly at the target counts as "not above": gamma rises
    assert oracle.exit_update(0.0, 0.5, 9, 10, 0.9, 0.02, 0.0, 0.0)[1] == pytest.approx(0.52, rel=1e-15)
    # full smoothing: nothing moves except gamma towards itself
    assert oracle.exit_update(0.3, 0.5, 4, 4, 0.9, 0.02, 1.0, 1.0) == pytest.approx((0.3, 0.5), rel=1e-15)
    # geometric approach of AR to a constant rate r: AR_t = r + (AR_0 - r) beta1^t; gamma_t = gamma_0 -+ t (1-beta2) eps
    ar, g, r, b1, b2, eps = 0.2, 0.6, 1.0, 0.7, 0.9, 0.01
    for t in range(1, 30):
        ar, g = oracle.exit_update(ar, g, 5, 5, 0.5, eps, b1, b2)
        assert ar == pytest.approx(r + (0.2 - r) * b1 ** t, rel=1e-12)
    # AR rose above 0.5 after the second update: one step up, then steps down
    first_above = next(t for t in range(1, 30) if 1.0 + (0.2 - 1.0) * b1 ** t > 0.5)
    ups, downs = first_above - 1, 29 - (first_above - 1)
    assert g == pytest.approx(0.6 + (ups - downs) * (1 - b2) * eps, rel=1e-12)


def test_mlp_thresholding_reduces_to_algorithm_1_and_brute_force():
    rng = np.random.default_rng(3)
    for _ in range(200):
        L = int(rng.integers(1, 30))
        C = rng.uniform(0.9, 1.0, 2 * L)
        alpha, m, n = float(rng.uniform(0.9, 1.0)), int(rng.integers(0, 6)), int(rng.integers(0, 5))
        base = oracle.admg(C[0::2], alpha, m, n)
        assert np.array_equal(oracle.admg2(C, alpha, m, n), base)                     # rule off
        assert np.array_equal(oracle.admg2(C, alpha, m, n, True, 1.5, True), base)    # threshold nothing reaches
        every = oracle.admg2(C, alpha, m, n, True, 0.0, True)                         # threshold everything reaches
        assert (every[1::2][:max(L - n, 0)] == 1).all() and (every[1::2][max(L - n, 0):] == 0).all()
        assert np.array_equal(every[0::2], base[0::2])                                # attention half untouched
    # every above/below pattern of both halves for small L against set algebra
    for L in (1, 2, 3):
        for pat in itertools.product([0.5, 0.99], repeat=2 * L):
            for m in range(0, L + 1):
                for n in range(0, L + 1):
                    mask = oracle.admg2(np.array(pat), 0.9, m, n, True, 0.9, True)
                    for l in range(1, L + 1):
                        freed, per = l <= L - n, (m > 0 and l % m == 0)
                        assert mask[2 * l - 2] == (freed and (pat[2 * l - 2] >= 0.9 or per))
                        assert mask[2 * l - 1] == (freed and (pat[2 * l - 1] >= 0.9 or per))


@pytest.mark.parametrize("shape", [SMALL_GQA, SMALL_MHA], ids=lambda s: s.name)
def test_neutral_corner_equals_the_fixed_length_loop(shape):
    orc = make_oracle(shape, seed=3)
    prompt = si.prompt(4, 9, shape.vocab)
    for k, alpha, m, n in ((3, 0.9, 2, 1), (4, 0.999, 0, 0), (1, 0.5, 3, 0)):
        want = orc.generate_spec(prompt, 14, k, alpha, m, n)
        got = orc.generate_adaptive(prompt, 14, k, alpha, m, n)
        assert np.array_equal(got[0], want[0]) and np.array_equal(got[2], want[2])
        for key in ("cycles", "drafted", "accepted", "emitted"):
            assert got[1][key] == want[1][key]
        assert np.allclose(got[3], want[3], rtol=0, atol=0)
        # a threshold no confidence can fall below never stops a cycle early either
        same = orc.generate_adaptive(prompt, 14, k, alpha, m, n, exit_mode=1, gamma0=0.0, eps=0.0)
        assert same[1]["drafted"] == want[1]["drafted"] and same[1]["cycles"] == want[1]["cycles"]


def test_threshold_above_one_drafts_one_token_per_cycle():
    shape = SMALL_GQA
    orc = make_oracle(shape, seed=5)
    prompt = si.prompt(1, 7, shape.vocab)
    one = orc.generate_spec(prompt, 12, 1, 0.9, 2, 1)
    got = orc.generate_adaptive(prompt, 12, 5, 0.9, 2, 1, exit_mode=1, gamma0=1.5, eps=0.0)
    assert np.array_equal(got[0], one[0])
    assert (got[4][:, 0] <= 1).all()
    for key in ("cycles", "drafted", "accepted"):
        assert got[1][key] == one[1][key]


@pytest.mark.parametrize("shape", [SMALL_GQA, SMALL_MHA], ids=lambda s: s.name)
def test_tokens_equal_plain_greedy_whatever_the_parameters(shape):
    orc = make_oracle(shape, seed=8)
    rng = np.random.default_rng(2)
    prompt = si.prompt(6, 11, shape.vocab)
    plain = orc.generate_plain(prompt, 16)
    stopped_early = 0
    for _ in range(10):
        kw = dict(alpha=float(rng.uniform(0.3, 1.0)), m=int(rng.integers(0, 4)), n=int(rng.integers(0, 3)),
                  alpha_mlp=float(rng.uniform(0.3, 1.0)), use_cs_mlp=bool(rng.integers(0, 2)),
                  refresh=bool(rng.integers(0, 2)), exit_mode=int(rng.integers(0, 2)),
                  gamma0=float(rng.uniform(0.0, 0.2)), ar0=float(rng.uniform(0, 1)), ar_target=float(rng.uniform(0.3, 0.95)),
                  eps=float(rng.uniform(0, 0.05)), beta1=float(rng.uniform(0, 1)), beta2=float(rng.uniform(0, 1)))
        k = int(rng.integers(1, 6))
        toks, st, mask, C, per = orc.generate_adaptive(prompt, 16, k, **kw)
        assert np.array_equal(toks, plain), kw
        assert st["emitted"] == 16 and st["drafted"] == per[:, 0].sum() and st["accepted"] == per[:, 1].sum()
        assert (per[:, 1] <= per[:, 0]).all() and (per[:, 0] <= k).all()
        stopped_early += int((per[:-1, 0] < k).any())
    assert stopped_early > 0          # the sweep does exercise early exits


def test_running_acs_is_the_acs_of_one_teacher_forced_pass():
    shape = SMALL_GQA
    orc = make_oracle(shape, seed=11)
    prompt = si.prompt(9, 10, shape.vocab)
    N = 15
    toks, st, mask, C, per = orc.generate_adaptive(prompt, N, 3, alpha=0.97, m=0, n=1, refresh=True)
    seq = np.concatenate([prompt, toks[:N - 1]])
    ref = make_oracle(shape, seed=11).forward(seq, 0, want_logits=False)["cos"]
    assert np.abs(C - ref).max() < 1e-12
    # without refresh the reported ACS is the prompt's
    C0 = orc.generate_adaptive(prompt, N, 3, alpha=0.97, m=0, n=1)[3]
    ref0 = make_oracle(shape, seed=11).forward(prompt, 0, want_logits=False)["cos"]
    assert np.abs(C0 - ref0).max() < 1e-12


def test_refresh_rebuilds_the_mask_when_the_running_acs_crosses_the_threshold():
    shape = SMALL_MHA
    orc = make_oracle(shape, seed=13)
    prompt = si.prompt(2, 6, shape.vocab)
    N = 18
    plain = orc.generate_plain(prompt, N)
    C_prompt = make_oracle(shape, seed=13).forward(prompt, 0, want_logits=False)["cos"]
    C_final = make_oracle(shape, seed=13).forward(np.concatenate([prompt, plain[:N - 1]]), 0, want_logits=False)["cos"]
    j = int(np.argmax(np.abs(C_prompt[0::2] - C_final[0::2])))          # the attention sublayer whose ACS moves most
    alpha = float((C_prompt[2 * j] + C_final[2 * j]) / 2)
    toks, st, mask, C, per = orc.generate_adaptive(prompt, N, 2, alpha=alpha, m=0, n=0, refresh=True)
    assert np.array_equal(toks, plain)
    assert np.array_equal(mask, oracle.admg2(C_final, alpha, 0, 0))
    assert not np.array_equal(mask, oracle.admg2(C_prompt, alpha, 0, 0)) and st["mask_changes"] >= 1
