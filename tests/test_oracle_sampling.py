"""Pins of the oracle's sampled decoding (speculative sampling at temperature > 0).

The paper cites the rule without printing it; what pins it is the property that defines it: whatever the draft
distribution, the emitted tokens are distributed exactly as samples of the full model.  The small functions are
pinned by closed forms and by exhaustive enumeration of the uniforms on midpoint grids (every decision is a
threshold on a uniform, so a grid of n points reproduces each probability to within 1/n per threshold).
"""
import numpy as np
import pytest
from scipy.special import softmax

import asd_inputs as si
import oracle
from helpers import SMALL_GQA, SMALL_MHA, make_oracle


def grid(n):
    return (np.arange(n) + 0.5) / n


def test_uniform_stream_matches_the_shared_generator():
    seen = set()
    for seed in (0, 1, 12345678901234):
        for index in (0, 1, 2, 77, 100000):
            for purpose in (0, 1, 2):
                u = oracle.uniform(seed, index, purpose)
                assert 0.0 <= u < 1.0
                assert u == si.sampling_uniform(seed, index, purpose)
                seen.add(u)
    assert len(seen) == 45
    us = np.array([oracle.uniform(5, i, 2) for i in range(20000)])
    assert abs(us.mean() - 0.5) < 0.01 and abs(us.var() - 1 / 12) < 0.005


def test_inverse_cdf_closed_forms_and_frequencies():
    w = [0.25, 0.25, 0.5]
    assert [oracle.sample_weights(w, u)[0] for u in (0.0, 0.1, 0.2499, 0.25, 0.3, 0.4999, 0.5, 0.99)] == [0, 0, 0, 1, 1, 1, 2, 2]
    assert oracle.sample_weights([0.0, 3.0, 0.0], 0.7)[0] == 1                 # zero-weight bins are never chosen
    assert oracle.sample_weights([2.0, 0.0, 0.0], 0.999999)[0] == 0
    assert oracle.sample_weights(w, 0.3)[1] == pytest.approx(0.05, rel=1e-12)   # margin: distance to the nearer bin edge
    rng = np.random.default_rng(0)
    n = 4000
    for _ in range(5):
        wts = rng.uniform(0, 1, 6) * (rng.uniform(0, 1, 6) > 0.3)
        wts[0] += 0.1
        cnt = np.bincount([oracle.sample_weights(wts, u)[0] for u in grid(n)], minlength=6)
        assert np.abs(cnt / n - wts / wts.sum()).max() <= 1.0 / n + 1e-12


def test_temperature_softmax_sampling():
    rng = np.random.default_rng(1)
    lg = rng.normal(0, 2, 9)
    n = 3000
    for T in (0.2, 0.6, 1.0, 3.0):
        cnt = np.bincount([oracle.sample_logits(lg, T, u)[0] for u in grid(n)], minlength=9)
        assert np.abs(cnt / n - softmax(lg / T)).max() <= 1.0 / n + 1e-12
    assert all(oracle.sample_logits(lg, 1e-3, u)[0] == int(np.argmax(lg)) for u in grid(50))       # T -> 0: greedy
    assert oracle.sample_logits([1000.0, 0.0, -1000.0], 0.5, 0.999)[0] == 0                          # no overflow


@pytest.mark.parametrize("case", range(4))
def test_one_draft_verification_emits_the_target_distribution(case):
    """kk = 1, V = 4: enumerate (draft uniform, accept uniform, replacement uniform) on midpoint grids."""
    rng = np.random.default_rng(10 + case)
    V, T, n = 4, [1.0, 0.6, 0.2, 2.0][case], 32
    ql = rng.normal(0, 1.5, (1, V))
    pl = rng.normal(0, 1.5, (2, V))
    if case == 3:
        ql[0] = pl[0] + np.array([3.0, -3.0, 0.0, 0.0])                # a draft model that is badly off
    first = np.zeros(V)
    second_given_accept = np.zeros(V)
    n_acc = 0
    for ud in grid(n):
        x, _ = oracle.sample_logits(ql[0], T, ud)
        for ua in grid(n):
            for ur in grid(n):
                a, nxt, _ = oracle.spec_accept(ql, pl, [x], T, [ua], [ur, ur])
                if a == 1:
                    first[x] += 1; second_given_accept[nxt] += 1; n_acc += 1
                else:
                    first[nxt] += 1
    want = softmax(pl[0] / T)
    assert np.abs(first / n ** 3 - want).max() < 3.0 / n                 # three thresholds, each resolved to 1/n
    if n_acc >= n * n:               # (peaked distributions with different modes may accept next to nothing)
        assert np.abs(second_given_accept / n_acc - softmax(pl[1] / T)).max() < 3.0 / n + n * n / n_acc / n
    # acceptance rate = sum_x min(p, q)
    assert abs(n_acc / n ** 3 - np.minimum(want, softmax(ql[0] / T)).sum()) < 3.0 / n


def test_two_draft_verification_first_token_marginal_and_acceptance_count():
    rng = np.random.default_rng(3)
    V, T, n = 3, 0.8, 12
    ql = rng.normal(0, 1, (2, V))
    pl = rng.normal(0, 1, (3, V))
    first = np.zeros(V)
    acc_hist = np.zeros(3)
    tot = 0
    for ud0 in grid(n):
        x0, _ = oracle.sample_logits(ql[0], T, ud0)
        for ud1 in grid(n):
            x1, _ = oracle.sample_logits(ql[1], T, ud1)
            for ua0 in grid(n):
                for ua1 in grid(n):
                    for ur in grid(n):
                        a, nxt, _ = oracle.spec_accept(ql, pl, [x0, x1], T, [ua0, ua1], [ur, ur, ur])
                        first[x0 if a >= 1 else nxt] += 1
                        acc_hist[a] += 1
                        tot += 1
    p0, q0 = softmax(pl[0] / T), softmax(ql[0] / T)
    p1, q1 = softmax(pl[1] / T), softmax(ql[1] / T)
    assert np.abs(first / tot - p0).max() < 4.0 / n
    b0, b1 = np.minimum(p0, q0).sum(), np.minimum(p1, q1).sum()
    assert abs(acc_hist[0] / tot - (1 - b0)) < 4.0 / n
    assert abs(acc_hist[2] / tot - b0 * b1) < 4.0 / n


def test_identical_distributions_always_accept_and_disjoint_support_always_rejects():
    rng = np.random.default_rng(4)
    lg = rng.normal(0, 2, (3, 7))
    for u in grid(9):
        x = [oracle.sample_logits(lg[0], 0.7, u)[0], oracle.sample_logits(lg[1], 0.7, 1 - u)[0]]
        a, nxt, _ = oracle.spec_accept(lg[:2], lg, x, 0.7, [0.999999, u], [u, u, u])
        assert a == 2 and nxt == oracle.sample_logits(lg[2], 0.7, u)[0]
    q = np.array([[0.0, -2000.0, -2000.0]])
    p = np.array([[-2000.0, 0.0, 1.0], [0.0, 0.0, 0.0]])
    for u in grid(9):
        a, nxt, _ = oracle.spec_accept(q, p, [0], 1.0, [u], [u, u])
        assert a == 0 and nxt == oracle.sample_weights([0.0, 1.0, np.e], u)[0]


@pytest.mark.parametrize("shape", [SMALL_GQA, SMALL_MHA], ids=lambda s: s.name)
def test_sampled_loop_bookkeeping(shape):
    orc = make_oracle(shape, seed=2)
    prompt = si.prompt(3, 8, shape.vocab)
    L2 = 2 * shape.n_layers
    skip = np.zeros(L2, np.uint8); skip[2] = 1
    a = orc.generate_sampled(prompt, 14, 3, 0.8, 42, skip)
    b = orc.generate_sampled(prompt, 14, 3, 0.8, 42, skip)
    c = orc.generate_sampled(prompt, 14, 3, 0.8, 43, skip)
    assert np.array_equal(a[0], b[0]) and a[1] == b[1] and not np.array_equal(a[0], c[0])
    assert a[1]["emitted"] == 14 and a[1]["accepted"] <= a[1]["drafted"]
    # the draft model equal to the full model: every draft is kept (same logits, ratio exactly 1)
    keep = orc.generate_sampled(prompt, 14, 3, 0.8, 42, np.zeros(L2, np.uint8))
    assert keep[1]["accepted"] == keep[1]["drafted"] > 0
    # temperature -> 0 is greedy decoding
    cold = orc.generate_sampled(prompt, 10, 2, 1e-4, 7, skip)
    assert np.array_equal(cold[0], orc.generate_plain(prompt, 10))
    # draft length 0 is plain sampling: token e drawn with U(e, 2) from the full model's logits
    plain = orc.generate_sampled(prompt, 6, 0, 0.8, 9, None)[0]
    ref = make_oracle(shape, seed=2)
    seq = list(prompt)
    lg = ref.forward(prompt, 0)["logits"][-1]
    for e in range(6):
        tok = oracle.sample_logits(lg, 0.8, oracle.uniform(9, e, 2))[0]
        assert tok == plain[e]
        lg = ref.forward([tok], len(seq))["logits"][0]
        seq.append(tok)


def test_sampled_loop_emits_the_full_models_distribution():
    """First two tokens over many seeds against the exact two-step distribution of the full model."""
    shape = SMALL_MHA
    orc = make_oracle(shape, seed=6)
    prompt = si.prompt(1, 5, shape.vocab)
    T, n = 1.0, 1500
    skip = np.zeros(2 * shape.n_layers, np.uint8); skip[1] = 1; skip[2] = 1       # a draft model that differs
    lg0 = orc.forward(prompt, 0)["logits"][-1]
    p0 = softmax(lg0 / T)
    top = np.argsort(p0)[::-1][:3]
    p1 = {}
    for t in top:
        orc.truncate(len(prompt))
        p1[t] = softmax(orc.forward([t], len(prompt), commit=False)["logits"][0] / T)
    c0 = np.zeros(shape.vocab)
    c1 = {t: np.zeros(shape.vocab) for t in top}
    acc = 0
    for seed in range(n):
        toks, st, _ = orc.generate_sampled(prompt, 3, 2, T, 1000 + seed, skip)
        c0[toks[0]] += 1
        acc += st["accepted"]
        if toks[0] in c1:
            c1[toks[0]][toks[1]] += 1
    assert 0 < acc < 2 * n                                   # drafts are sometimes kept, sometimes replaced
    # binomial 4-sigma bounds per compared cell
    for t in top:
        assert abs(c0[t] / n - p0[t]) < 4 * np.sqrt(p0[t] * (1 - p0[t]) / n)
        m = c1[t].sum()
        best = np.argsort(p1[t])[::-1][:3]
        for y in best:
            assert abs(c1[t][y] / m - p1[t][y]) < 4 * np.sqrt(p1[t][y] * (1 - p1[t][y]) / m) + 1e-9
