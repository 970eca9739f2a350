"""Pins of the oracle's ADMG (Algorithm 1) and of its speculative greedy loop (Section 1)."""
import itertools
import os

import numpy as np
import pytest

import asd_inputs as si
import oracle
from helpers import SMALL_GQA, SMALL_MHA, make_oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "admg_table2_closed_forms.txt")


def sets_of(mask):
    """1-based (remove_ATTN, remove_MLP) from a skip mask."""
    L = len(mask) // 2
    return ({l for l in range(1, L + 1) if mask[2 * (l - 1)]},
            {l for l in range(1, L + 1) if mask[2 * (l - 1) + 1]})


def test_closed_forms_for_table2_hyperparameters():
    rows = [ln.split("|") for ln in open(GOLD) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 8
    for lhs, rhs in rows:
        L, m, n = map(int, lhs.split())
        first, last, count = rhs.split()
        expect = set() if count == "0" else set(range(int(first), int(last) + 1, m))
        assert len(expect) == int(count)
        ra, rm = sets_of(oracle.admg(np.zeros(L), 0.985, m, n))      # no C_l reaches alpha
        assert rm == expect and ra == expect


def test_brute_force_all_threshold_patterns():
    """Every above/below-alpha pattern for L <= 7 and all m, n against set algebra on ranges."""
    alpha = 0.985
    for L in range(1, 8):
        for pattern in itertools.product([0.5, 0.985, 0.99], repeat=L):
            C = np.array(pattern)
            hot = {l for l in range(1, L + 1) if C[l - 1] >= alpha}
            for m in range(0, L + 2):
                for n in range(0, L + 2):
                    allowed = set(range(1, L - n + 1))
                    multiples = set(range(m, L + 1, m)) if m else set()
                    ra, rm = sets_of(oracle.admg(C, alpha, m, n))
                    assert rm == multiples & allowed
                    assert ra == (hot & allowed) | rm


def test_invariants_and_ablation_modes():
    rng = np.random.default_rng(1)
    for _ in range(200):
        L = int(rng.integers(2, 41))
        C = rng.uniform(0.9, 1.0, L)
        m, n = int(rng.integers(0, 6)), int(rng.integers(0, 5))
        a1, a2 = sorted(rng.uniform(0.9, 1.0, 2))
        ra, rm = sets_of(oracle.admg(C, a1, m, n))
        assert rm <= ra                                   # a removed MLP's attention is removed too
        assert not ra or max(ra) <= L - n                 # rule 2
        ra_hi, _ = sets_of(oracle.admg(C, a2, m, n))
        assert ra_hi <= ra                                # raising alpha never removes more
        # rule subsets of the ablation: CS only, CS + rule 2, rules 1 & 2, all three
        cs_only = sets_of(oracle.admg(C, a1, 0, 0))
        cs_r2 = sets_of(oracle.admg(C, a1, 0, n))
        r12 = sets_of(oracle.admg(C, a1, m, n, use_cs=False))
        assert cs_only[1] == set() and cs_r2[1] == set()
        assert cs_r2[0] == {l for l in cs_only[0] if l <= L - n}
        assert r12[0] == r12[1] == rm
        assert ra == cs_r2[0] | r12[0]
    # the threshold is inclusive
    assert sets_of(oracle.admg(np.array([0.985, 0.9849999]), 0.985, 0, 0))[0] == {1}
    with pytest.raises(ValueError):
        oracle.admg(np.zeros(4), 0.985, -1, 0)


@pytest.fixture(scope="module")
def tiny():
    s = si.SHAPES["tiny"]
    return s, make_oracle(s, seed=0, max_seq=96), si.prompt(0, s.prompt_len, s.vocab)


def test_speculative_output_equals_plain_greedy_for_every_mask_and_k(tiny):
    s, o, prompt = tiny
    N = 24
    plain = o.generate_plain(prompt, N)
    rng = np.random.default_rng(0)
    masks = [np.zeros(8, np.uint8), np.ones(8, np.uint8)] + [rng.integers(0, 2, 8).astype(np.uint8) for _ in range(4)]
    for mask in masks:
        for k in (0, 1, 3, 4, 8):
            out, st, used, _ = o.generate_spec(prompt, N, k, fixed_mask=mask)
            assert np.array_equal(out, plain)
            assert np.array_equal(used, mask)
            assert st["emitted"] == N == st["accepted"] + st["cycles"] + 1
            assert o.kv_len == len(prompt) + N - 1
            assert st["accepted"] <= st["drafted"] <= k * st["cycles"]
    # paper's hyper-parameters route (ADMG from the prompt's ACS)
    out, st, used, C = o.generate_spec(prompt, N, 4, alpha=0.985, m=2, n=1)
    assert np.array_equal(out, plain)
    assert np.array_equal(used, oracle.admg(C[0::2], 0.985, 2, 1))
    o.reset()
    assert np.abs(C - o.forward(prompt, 0)["cos"]).max() < 1e-15


def test_all_keep_draft_accepts_everything(tiny):
    """D = M: every draft is accepted, so a cycle emits k+1 tokens until the tail."""
    s, o, prompt = tiny
    for N, k in ((24, 4), (17, 3), (9, 8), (2, 4)):
        out, st, _, _ = o.generate_spec(prompt, N, k, fixed_mask=np.zeros(8, np.uint8))
        assert st["cycles"] == -(-(N - 1) // (k + 1))
        assert st["accepted"] == st["drafted"] == N - 1 - st["cycles"]


def test_all_skip_draft_is_lm_head_of_embedding():
    s = SMALL_MHA
    o = make_oracle(s, seed=8, gain_std=0.1)
    w = {(t, l): si.as_f64(a) for t, l, a in si.all_tensors(s, 8, 0.1)}
    tok = np.array([5, 17], np.int32)
    r = o.forward(tok, 0, skip=np.ones(2 * s.n_layers, np.uint8))
    E = w[(si.T_EMBED, 0)][tok]
    xn = E / np.sqrt((E * E).mean(-1, keepdims=True) + s.rms_eps) * w[(si.T_FINAL_NORM, 0)]
    assert np.abs(r["logits"] - xn @ w[(si.T_LM_HEAD, 0)].T).max() < 1e-13
    assert (r["cos_rows"] == 1.0).all()


def test_gqa_model_speculative_equals_plain():
    s = SMALL_GQA
    o = make_oracle(s, seed=12)
    prompt = si.prompt(12, s.prompt_len, s.vocab)
    plain = o.generate_plain(prompt, 14)
    out, st, used, _ = o.generate_spec(prompt, 14, 3, alpha=0.99, m=2, n=1)
    assert np.array_equal(out, plain) and used[3] == 1 and used[5] == 0
