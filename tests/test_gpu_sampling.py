"""GPU checks of sampled decoding (temperature > 0): the sampling kernels against the oracle's rule on identical
logits, and the sampled loop end to end.

Every decision is a threshold on a counter-based uniform that both sides draw identically; the two sides compute
the thresholds in different precision (fp32 weights, blocked sums / double, sequential), so a decision may differ
only where the oracle reports that the uniform fell within a hair of its threshold (relative margin < 1e-6,
about ten times the fp32 rounding of a weight; a bin of a flat 32000-token distribution is 3e-5 wide).
"""
import numpy as np
import pytest

import asd_inputs as si
import oracle
import paper_2410_01028_amd as asd
from test_gpu_parity import build_pair

pytestmark = pytest.mark.gpu

MARGIN = 1e-6
BIG_VOCAB = si.Shape("big-vocab", 1, 64, 2, 2, 32, 64, 32000, si.DT_F32, 4, 4, 2)


def oracle_step(q, p, T, seed, index0):
    kk = p.shape[0] - 1
    mg = 1.0
    drafts = []
    for j in range(kk):
        x, m = oracle.sample_logits(q[j], T, oracle.uniform(seed, index0 + j, 0))
        drafts.append(x); mg = min(mg, m)
    ua = [oracle.uniform(seed, index0 + j, 1) for j in range(kk + 1)]
    ur = [oracle.uniform(seed, index0 + j, 2) for j in range(kk + 1)]
    a, nxt, m = oracle.spec_accept(q if kk else np.zeros((0, p.shape[1])), p, drafts, T, ua, ur)
    return np.array(drafts, np.int32), a, nxt, min(mg, m)


@pytest.mark.parametrize("shape", [si.SHAPES["tiny"], BIG_VOCAB], ids=lambda s: s.name)
def test_sampling_kernels_against_the_rule_on_identical_logits(shape):
    eng = asd.Engine(asd.make_config(shape, 64))
    rng = np.random.default_rng(7)
    V = shape.vocab
    near = total = rejected = kept_all = 0
    for trial in range(60):
        kk = int(rng.integers(0, 7))
        T = float(rng.choice([0.2, 0.6, 1.0, 1.7]))
        p = rng.normal(0, 2.0, (kk + 1, V)).astype(np.float32)
        q = (p[:kk] + rng.normal(0, float(rng.choice([0.0, 0.1, 0.5, 2.0])), (kk, V))).astype(np.float32)
        seed, index0 = int(rng.integers(0, 2 ** 40)), int(rng.integers(0, 1000))
        drafts, a, nxt = eng.spec_sample(q, p, T, seed, index0)
        wd, wa, wn, mg = oracle_step(q.astype(np.float64), p.astype(np.float64), T, seed, index0)
        total += 1
        if mg < MARGIN:
            near += 1
            continue
        assert np.array_equal(drafts, wd) and a == wa and nxt == wn, (trial, kk, T, mg)
        rejected += int(a < kk); kept_all += int(kk > 0 and a == kk)
    assert near <= total // 10 and rejected > 5 and kept_all > 5


def test_degenerate_rows():
    shape = si.SHAPES["tiny"]
    eng = asd.Engine(asd.make_config(shape, 64))
    V = shape.vocab
    # identical distributions: every draft kept, whatever the uniforms
    lg = np.random.default_rng(1).normal(0, 3, (4, V)).astype(np.float32)
    for seed in range(5):
        drafts, a, nxt = eng.spec_sample(lg[:3], lg, 0.7, seed, 0)
        assert a == 3
    # one-hot-like rows: draws are forced
    p = np.full((2, V), -1e4, np.float32); p[0, 5] = 0; p[1, 9] = 0
    q = np.full((1, V), -1e4, np.float32); q[0, 17] = 0
    drafts, a, nxt = eng.spec_sample(q, p, 1.0, 3, 0)
    assert drafts[0] == 17 and a == 0 and nxt == 5
    q[0, 17] = -1e4; q[0, 5] = 0
    drafts, a, nxt = eng.spec_sample(q, p, 1.0, 3, 0)
    assert drafts[0] == 5 and a == 1 and nxt == 9
    with pytest.raises(asd.AsdError):
        eng.spec_sample(q, p, 0.0, 3, 0)


def test_sampled_loop_invariants():
    shape = si.SHAPES["tiny"]
    eng = asd.Engine(asd.make_config(shape, 160)).init_synthetic(4)
    prompt = si.prompt(5, 30, shape.vocab)
    L2 = 2 * shape.n_layers
    N = 40
    skip = np.zeros(L2, np.uint8); skip[2] = 1; skip[5] = 1
    a, sa, _ = eng.generate(prompt, N, 4, fixed_mask=skip, temperature=0.8, seed=11, use_graphs=False)
    b, sb, _ = eng.generate(prompt, N, 4, fixed_mask=skip, temperature=0.8, seed=11, use_graphs=True)
    c, sc, _ = eng.generate(prompt, N, 4, fixed_mask=skip, temperature=0.8, seed=12, use_graphs=True)
    assert np.array_equal(a, b) and sa["accepted"] == sb["accepted"] and not np.array_equal(a, c)
    assert sa["emitted"] == N and 0 < sa["accepted"] <= sa["drafted"]
    assert (a >= 0).all() and (a < shape.vocab).all()
    # the draft model equal to the full model: a draft row's logits equal the verification row's bit for bit, ratio 1
    keep, sk, _ = eng.generate(prompt, N, 4, fixed_mask=np.zeros(L2, np.uint8), temperature=0.8, seed=11)
    assert sk["accepted"] == sk["drafted"] > 0
    # temperature -> 0 is greedy decoding
    plain, _, _ = eng.generate(prompt, N, 0)
    cold, _, _ = eng.generate(prompt, N, 3, fixed_mask=skip, temperature=1e-3, seed=5)
    assert np.array_equal(cold, plain)
    # mask refresh works under sampling as well
    out, st, _ = eng.generate(prompt, N, 3, alpha=0.9, m=0, n=1, refresh=True, temperature=0.6, seed=2)
    assert st["emitted"] == N
    with pytest.raises(asd.AsdError):
        eng.generate(prompt, N, 3, fixed_mask=skip, temperature=0.5, exit_mode=1)


def test_sampled_loop_against_oracle():
    shape = si.SHAPES["tiny"]
    eng, orc = build_pair(shape, seed=3, max_seq=96)
    prompt = si.prompt(6, 16, shape.vocab)
    L2 = 2 * shape.n_layers
    skip = np.zeros(L2, np.uint8); skip[3] = 1; skip[4] = 1
    compared = 0
    for seed in range(8):
        for k, T in ((3, 0.6), (0, 1.0), (5, 0.2)):
            want, wst, mg = orc.generate_sampled(prompt, 24, k, T, seed, skip)
            if mg < 2e-5:           # a draw within the two sides' logit differences (fp32: ~3e-7 of the largest logit, divided by T) of a threshold: either outcome is valid
                continue
            got, gst, _ = eng.generate(prompt, 24, k, fixed_mask=skip, temperature=T, seed=seed)
            assert np.array_equal(got, want), (seed, k, T, mg)
            assert all(gst[x] == wst[x] for x in ("cycles", "drafted", "accepted", "emitted"))
            compared += 1
    assert compared >= 8


def test_register_and_memory_variants_of_the_sampling_kernels_draw_the_same():
    """The sampling kernels hold a thread's share of a logit row in registers when the vocabulary allows it, and read
    it from memory at every use otherwise: the same arithmetic in the same order, so the same draws, bit for bit
    (drafts, accepted counts, replacements, and a whole sampled decode)."""
    shape = si.SHAPES["tiny"].with_(vocab=4096)
    rng = np.random.default_rng(11)
    outs = []
    for mem in (False, True):
        eng = asd.Engine(asd.make_config(shape, 128, debug_flags=asd.DBG_SAMPLE_MEM if mem else 0)).init_synthetic(3)
        got = []
        r = np.random.default_rng(5)
        for case in range(12):
            kk = int(r.integers(0, 5))
            q = r.normal(0, 2.5, (kk, shape.vocab)).astype(np.float32)
            p = (q[:kk] + r.normal(0, 1.0, (kk, shape.vocab))).astype(np.float32) if kk else np.zeros((0, shape.vocab), np.float32)
            p = np.concatenate([p, r.normal(0, 2.5, (1, shape.vocab)).astype(np.float32)])
            drafts, a, nxt = eng.spec_sample(q, p, 0.7, seed=case, index0=3 * case)
            got += [np.asarray(drafts), a, nxt]
        prompt = si.prompt(1, 20, shape.vocab)
        toks, st, _ = eng.generate(prompt, 40, 3, alpha=0.9, m=2, n=1, temperature=0.8, seed=9)
        got += [toks, st["accepted"], st["drafted"]]
        outs.append(got)
        eng.close()
    for x, y in zip(*outs):
        assert np.array_equal(x, y)
