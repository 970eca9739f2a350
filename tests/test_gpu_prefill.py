"""GPU parity of the prompt pass taken in blocks (large-M contractions) against the CPU oracle.

What is checked after a prompt of n tokens: the ACS of every sublayer (Section 3.2, the definition of C_l; 1e-3 absolute), the last row's
logits (2e-2 bf16 / 1e-4 fp32, inf-norm relative), the first greedy token where the oracle's top-2 gap is clear,
and the KV cache the pass wrote, through a teacher-forced multi-row pass right behind it.  Prompt lengths
cover a ragged last 16-row chunk, a ragged last workgroup row block, contexts that span several 256-key
attention groups, and a prompt longer than one 512-row block.
"""
import numpy as np
import pytest

import asd_inputs as si
import paper_2410_01028_amd as asd
from helpers import SMALL_GQA
from test_gpu_parity import BF_GQA, MID16, MID32, TOL, COS_TOL, build_pair, check_forward, rel_err

pytestmark = pytest.mark.gpu

CASES = [(si.SHAPES["tiny"], 37), (si.SHAPES["tiny"], 100), (SMALL_GQA, 77), (BF_GQA, 77), (BF_GQA, 130),
         (MID32, 150), (MID16, 300), (MID16, 600)]


@pytest.mark.parametrize("shape,n", CASES, ids=[f"{s.name}-{n}" for s, n in CASES])
def test_blocked_prompt_pass_against_oracle(shape, n):
    eng, orc = build_pair(shape, seed=4, max_seq=n + 40)
    toks = si.prompt(5, n + 6, shape.vocab)
    first, acs, lg = eng.prefill(toks[:n], want_logits=True)
    assert eng.kv_len == n
    o = orc.forward(toks[:n], 0)
    assert np.abs(acs - o["cos"]).max() < COS_TOL
    assert rel_err(lg, o["logits"][-1]) < TOL[shape.dtype]
    top2 = np.sort(o["logits"][-1])[-2:]
    if top2[1] - top2[0] > 2 * TOL[shape.dtype] * np.abs(o["logits"][-1]).max():
        assert first == o["argmax"][-1]
    check_forward(eng, orc, toks[n:n + 6], n, None, TOL[shape.dtype])


@pytest.mark.parametrize("shape", [si.SHAPES["tiny"], MID16], ids=lambda s: s.name)
def test_blocked_and_chunked_prompt_pass_agree(shape):
    n = 210
    eng = eng2 = None
    W = list(si.all_tensors(shape, 9))
    import paper_2410_01028_amd as asd
    eng = asd.Engine(asd.make_config(shape, 256)).load(W)
    eng2 = asd.Engine(asd.make_config(shape, 256)).load(W)
    toks = si.prompt(1, n + 4, shape.vocab)
    f1, acs1, lg1 = eng.prefill(toks[:n], want_logits=True)
    f2, acs2, lg2 = eng2.prefill(toks[:n], want_logits=True, chunked=True)
    tol = TOL[shape.dtype]
    assert np.abs(acs1 - acs2).max() < COS_TOL
    assert rel_err(lg1, lg2) < tol
    a = eng.forward(toks[n:n + 4], n)["logits"]
    b = eng2.forward(toks[n:n + 4], n)["logits"]
    assert rel_err(a, b).max() < tol


def test_short_prompts_take_the_decode_kernels():
    shape = si.SHAPES["tiny"]
    eng, orc = build_pair(shape, seed=2, max_seq=64)
    toks = si.prompt(8, 16, shape.vocab)
    first, acs, lg = eng.prefill(toks, want_logits=True)
    first2, acs2, lg2 = eng.prefill(toks, want_logits=True, chunked=True)
    assert first == first2 and np.array_equal(acs, acs2) and np.array_equal(lg, lg2)


@pytest.mark.parametrize("n", [16, 17, 512, 513, 1039], ids=lambda n: f"n{n}")
def test_block_boundaries_agree_with_the_chunked_pass(n):
    """Prompt lengths at the 16-row and 512-row boundaries (one row spilling into a new chunk / a new block)."""
    import paper_2410_01028_amd as asd
    shape = BF_GQA
    W = list(si.all_tensors(shape, 12))
    eng = asd.Engine(asd.make_config(shape, 1088)).load(W)
    ref = asd.Engine(asd.make_config(shape, 1088)).load(W)
    toks = si.prompt(n, n + 3, shape.vocab)
    f1, acs1, lg1 = eng.prefill(toks[:n], want_logits=True)
    f2, acs2, lg2 = ref.prefill(toks[:n], want_logits=True, chunked=True)
    assert eng.kv_len == n and np.abs(acs1 - acs2).max() < COS_TOL
    assert rel_err(lg1, lg2) < TOL[shape.dtype]
    a = eng.forward(toks[n:n + 3], n)["logits"]
    b = ref.forward(toks[n:n + 3], n)["logits"]
    assert rel_err(a, b).max() < TOL[shape.dtype]


@pytest.mark.parametrize("force_w4", [False, True], ids=["default-attention", "four-waves-per-simd-attention"])
def test_long_context_against_oracle(force_w4):
    """A context of ten 256-key groups per head on a small grouped-query model: the blocked prompt pass (five 512-row
    blocks), then multi-row and single-row passes on top of it, against the oracle; once with the decode attention
    variant that long contexts on large models select."""
    shape = BF_GQA
    n = 2500
    eng, orc = build_pair(shape, seed=7, max_seq=n + 40, debug_flags=asd.DBG_ATT_W4 if force_w4 else 0)
    toks = si.prompt(3, n + 20, shape.vocab)
    first, acs, lg = eng.prefill(toks[:n], want_logits=True)
    o = orc.forward(toks[:n], 0)
    assert np.abs(acs - o["cos"]).max() < COS_TOL
    assert rel_err(lg, o["logits"][-1]) < TOL[shape.dtype]
    pos = n
    for m in (7, 1, 2, 1):
        check_forward(eng, orc, toks[pos:pos + m], pos, None, TOL[shape.dtype])
        pos += m
