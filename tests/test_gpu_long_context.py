"""GPU parity of decode attention at contexts of more than 16 groups of 256 keys per head (beyond 4096 positions),
the operating range of the long-context workload (Section 1: every decoded token reloads the whole KV cache).

There the final merge of a head's group partials takes its second loop (16 partials are preloaded, the rest come 8
per trip), which shorter contexts never enter.  The engine is compared with the CPU oracle element by element: the
prompt's ACS and last-row logits (prompt pass in blocks), then multi-row and single-row passes whose rows straddle a
group boundary, for head_dim 32 (grouped-query) and head_dim 128, with both register variants of the attention kernel.

Stated tolerances: logits 2e-2 (bf16) of the row's largest |logit|, cosines 1e-3; asserted: the working bounds of
test_gpu_parity.py (2e-4, 2e-5).
"""
import functools

import numpy as np
import pytest

import asd_inputs as si
import oracle
import paper_2410_01028_amd as asd
from test_gpu_parity import BF_GQA, MID16, TOL, COS_TOL, rel_err

pytestmark = pytest.mark.gpu

# (shape, prompt length): the prompt ends two positions before a group boundary (4608 = 18 * 256, 4352 = 17 * 256)
CASES = {"bf-gqa": (BF_GQA, 4606), "mid16": (MID16, 4350)}
FOLLOW = (7, 1, 2, 1)          # rows of the passes after the prompt; the first one straddles the boundary


@functools.lru_cache(maxsize=None)
def oracle_run(name):
    """The oracle's results for the prompt and the passes after it (computed once per shape)."""
    shape, n = CASES[name]
    W = list(si.all_tensors(shape, 7))
    orc = oracle.Oracle(shape, n + 40, kv_storage=True).load(W)
    toks = si.prompt(3, n + 20, shape.vocab)
    o = orc.forward(toks[:n], 0)
    res = [{"cos": o["cos"], "last_logits": o["logits"][-1].copy(), "argmax": int(o["argmax"][-1])}]
    pos = n
    for m in FOLLOW:
        r = orc.forward(toks[pos:pos + m], pos)
        res.append({k: np.array(r[k]) for k in ("logits", "cos_rows", "cos", "argmax")})
        pos += m
    orc.close()
    return W, toks, res


VARIANTS = {"default-attention": 0, "four-waves-per-simd-attention": asd.DBG_ATT_W4}


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("name", list(CASES))
def test_more_than_16_groups_per_head_against_oracle(name, variant):
    shape, n = CASES[name]
    W, toks, want = oracle_run(name)
    tol = TOL[shape.dtype]
    eng = asd.Engine(asd.make_config(shape, n + 40, debug_flags=VARIANTS[variant])).load(W)
    first, acs, lg = eng.prefill(toks[:n], want_logits=True)
    assert eng.kv_len == n and n // 256 + 1 > 16
    assert np.abs(acs - want[0]["cos"]).max() < COS_TOL
    assert rel_err(lg, want[0]["last_logits"]) < tol
    pos = n
    for m, w in zip(FOLLOW, want[1:]):
        g = eng.forward(toks[pos:pos + m], pos)
        err = rel_err(g["logits"], w["logits"])
        assert err.max() < tol, (pos, m, err)
        assert np.abs(g["cos_rows"] - w["cos_rows"]).max() < COS_TOL
        assert np.abs(g["cos"] - w["cos"]).max() < COS_TOL
        top2 = np.sort(w["logits"], -1)[:, -2:]
        clear = (top2[:, 1] - top2[:, 0]) > 2 * tol * np.abs(w["logits"]).max(-1)
        assert np.array_equal(g["argmax"][clear], w["argmax"][clear])
        pos += m
    # rows of a multi-row pass equal single-row passes bit for bit at this depth of context too
    multi = eng.forward(toks[pos:pos + 5], pos, commit=False)
    for i in range(5):
        one = eng.forward(toks[pos + i:pos + i + 1], pos + i)
        assert np.array_equal(one["logits"][0], multi["logits"][i]), i
    eng.close()
