"""Parity at the benchmark's full width and depth (7B shape, bf16) on a short context, plus properties
that hold at the full benchmark sizes (prompt 512, 256 tokens) in the launch configuration bench.py times.

Stated tolerances: logits 2e-2 of the row's largest |logit|, cosines 1e-3.  Measured at the 7B depth against the
oracle with its cache in the storage type: 1e-3 and 3e-5 (32 layers of random weights amplify every rounding), so the
assertions use 5e-3 and 1e-4 as working bounds."""
import numpy as np
import pytest

import asd_inputs as si
import oracle
import paper_2410_01028_amd as asd

pytestmark = pytest.mark.gpu

TOL, COS_TOL = 5e-3, 1e-4


@pytest.fixture(scope="module")
def eng7b():
    s = si.SHAPES["7b"]
    e = asd.Engine(asd.make_config(s, s.prompt_len + s.n_new + 16, page_tokens=256))
    e.init_synthetic(0)
    yield s, e
    e.close()


def test_7b_shape_short_context_against_oracle(eng7b):
    """Teacher-forced logits and cosines of 6 prompt rows + 2 single rows, all 32 layers, oracle in fp64."""
    s, eng = eng7b
    orc = oracle.Oracle(s, 16, kv_storage=True)
    for t, l, a in si.all_tensors(s, 0):
        orc.set_weight(t, l, a)
    toks = si.prompt(0, 8, s.vocab)
    eng.reset()
    for lo, hi in ((0, 6), (6, 7), (7, 8)):
        g = eng.forward(toks[lo:hi], lo)
        o = orc.forward(toks[lo:hi], lo)
        err = np.abs(g["logits"] - o["logits"]).max(-1) / np.abs(o["logits"]).max(-1)
        assert err.max() < TOL, err
        assert np.abs(g["cos_rows"] - o["cos_rows"]).max() < COS_TOL
    mask = si.fixed_keep_mask(s.n_layers, 2)
    g = eng.forward(toks[:3], 8, mask, commit=False)
    o = orc.forward(toks[:3], 8, mask, commit=False)
    err = np.abs(g["logits"] - o["logits"]).max(-1) / np.abs(o["logits"]).max(-1)
    assert err.max() < TOL, err
    assert np.abs(g["cos_rows"] - o["cos_rows"]).max() < COS_TOL
    orc.close()


def test_7b_shape_prompt_blocks_against_oracle(eng7b):
    """The prompt pass in blocks (large-M kernels) at full width and depth: 40 prompt rows against the oracle, then the
    full 512-row prompt against the decode-kernel path (both on the GPU)."""
    s, eng = eng7b
    orc = oracle.Oracle(s, 48, kv_storage=True)
    for t, l, a in si.all_tensors(s, 0):
        orc.set_weight(t, l, a)
    toks = si.prompt(0, 44, s.vocab)
    first, acs, lg = eng.prefill(toks[:40], want_logits=True)
    o = orc.forward(toks[:40], 0)
    assert np.abs(acs - o["cos"]).max() < COS_TOL
    assert np.abs(lg - o["logits"][-1]).max() / np.abs(o["logits"][-1]).max() < TOL
    g = eng.forward(toks[40:44], 40)                      # reads the cache the block pass wrote
    o2 = orc.forward(toks[40:44], 40)
    err = np.abs(g["logits"] - o2["logits"]).max(-1) / np.abs(o2["logits"]).max(-1)
    assert err.max() < TOL, err
    orc.close()
    prompt = si.prompt(0, s.prompt_len, s.vocab)
    f1, a1, l1 = eng.prefill(prompt, want_logits=True)
    n1 = eng.forward(prompt[:3], s.prompt_len, commit=False)["logits"]
    f2, a2, l2 = eng.prefill(prompt, want_logits=True, chunked=True)
    n2 = eng.forward(prompt[:3], s.prompt_len, commit=False)["logits"]
    assert f1 == f2 and np.abs(a1 - a2).max() < COS_TOL
    assert np.abs(l1 - l2).max() / np.abs(l2).max() < TOL
    assert (np.abs(n1 - n2).max(-1) / np.abs(n2).max(-1)).max() < TOL


def test_7b_full_benchmark_sizes_properties(eng7b):
    s, eng = eng7b
    prompt = si.prompt(0, s.prompt_len, s.vocab)
    N = 64
    plain, st, _ = eng.generate(prompt, N, 0)
    L2 = 2 * s.n_layers
    for k, kw in ((4, dict(alpha=0.985, m=3, n=2)), (6, dict(fixed_mask=si.fixed_keep_mask(s.n_layers, 2))),
                  (8, dict(fixed_mask=np.zeros(L2, np.uint8)))):
        out, st, mask = eng.generate(prompt, N, k, **kw)
        assert np.array_equal(out, plain)
        assert st["emitted"] == N == st["accepted"] + st["cycles"] + 1
        assert eng.kv_len == s.prompt_len + N - 1
    assert st["cycles"] == -(-(N - 1) // 9) and st["accepted"] == st["drafted"]      # all-keep: every draft accepted
    first, acs, _ = eng.prefill(prompt)
    assert (acs <= 1.0).all() and (acs >= -1.0).all() and first == plain[0]
    # determinism: the same pass twice gives the same bits
    a = eng.forward(prompt[:5], s.prompt_len, commit=False)
    b = eng.forward(prompt[:5], s.prompt_len, commit=False)
    assert np.array_equal(a["logits"], b["logits"]) and np.array_equal(a["cos_rows"], b["cos_rows"])
    # rows of a verify pass equal single-row passes at the full shape
    for i in range(5):
        one = eng.forward(prompt[i:i + 1], s.prompt_len + i)
        assert np.array_equal(one["logits"][0], a["logits"][i])


def test_7b_long_context_benchmark_sizes_properties():
    """The long-context workload at its full sizes (prompt 8192, 32 layers, cache sized as bench.py sizes it): output
    equal to plain greedy decoding under the fixed masks the workload names and under the all-keep mask, the cache
    bookkeeping, rows of a 7-row verification pass equal to single-row passes bit for bit at a context of 32 groups
    per head, and the block prompt path against the chunked one."""
    s = si.SHAPES["7b-long"]
    eng = asd.Engine(asd.make_config(s, s.prompt_len + s.n_new + 16, page_tokens=256)).init_synthetic(0)
    prompt = si.prompt(0, s.prompt_len, s.vocab)
    N, k, L2 = 24, s.draft_len, 2 * s.n_layers
    plain, st, _ = eng.generate(prompt, N, 0)
    for kw in (dict(fixed_mask=si.fixed_keep_mask(s.n_layers, 2)), dict(fixed_mask=si.fixed_keep_mask(s.n_layers, 4)),
               dict(fixed_mask=np.zeros(L2, np.uint8))):
        out, st, mask = eng.generate(prompt, N, k, **kw)
        assert np.array_equal(out, plain)
        assert st["emitted"] == N == st["accepted"] + st["cycles"] + 1
        assert eng.kv_len == s.prompt_len + N - 1
    assert st["cycles"] == -(-(N - 1) // (k + 1)) and st["accepted"] == st["drafted"]     # all-keep: every draft accepted
    first, acs, lg = eng.prefill(prompt, want_logits=True)
    assert (acs <= 1.0).all() and (acs >= -1.0).all() and first == plain[0] and eng.kv_len == s.prompt_len
    rows = np.concatenate([plain[:1], prompt[:k]]).astype(np.int32)
    a = eng.forward(rows, s.prompt_len, commit=False)
    b = eng.forward(rows, s.prompt_len, commit=False)
    assert np.array_equal(a["logits"], b["logits"]) and np.array_equal(a["cos_rows"], b["cos_rows"])
    for i in range(k + 1):
        one = eng.forward(rows[i:i + 1], s.prompt_len + i)
        assert np.array_equal(one["logits"][0], a["logits"][i])
    assert int(np.argmax(a["logits"][0])) == plain[1]
    # the two prompt paths differ in summation order only
    first_c, acs_c, lg_c = eng.prefill(prompt[:2048], want_logits=True, chunked=True)
    first_b, acs_b, lg_b = eng.prefill(prompt[:2048], want_logits=True)
    assert np.abs(lg_c - lg_b).max() / np.abs(lg_b).max() < TOL and np.abs(acs_c - acs_b).max() < COS_TOL
    eng.close()


@pytest.mark.parametrize("name", ["13b", "70b"])
def test_other_shapes_run_and_keep_invariants(name):
    """13B and 70B-GQA shapes at full width, reduced depth (4 layers) to keep the test short."""
    s = si.SHAPES[name].with_(n_layers=4)
    eng = asd.Engine(asd.make_config(s, 512, page_tokens=256)).init_synthetic(0)
    orc = oracle.Oracle(s, 16, kv_storage=True)
    for t, l, a in si.all_tensors(s, 0):
        orc.set_weight(t, l, a)
    toks = si.prompt(0, 200, s.vocab)
    g = eng.forward(toks[:5], 0)
    o = orc.forward(toks[:5], 0)
    err = np.abs(g["logits"] - o["logits"]).max(-1) / np.abs(o["logits"]).max(-1)
    assert err.max() < TOL, err
    assert np.abs(g["cos_rows"] - o["cos_rows"]).max() < COS_TOL
    orc.close()
    plain, _, _ = eng.generate(toks, 24, 0)
    out, st, _ = eng.generate(toks, 24, 6, fixed_mask=np.array([0, 0, 1, 0, 0, 1, 0, 0], np.uint8))
    assert np.array_equal(out, plain) and st["emitted"] == 24
    eng.close()


def _oracle_for(shape, max_seq):
    orc = oracle.Oracle(shape, max_seq, kv_storage=True)
    for t, l, a in si.all_tensors(shape, 0):
        orc.set_weight(t, l, a)
    return orc


def test_13b_shape_full_depth_against_oracle():
    """The 13B shape at its full 40 layers and width (the family the paper runs, Section 4): teacher-forced logits and
    per-row cosines of a 4-row pass, a single row on top of it and a masked 2-row pass against the oracle (about 26 GB of
    host weights).  Working bounds as at the 7B depth; stated: 2e-2 / 1e-3."""
    s = si.SHAPES["13b"]
    eng = asd.Engine(asd.make_config(s, 64, page_tokens=64)).init_synthetic(0)
    orc = _oracle_for(s, 16)
    toks = si.prompt(0, 8, s.vocab)
    worst = 0.0
    for lo, hi, mask in ((0, 4, None), (4, 5, None), (5, 7, si.fixed_keep_mask(s.n_layers, 2))):
        g = eng.forward(toks[lo:hi], lo, mask)
        o = orc.forward(toks[lo:hi], lo, mask)
        err = np.abs(g["logits"] - o["logits"]).max(-1) / np.abs(o["logits"]).max(-1)
        worst = max(worst, float(err.max()))
        assert err.max() < TOL, err
        assert np.abs(g["cos_rows"] - o["cos_rows"]).max() < COS_TOL
    print(f"13b, 40 layers: worst logit error {worst:.2e} of the row maximum")
    orc.close()
    eng.close()


def test_70b_shape_full_depth_against_oracle():
    """The 70B grouped-query shape at full width and as many layers as the host's memory holds for the oracle's copy of
    the weights (1.72 GB per layer in bf16; all 80 layers need about 140 GB): a 3-row pass and a single row against the
    oracle.  The layer count used is printed; fewer than 80 only on a host with less free memory."""
    import psutil
    s = si.SHAPES["70b"]
    per_layer = 2 * (s.d_model * (s.q_dim + 2 * s.kv_dim) + s.q_dim * s.d_model + 3 * s.d_model * s.d_ffn)
    fixed = 2 * 2 * s.vocab * s.d_model
    avail = psutil.virtual_memory().available
    layers = int(min(s.n_layers, (min(avail, 250 << 30) * 0.7 - fixed) // per_layer))
    assert layers >= 8, f"only {avail >> 30} GiB of host memory available"
    s = s.with_(n_layers=layers)
    eng = asd.Engine(asd.make_config(s, 64, page_tokens=64)).init_synthetic(0)
    orc = _oracle_for(s, 16)
    toks = si.prompt(0, 8, s.vocab)
    worst = 0.0
    for lo, hi in ((0, 3), (3, 4)):
        g = eng.forward(toks[lo:hi], lo)
        o = orc.forward(toks[lo:hi], lo)
        err = np.abs(g["logits"] - o["logits"]).max(-1) / np.abs(o["logits"]).max(-1)
        worst = max(worst, float(err.max()))
        assert err.max() < 2 * TOL, err
        assert np.abs(g["cos_rows"] - o["cos_rows"]).max() < COS_TOL
    print(f"70b-gqa, {layers} layers: worst logit error {worst:.2e} of the row maximum")
    orc.close()
    eng.close()


def test_7b_width_two_attention_groups_against_oracle():
    """The 7B width (32 heads x 128, d_model 4096, FFN 11008, full vocabulary) at a context past 512 positions, where a
    head's keys span three 256-key groups merged across workgroups, on a 4-layer model the oracle finishes in
    seconds: the prompt pass in blocks, then a 5-row pass straddling nothing and a single row, against the oracle."""
    s = si.SHAPES["7b"].with_(n_layers=4)
    n = 520
    eng = asd.Engine(asd.make_config(s, 640, page_tokens=256)).init_synthetic(0)
    orc = _oracle_for(s, 640)
    toks = si.prompt(0, n + 8, s.vocab)
    first, acs, lg = eng.prefill(toks[:n], want_logits=True)
    o = orc.forward(toks[:n], 0)
    assert np.abs(acs - o["cos"]).max() < COS_TOL
    assert np.abs(lg - o["logits"][-1]).max() / np.abs(o["logits"][-1]).max() < TOL
    for lo, hi in ((n, n + 5), (n + 5, n + 6)):
        g = eng.forward(toks[lo:hi], lo)
        r = orc.forward(toks[lo:hi], lo)
        err = np.abs(g["logits"] - r["logits"]).max(-1) / np.abs(r["logits"]).max(-1)
        assert err.max() < TOL, err
        assert np.abs(g["cos_rows"] - r["cos_rows"]).max() < COS_TOL
    orc.close()
    eng.close()
