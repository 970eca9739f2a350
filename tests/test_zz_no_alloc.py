"""The forward entry point that allocates nothing (static device scratch) against asd_forward, through the C ABI:
same kernels, so logits, cosines and greedy tokens must agree bit for bit; two calls in a row, the second with fewer
rows; contexts of one and of several attention groups; a skip mask; an out-of-vocabulary token id on the device."""
import numpy as np
import pytest
import torch

import asd_inputs as si
import paper_2410_01028_amd as asd
from test_gpu_parity import MID16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape,ctx", [(si.SHAPES["tiny"], 40), (MID16, 150), (MID16, 600)], ids=["tiny-40", "mid16-150", "mid16-600"])
def test_forward_noalloc_matches_forward_bitwise(shape, ctx):
    eng = asd.Engine(asd.make_config(shape, 768)).init_synthetic(3)
    toks = si.prompt(2, ctx + 20, shape.vocab)
    eng.prefill(toks[:ctx])
    L2, V = 2 * shape.n_layers, shape.vocab
    mask = np.zeros(L2, np.uint8); mask[2] = mask[5] = 1
    dev = eng.device
    with torch.cuda.stream(eng.stream):
        for rows, skip in ((7, None), (3, mask), (1, None)):           # consecutive calls, each smaller than the one before
            want = eng.forward(toks[ctx:ctx + rows], ctx, skip, commit=False)
            d_tok = torch.from_numpy(toks[ctx:ctx + rows].copy()).to(dev)
            d_logits = torch.full((rows, V), float("nan"), dtype=torch.float32, device=dev)
            d_cos = torch.full((L2,), float("nan"), dtype=torch.float32, device=dev)
            d_am = torch.full((rows,), -1, dtype=torch.int32, device=dev)
            eng.stream.synchronize()
            eng.forward_noalloc(d_tok, ctx, skip, False, d_logits, d_cos, d_am)
            eng.check()
            assert np.array_equal(d_logits.cpu().numpy(), want["logits"]), rows
            assert np.array_equal(d_cos.cpu().numpy(), want["cos"]), rows
            assert np.array_equal(d_am.cpu().numpy(), want["argmax"]), rows
            assert eng.kv_len == ctx
        # committing call, then the cache it wrote serves an ordinary pass
        d_tok = torch.from_numpy(toks[ctx:ctx + 4].copy()).to(dev)
        eng.stream.synchronize()
        eng.forward_noalloc(d_tok, ctx, None, True, None, None, None)
        eng.check()
        assert eng.kv_len == ctx + 4
        a = eng.forward(toks[ctx + 4:ctx + 6], ctx + 4, commit=False)
        eng.truncate(ctx)
        eng.forward(toks[ctx:ctx + 4], ctx)
        b = eng.forward(toks[ctx + 4:ctx + 6], ctx + 4, commit=False)
        assert np.array_equal(a["logits"], b["logits"])
        eng.truncate(ctx)
        # a token id that is not in the vocabulary is flagged, not dereferenced
        bad = torch.tensor([V + 5], dtype=torch.int32, device=dev)
        eng.stream.synchronize()
        eng.forward_noalloc(bad, ctx, None, False, None, None, None)
        with pytest.raises(asd.AsdError) as ei:
            eng.check()
        assert ei.value.code == asd.E_INVAL
    eng.close()


def test_forward_noalloc_refuses_what_does_not_fit():
    shape = si.SHAPES["tiny"]
    eng = asd.Engine(asd.make_config(shape, 128, max_rows=4)).init_synthetic(0)
    dev = eng.device
    t = torch.zeros(8, dtype=torch.int32, device=dev)
    with pytest.raises(asd.AsdError):
        eng.forward_noalloc(t, 0)                      # more rows than max_rows
    with pytest.raises(asd.AsdError):
        eng.forward_noalloc(t[:2], 5)                  # pos0 != kv_len
    eng.close()
    # a context whose attention partials exceed the static array: 32 heads x 128 dims beyond 7680 positions
    big = si.Shape("wide", 1, 4096, 32, 32, 128, 256, 256, si.DT_BF16, 8, 8, 2)
    eng = asd.Engine(asd.make_config(big, 9000, page_tokens=256)).init_synthetic(0)
    toks = si.prompt(1, 8200, big.vocab)
    eng.prefill(toks[:7000])
    t = torch.from_numpy(toks[:4].copy()).to(eng.device)
    eng.forward_noalloc(t, 7000, None, True)           # fits
    eng.check()
    eng.prefill(toks[:8000])
    with pytest.raises(asd.AsdError) as ei:
        eng.forward_noalloc(t, 8000, None, False)
    assert ei.value.code == asd.E_NOMEM
    eng.close()
