"""The engine reads nothing of the caller's arena that it has not written itself: an arena handed over full of 0xFF
bytes (NaN as bf16 and fp32, -1 as an index or a counter) gives the same bits as one handed over full of zeros, through
every entry point of the path (Section 1's draft / verify cycle, Section 3.2's prompt pass with its ACS, a forward pass
under a mask, sampled decoding).

What this catches: a weight matrix's zero padding of the K range (d_ffn 208 is not a whole k-block) or a norm gain left
to the allocator; a partial-sum, arrival-counter, candidate, state or page-table word that asd_create does not set and
a kernel reads before writing; a cache slot that is read before the library wrote or cleared it.  The page table is a
permutation, so every cache access goes through it, and the capacity leaves whole pages that are never written."""
import numpy as np
import pytest

import asd_inputs as si
import paper_2410_01028_amd as asd
from helpers import SMALL_GQA
from test_gpu_parity import BF_GQA

pytestmark = pytest.mark.gpu


def run_everything(shape, fill):
    W = list(si.all_tensors(shape, 11))
    eng = asd.Engine(asd.make_config(shape, 768, page_tokens=64), arena_fill=fill).load(W)
    eng.set_page_table(np.random.default_rng(5).permutation(12))
    toks = si.prompt(2, 400, shape.vocab)
    out = {}
    first, acs, lg = eng.prefill(toks[:300], want_logits=True)          # prompt pass in blocks (300 rows: ragged)
    out["prefill"] = (np.array([first]), acs, lg)
    g = eng.forward(toks[300:305], 300)                                  # 5-row pass across the 320 chunk boundary - 16
    out["forward5"] = (g["logits"], g["cos_rows"], g["argmax"])
    mask = si.fixed_keep_mask(shape.n_layers, 2)
    g = eng.forward(toks[305:306], 305, mask)                            # a draft-style row under a mask
    out["masked1"] = (g["logits"], g["cos_rows"], g["argmax"])
    eng.reset()
    first, acs, lg = eng.prefill(toks[:13], want_logits=True, chunked=True)   # the multi-row kernels on a short prompt
    out["prefill_chunked"] = (np.array([first]), acs, lg)
    eng.reset()
    for name, kw in (("spec_fixed_mask", dict(fixed_mask=mask)), ("spec_admg", dict(alpha=0.9, m=3, n=1)),
                     ("sampled", dict(alpha=0.9, m=0, n=0, temperature=0.7, seed=3))):
        toks_out, stats, _ = eng.generate(toks[:70], 40, 4, **kw)
        out[name] = (toks_out, np.array([stats["cycles"], stats["drafted"], stats["accepted"]]))
    eng.close()
    return out


@pytest.mark.parametrize("shape", [BF_GQA, SMALL_GQA], ids=["bf16-gqa", "fp32-gqa"])
def test_arena_of_ff_bytes_gives_the_same_bits_as_an_arena_of_zeros(shape):
    clean = run_everything(shape, 0x00)
    dirty = run_everything(shape, 0xFF)
    for name in clean:
        for a, b in zip(clean[name], dirty[name]):
            a, b = np.asarray(a), np.asarray(b)
            assert np.all(np.isfinite(b.astype(np.float64))), name
            assert np.array_equal(a, b), name
