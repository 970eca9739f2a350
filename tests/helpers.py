"""Small helpers shared by the tests (no method arithmetic)."""
import numpy as np

import asd_inputs as si
import oracle

SMALL_GQA = si.Shape("small-gqa", 3, 128, 8, 2, 32, 208, 320, si.DT_F32, 12, 10, 3)
SMALL_MHA = si.Shape("small-mha", 2, 64, 4, 4, 16, 112, 96, si.DT_F32, 9, 8, 3)


def make_oracle(shape, seed=0, max_seq=256, gain_std=0.0, kv_storage=False):
    return oracle.Oracle(shape, max_seq, kv_storage).load(si.all_tensors(shape, seed, gain_std))


def weights_dict(shape, seed=0, gain_std=0.0):
    return {(t, l): a for t, l, a in si.all_tensors(shape, seed, gain_std)}
