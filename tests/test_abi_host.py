"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its
host-only entry points (arena sizing, Algorithm 1, argument validation) behave."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import asd_inputs as si
import oracle
import paper_2410_01028_amd as asd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "asd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(asd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 20 and "asd_generate" in names and "asd_forward" in names
    L = asd.lib()
    for n in names:
        assert hasattr(L, n), f"libasd.so does not export {n}"


def test_arena_sizing_and_config_validation():
    s = si.SHAPES["7b"]
    cfg = asd.make_config(s, 1024)
    need = asd.arena_bytes(cfg)
    weights = 2 * (2 * s.vocab * s.d_model + s.n_layers * (4 * s.d_model * s.d_model + 3 * s.d_model * s.d_ffn))
    kv = 2 * s.n_layers * 2 * 1024 * s.n_kv_heads * s.head_dim
    assert weights + kv < need < weights + kv + (1 << 30)
    for field, bad in (("dtype", 7), ("d_model", 100), ("head_dim", 48), ("page_tokens", 100), ("max_rows", 17),
                       ("n_kv_heads", 5), ("max_seq", 0), ("vocab", 1001)):
        c = asd.make_config(s, 1024)
        setattr(c, field, bad)
        assert asd.arena_bytes(c) == 0, field
    # create without a device arena is refused before any device call
    h = ctypes.c_void_p()
    assert asd.lib().asd_create(ctypes.byref(cfg), None, need, None, ctypes.byref(h)) == asd.E_INVAL
    assert b"arena" in asd.lib().asd_last_error(None)
    assert asd.lib().asd_create(None, None, 0, None, ctypes.byref(h)) == asd.E_INVAL


def test_capacity_beyond_the_attention_merge_limit_is_refused():
    """The decode-attention merge keeps the statistics of at most 256 groups of 256 keys per head: a cache of more than
    65536 positions (after rounding up to whole pages) is refused when the engine is sized, not silently truncated."""
    s = si.SHAPES["tiny"]
    assert asd.arena_bytes(asd.make_config(s, asd.MAX_SEQ, page_tokens=256)) > 0
    assert asd.arena_bytes(asd.make_config(s, asd.MAX_SEQ + 1, page_tokens=256)) == 0
    assert asd.arena_bytes(asd.make_config(s, asd.MAX_SEQ - 36, page_tokens=192)) == 0      # 342 pages of 192 = 65664: rounds up past the limit
    h = ctypes.c_void_p()
    cfg = asd.make_config(s, asd.MAX_SEQ + 1, page_tokens=256)
    assert asd.lib().asd_create(ctypes.byref(cfg), None, 1 << 40, None, ctypes.byref(h)) == asd.E_INVAL
    assert b"ASD_MAX_SEQ" in asd.lib().asd_last_error(None)


def test_debug_switches_are_configuration_fields_not_environment(monkeypatch):
    """Launch-shape switches live in the configuration: the library reads no environment variable, so the arena it asks
    for depends on the configuration alone."""
    s = si.SHAPES["7b"]
    base = asd.arena_bytes(asd.make_config(s, 1024))
    for name in ("ASD_TUNE", "ASD_PF_TUNE", "ASD_PERSIST", "ASD_ATT_W4", "ASD_ATT_GH1", "ASD_RS_POW2", "ASD_SAMPLE_MEM"):
        monkeypatch.setenv(name, "qkv=2,8,0,0" if "TUNE" in name else "1")
    assert asd.arena_bytes(asd.make_config(s, 1024)) == base
    tuned = asd.arena_bytes(asd.make_config(s, 1024, debug_flags=asd.DBG_ATT_W4, debug_tune="o=2,8,0,0"))
    assert tuned > 0


def test_admg_matches_oracle_on_all_patterns():
    alpha = 0.985
    for L in range(1, 7):
        for pattern in itertools.product([0.5, 0.985, 0.99], repeat=L):
            C = np.array(pattern, dtype=np.float32)
            for m in range(0, L + 2):
                for n in range(0, L + 2):
                    # alpha is compared in fp32 by the engine; use the fp32 value on both sides
                    want = oracle.admg(C.astype(np.float64), float(np.float32(alpha)), m, n)
                    assert np.array_equal(asd.admg(C, alpha, m, n), want)
    rng = np.random.default_rng(0)
    for _ in range(100):
        L = int(rng.integers(1, 81))
        C = rng.uniform(0.9, 1.0, L).astype(np.float32)
        m, n, cs = int(rng.integers(0, 6)), int(rng.integers(0, 5)), bool(rng.integers(0, 2))
        assert np.array_equal(asd.admg(C, alpha, m, n, cs), oracle.admg(C.astype(np.float64), float(np.float32(alpha)), m, n, cs))


def test_admg_rejects_bad_arguments():
    C = np.zeros(4, np.float32)
    for args in ((1.5, 3, 2), (0.0, 3, 2), (0.985, -1, 2), (0.985, 3, -1)):
        with pytest.raises(asd.AsdError):
            asd.admg(C, *args)
    assert asd.lib().asd_admg(None, 4, 0.985, 3, 2, 1, None) == asd.E_INVAL
    assert asd.admg(C, 7.0, 3, 2, use_cs=False).sum() == 0 + 0   # alpha unused without CS thresholding: L=4, m=3, n=2 removes nothing


def test_null_engine_is_refused():
    L = asd.lib()
    assert L.asd_reset(None) == asd.E_INVAL
    assert L.asd_truncate(None, 0) == asd.E_INVAL
    assert L.asd_forward(None, None, 1, 0, None, 1, None, None, None, None) == asd.E_INVAL
    assert L.asd_generate(None, None, 1, 1, None, None, None, None) == asd.E_INVAL


def test_admg2_matches_oracle_and_reduces_to_admg():
    rng = np.random.default_rng(5)
    for _ in range(300):
        L = int(rng.integers(1, 40))
        C = rng.uniform(0.9, 1.0, 2 * L).astype(np.float32)
        alpha, amlp = float(np.float32(rng.uniform(0.9, 0.999))), float(np.float32(rng.uniform(0.9, 0.999)))
        m, n = int(rng.integers(0, 6)), int(rng.integers(0, 5))
        cs, csm = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        want = oracle.admg2(C.astype(np.float64), alpha, m, n, cs, amlp, csm)
        assert np.array_equal(asd.admg2(C, alpha, m, n, cs, amlp, csm), want)
        assert np.array_equal(asd.admg2(C, alpha, m, n, cs), asd.admg(C[0::2], alpha, m, n, cs))
    with pytest.raises(asd.AsdError):
        asd.admg2(np.zeros(8, np.float32), 0.9, 1, 1, True, 1.5, True)
