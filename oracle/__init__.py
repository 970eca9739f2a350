"""CPU oracle (test infrastructure only): ctypes binding of asd_oracle.c.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the HIP engine.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "asd_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (OpenMP over independent output elements)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "max_seq", "dtype")] + \
               [("rms_eps", ctypes.c_double), ("rope_theta", ctypes.c_double), ("kv_storage", ctypes.c_int32)]


class _GenParams(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_double), ("m", ctypes.c_int32), ("n", ctypes.c_int32),
                ("use_cs", ctypes.c_int32), ("draft_len", ctypes.c_int32), ("mask_mode", ctypes.c_int32),
                ("fixed_mask", ctypes.c_void_p)]


class _GenStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("cycles", "drafted", "accepted", "emitted")]


class _AdaptParams(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_double), ("m", ctypes.c_int32), ("n", ctypes.c_int32), ("use_cs", ctypes.c_int32),
                ("alpha_mlp", ctypes.c_double), ("use_cs_mlp", ctypes.c_int32), ("refresh", ctypes.c_int32),
                ("fixed_mask", ctypes.c_void_p), ("draft_len", ctypes.c_int32), ("exit_mode", ctypes.c_int32),
                ("gamma0", ctypes.c_double), ("ar0", ctypes.c_double), ("ar_target", ctypes.c_double),
                ("eps", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double)]


class _AdaptStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("cycles", "drafted", "accepted", "emitted", "mask_changes")] + \
               [("gamma", ctypes.c_double), ("ar", ctypes.c_double)]


_lib = None


def _L():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.orc_create.restype = vp
        L.orc_create.argtypes = [ctypes.POINTER(_Config)]
        L.orc_destroy.argtypes = [vp]
        L.orc_set_weight.argtypes = [vp, i32, i32, vp]
        L.orc_reset.argtypes = [vp]
        L.orc_truncate.argtypes = [vp, i32]
        L.orc_kv_len.argtypes = [vp]
        L.orc_get_kv.argtypes = [vp, i32, i32, i32, vp, vp]
        L.orc_forward.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, vp, vp]
        L.orc_acs.argtypes = [vp, i32, i32, vp]
        L.orc_cosine.restype = ctypes.c_double
        L.orc_cosine.argtypes = [vp, vp, i32]
        L.orc_admg.argtypes = [vp, i32, ctypes.c_double, i32, i32, i32, vp]
        L.orc_generate_plain.argtypes = [vp, vp, i32, i32, vp]
        L.orc_generate_spec.argtypes = [vp, vp, i32, i32, ctypes.POINTER(_GenParams), vp,
                                        ctypes.POINTER(_GenStats), vp, vp]
        L.orc_top1_prob.restype = ctypes.c_double
        L.orc_top1_prob.argtypes = [vp, i32]
        dp = ctypes.POINTER(ctypes.c_double)
        L.orc_exit_update.restype = None
        L.orc_exit_update.argtypes = [dp, dp, i32, i32] + [ctypes.c_double] * 4
        L.orc_admg2.argtypes = [vp, i32, ctypes.c_double, i32, i32, i32, ctypes.c_double, i32, vp]
        L.orc_generate_adaptive.argtypes = [vp, vp, i32, i32, ctypes.POINTER(_AdaptParams), vp,
                                            ctypes.POINTER(_AdaptStats), vp, vp, vp]
        u64, f64 = ctypes.c_uint64, ctypes.c_double
        L.orc_uniform.restype = f64
        L.orc_uniform.argtypes = [u64, ctypes.c_int64, i32]
        L.orc_sample_weights.argtypes = [vp, i32, f64, dp]
        L.orc_sample_logits.argtypes = [vp, i32, f64, f64, dp]
        L.orc_spec_accept.argtypes = [vp, vp, vp, i32, i32, f64, vp, vp, ctypes.POINTER(i32), dp]
        L.orc_generate_sampled.argtypes = [vp, vp, i32, i32, i32, vp, f64, u64, vp, ctypes.POINTER(_GenStats), dp]
        _lib = L
    return _lib


def cosine(x, y) -> float:
    x = np.ascontiguousarray(x, dtype=np.float64)
    y = np.ascontiguousarray(y, dtype=np.float64)
    return float(_L().orc_cosine(x.ctypes.data, y.ctypes.data, x.size))


def admg(C_attn, alpha: float, m: int, n: int, use_cs: bool = True) -> np.ndarray:
    """Algorithm 1: skip mask [2L] (index 2l attention, 2l+1 MLP, 0-based l; 1 = removed)."""
    C = np.ascontiguousarray(C_attn, dtype=np.float64)
    mask = np.zeros(2 * C.size, dtype=np.uint8)
    rc = _L().orc_admg(C.ctypes.data, C.size, alpha, m, n, int(use_cs), mask.ctypes.data)
    if rc:
        raise ValueError("orc_admg: invalid argument")
    return mask


def admg2(C_all, alpha: float, m: int, n: int, use_cs: bool = True, alpha_mlp: float = 2.0,
          use_cs_mlp: bool = False) -> np.ndarray:
    """Algorithm 1 plus CS thresholding of the MLP sublayers; C_all [2L] (attention, MLP interleaved)."""
    C = np.ascontiguousarray(C_all, dtype=np.float64)
    mask = np.zeros(C.size, dtype=np.uint8)
    rc = _L().orc_admg2(C.ctypes.data, C.size // 2, alpha, m, n, int(use_cs), alpha_mlp, int(use_cs_mlp), mask.ctypes.data)
    if rc:
        raise ValueError("orc_admg2: invalid argument")
    return mask


def top1_prob(logits) -> float:
    lg = np.ascontiguousarray(logits, dtype=np.float64)
    return float(_L().orc_top1_prob(lg.ctypes.data, lg.size))


def exit_update(ar: float, gamma: float, a: int, d: int, ar_target: float, eps: float, beta1: float, beta2: float):
    """One threshold update of the adaptive draft exit; returns (ar, gamma)."""
    x, y = ctypes.c_double(ar), ctypes.c_double(gamma)
    _L().orc_exit_update(ctypes.byref(x), ctypes.byref(y), a, d, ar_target, eps, beta1, beta2)
    return x.value, y.value


def uniform(seed: int, index: int, purpose: int) -> float:
    """The sampling stream's uniform for output index `index`: purpose 0 draft, 1 accept test, 2 replacement / extra / plain."""
    return float(_L().orc_uniform(seed, index, purpose))


def sample_weights(w, u: float):
    """Inverse-CDF draw from non-negative weights; returns (index, relative margin to the nearer bin boundary)."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    mg = ctypes.c_double()
    return int(_L().orc_sample_weights(w.ctypes.data, w.size, u, ctypes.byref(mg))), mg.value


def sample_logits(logits, T: float, u: float):
    lg = np.ascontiguousarray(logits, dtype=np.float64)
    mg = ctypes.c_double()
    return int(_L().orc_sample_logits(lg.ctypes.data, lg.size, T, u, ctypes.byref(mg))), mg.value


def spec_accept(q_logits, p_logits, x, T: float, u_acc, u_res):
    """Speculative-sampling verification of drafts x [kk]; returns (accepted count, next token, smallest margin)."""
    q = np.ascontiguousarray(q_logits, dtype=np.float64)
    p = np.ascontiguousarray(p_logits, dtype=np.float64)
    xs = np.ascontiguousarray(x, dtype=np.int32)
    kk, V = xs.size, p.shape[-1]
    assert p.shape == (kk + 1, V) and (kk == 0 or q.shape == (kk, V))
    ua = np.ascontiguousarray(u_acc, dtype=np.float64)
    ur = np.ascontiguousarray(u_res, dtype=np.float64)
    assert ua.size >= kk and ur.size >= kk + 1
    nxt, mg = ctypes.c_int32(), ctypes.c_double()
    a = _L().orc_spec_accept(q.ctypes.data, p.ctypes.data, xs.ctypes.data, kk, V, T, ua.ctypes.data, ur.ctypes.data,
                             ctypes.byref(nxt), ctypes.byref(mg))
    return int(a), int(nxt.value), mg.value


def acs(cos_rows) -> np.ndarray:
    cr = np.ascontiguousarray(cos_rows, dtype=np.float64)
    out = np.empty(cr.shape[1], dtype=np.float64)
    _L().orc_acs(cr.ctypes.data, cr.shape[0], cr.shape[1], out.ctypes.data)
    return out


class Oracle:
    """One model instance: weights in storage type; the KV cache keeps K / V as computed (double), or, with
    kv_storage=True, rounded to the model's storage type as the workloads define their caches."""

    def __init__(self, shape, max_seq: int, kv_storage: bool = False):
        self.shape = shape
        self.max_seq = max_seq
        c = _Config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                    shape.d_ffn, shape.vocab, max_seq, shape.dtype, shape.rms_eps, shape.rope_theta, int(kv_storage))
        self._h = _L().orc_create(ctypes.byref(c))
        if not self._h:
            raise ValueError("orc_create: invalid configuration")

    def close(self):
        if self._h:
            _L().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown
            pass

    def set_weight(self, tensor: int, layer: int, arr: np.ndarray):
        a = np.ascontiguousarray(arr)
        if _L().orc_set_weight(self._h, tensor, layer, a.ctypes.data):
            raise ValueError("orc_set_weight failed")

    def load(self, tensors):
        for t, l, a in tensors:
            self.set_weight(t, l, a)
        return self

    def reset(self):
        _L().orc_reset(self._h)

    def truncate(self, n: int):
        if _L().orc_truncate(self._h, n):
            raise ValueError("orc_truncate: bad length")

    @property
    def kv_len(self) -> int:
        return _L().orc_kv_len(self._h)

    def get_kv(self, layer: int, pos0: int, n: int):
        """(K, V) of positions pos0 .. pos0+n-1 of one layer as the cache holds them: float64 [n, n_kv_heads, head_dim]."""
        k = np.empty((n, self.shape.n_kv_heads, self.shape.head_dim))
        v = np.empty_like(k)
        if _L().orc_get_kv(self._h, layer, pos0, n, k.ctypes.data, v.ctypes.data):
            raise ValueError("orc_get_kv: bad layer or positions")
        return k, v

    def forward(self, tokens, pos0: int, skip=None, commit: bool = True, want_logits=True, want_hidden=False):
        """Returns dict(logits [n,V], cos_rows [n,2L], cos [2L] mean over rows, argmax [n], hidden [n,d])."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        n, s = tok.size, self.shape
        logits = np.empty((n, s.vocab), dtype=np.float64) if want_logits else None
        cos_rows = np.empty((n, 2 * s.n_layers), dtype=np.float64)
        am = np.empty(n, dtype=np.int32)
        hid = np.empty((n, s.d_model), dtype=np.float64) if want_hidden else None
        sk = None if skip is None else np.ascontiguousarray(skip, dtype=np.uint8)
        rc = _L().orc_forward(self._h, tok.ctypes.data, n, pos0, None if sk is None else sk.ctypes.data,
                              int(commit), None if logits is None else logits.ctypes.data,
                              cos_rows.ctypes.data, am.ctypes.data, None if hid is None else hid.ctypes.data)
        if rc:
            raise ValueError(f"orc_forward failed ({rc})")
        return {"logits": logits, "cos_rows": cos_rows, "cos": acs(cos_rows), "argmax": am, "hidden": hid}

    def generate_plain(self, prompt, n_new: int) -> np.ndarray:
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(n_new, dtype=np.int32)
        rc = _L().orc_generate_plain(self._h, p.ctypes.data, p.size, n_new, out.ctypes.data)
        if rc:
            raise ValueError(f"orc_generate_plain failed ({rc})")
        return out

    def generate_spec(self, prompt, n_new: int, draft_len: int, alpha=0.985, m=3, n=2, use_cs=True,
                      fixed_mask=None):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(n_new, dtype=np.int32)
        fm = None if fixed_mask is None else np.ascontiguousarray(fixed_mask, dtype=np.uint8)
        gp = _GenParams(alpha, m, n, int(use_cs), draft_len, 0 if fm is None else 1,
                        None if fm is None else fm.ctypes.data)
        st = _GenStats()
        L2 = 2 * self.shape.n_layers
        mask = np.zeros(L2, dtype=np.uint8)
        C = np.zeros(L2, dtype=np.float64)
        rc = _L().orc_generate_spec(self._h, p.ctypes.data, p.size, n_new, ctypes.byref(gp), out.ctypes.data,
                                    ctypes.byref(st), mask.ctypes.data, C.ctypes.data)
        if rc:
            raise ValueError(f"orc_generate_spec failed ({rc})")
        stats = {k: int(getattr(st, k)) for k in ("cycles", "drafted", "accepted", "emitted")}
        return out, stats, mask, C

    def generate_adaptive(self, prompt, n_new: int, draft_len: int, alpha=0.985, m=3, n=2, use_cs=True,
                          alpha_mlp=2.0, use_cs_mlp=False, refresh=False, fixed_mask=None, exit_mode=0,
                          gamma0=0.0, ar0=1.0, ar_target=0.9, eps=0.01, beta1=0.5, beta2=0.9):
        """Speculative loop with a variable draft length and optional mask refresh.
        Returns (tokens, stats, last mask, running ACS [2L], per-cycle (drafted, accepted) [cycles, 2])."""
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(n_new, dtype=np.int32)
        fm = None if fixed_mask is None else np.ascontiguousarray(fixed_mask, dtype=np.uint8)
        gp = _AdaptParams(alpha, m, n, int(use_cs), alpha_mlp, int(use_cs_mlp), int(refresh),
                          None if fm is None else fm.ctypes.data, draft_len, exit_mode,
                          gamma0, ar0, ar_target, eps, beta1, beta2)
        st = _AdaptStats()
        L2 = 2 * self.shape.n_layers
        mask = np.zeros(L2, dtype=np.uint8)
        C = np.zeros(L2, dtype=np.float64)
        per = np.zeros((n_new, 2), dtype=np.int32)
        rc = _L().orc_generate_adaptive(self._h, p.ctypes.data, p.size, n_new, ctypes.byref(gp), out.ctypes.data,
                                        ctypes.byref(st), mask.ctypes.data, C.ctypes.data, per.ctypes.data)
        if rc:
            raise ValueError(f"orc_generate_adaptive failed ({rc})")
        stats = {k: int(getattr(st, k)) for k in ("cycles", "drafted", "accepted", "emitted", "mask_changes")}
        stats["gamma"], stats["ar"] = float(st.gamma), float(st.ar)
        return out, stats, mask, C, per[:stats["cycles"]]

    def generate_sampled(self, prompt, n_new: int, draft_len: int, T: float, seed: int, mask=None):
        """Sampled (temperature T) self-speculative decoding; returns (tokens, stats, smallest decision margin)."""
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(n_new, dtype=np.int32)
        mk = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
        st = _GenStats()
        mg = ctypes.c_double()
        rc = _L().orc_generate_sampled(self._h, p.ctypes.data, p.size, n_new, draft_len, None if mk is None else mk.ctypes.data,
                                       T, seed, out.ctypes.data, ctypes.byref(st), ctypes.byref(mg))
        if rc:
            raise ValueError(f"orc_generate_sampled failed ({rc})")
        return out, {k: int(getattr(st, k)) for k in ("cycles", "drafted", "accepted", "emitted")}, mg.value
