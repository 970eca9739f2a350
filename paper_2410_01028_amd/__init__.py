"""MI355X engine for adaptive self-speculative decoding: thin ctypes binding of libasd.so.

Argument marshalling only: every step of the decoding path runs in the HIP kernels
of the C-ABI library declared in include/asd.h.  PyTorch supplies device memory
(the arena) and the stream.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libasd.so")

OK, E_INVAL, E_STATE, E_NOMEM, E_IO, E_HIP = 0, -1, -2, -3, -4, -5
DT_F32, DT_BF16 = 0, 1
MAX_ROWS = 16
MAX_SEQ = 65536
# development / test switches of Config.debug_flags (none changes what is computed)
DBG_ATT_W4, DBG_ATT_GH1, DBG_RS_POW2, DBG_SAMPLE_MEM = 1, 2, 4, 8
KERNEL_CLASSES = ("embed", "qkv", "attn", "oproj", "gateup", "down", "lmhead", "finish")


class AsdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"asd error {code}: {msg}")
        self.code = code


class Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
                 "max_seq", "page_tokens", "max_rows", "dtype")] + \
               [("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float),
                ("debug_flags", ctypes.c_uint32), ("debug_tune", ctypes.c_char_p)]


class GenParams(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_float), ("m", ctypes.c_int32), ("n", ctypes.c_int32), ("use_cs", ctypes.c_int32),
                ("draft_len", ctypes.c_int32), ("mask_mode", ctypes.c_int32), ("fixed_mask", ctypes.c_void_p),
                ("use_graphs", ctypes.c_int32), ("alpha_mlp", ctypes.c_float), ("use_cs_mlp", ctypes.c_int32),
                ("exit_mode", ctypes.c_int32)] + \
               [(n, ctypes.c_double) for n in ("gamma0", "ar0", "ar_target", "eps", "beta1", "beta2")] + \
               [("temperature", ctypes.c_float), ("seed", ctypes.c_uint64), ("sample_index0", ctypes.c_int64)]


class GenStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("cycles", "drafted", "accepted", "emitted")] + \
               [("ms_prefill", ctypes.c_double), ("ms_decode", ctypes.c_double), ("mask_changes", ctypes.c_int64),
                ("gamma", ctypes.c_double), ("ar", ctypes.c_double)] + \
               [(n, ctypes.c_double) for n in ("ms_draft", "ms_verify", "ms_other", "bytes_draft", "bytes_verify")]


PREFILL_CLASSES = ("rows", "qkv", "attn", "oproj", "gateup", "down", "lmhead")


class PrefillTimes(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_double * 7), ("launches", ctypes.c_int32 * 7), ("flops", ctypes.c_double * 7),
                ("ms_total", ctypes.c_double)]


class KernelTimes(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_double * 8), ("launches", ctypes.c_int32 * 8), ("bytes", ctypes.c_double * 8),
                ("ms_total", ctypes.c_double)]


_lib = None


def lib():
    """Load libasd.so (built by paper_2410_01028_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2410_01028_amd.build` first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        cfgp = ctypes.POINTER(Config)
        L.asd_arena_bytes.restype = sz
        L.asd_arena_bytes.argtypes = [cfgp]
        L.asd_create.argtypes = [cfgp, vp, sz, vp, ctypes.POINTER(vp)]
        L.asd_destroy.argtypes = [vp]
        L.asd_destroy.restype = None
        L.asd_last_error.restype = ctypes.c_char_p
        L.asd_last_error.argtypes = [vp]
        L.asd_set_weight.argtypes = [vp, i32, i32, vp, sz, i32]
        L.asd_get_weight.argtypes = [vp, i32, i32, vp, sz]
        L.asd_get_kv.argtypes = [vp, i32, i32, i32, vp, vp]
        L.asd_init_synthetic.argtypes = [vp, ctypes.c_uint64]
        L.asd_load_weights_file.argtypes = [vp, ctypes.c_char_p]
        L.asd_set_page_table.argtypes = [vp, vp, i32]
        L.asd_reset.argtypes = [vp]
        L.asd_truncate.argtypes = [vp, i32]
        L.asd_kv_len.argtypes = [vp]
        L.asd_forward.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, vp, vp]
        L.asd_forward_noalloc.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, vp]
        L.asd_check.argtypes = [vp]
        L.asd_prefill.argtypes = [vp, vp, i32, vp, vp, vp]
        L.asd_prefill_chunked.argtypes = [vp, vp, i32, vp, vp, vp]
        L.asd_admg2.argtypes = [vp, i32, ctypes.c_float, i32, i32, i32, ctypes.c_float, i32, vp]
        L.asd_admg.argtypes = [vp, i32, ctypes.c_float, i32, i32, i32, vp]
        L.asd_spec_sample.argtypes = [vp, vp, vp, i32, ctypes.c_float, ctypes.c_uint64, ctypes.c_int64, vp, vp, vp]
        L.asd_decode.argtypes = [vp, i32, i32, ctypes.POINTER(GenParams), vp, ctypes.POINTER(GenStats), vp]
        L.asd_generate.argtypes = [vp, vp, i32, i32, ctypes.POINTER(GenParams), vp, ctypes.POINTER(GenStats), vp]
        L.asd_time_pass.argtypes = [vp, i32, vp, i32, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.asd_profile_forward.argtypes = [vp, i32, vp, ctypes.POINTER(KernelTimes)]
        L.asd_copy_bench.argtypes = [vp, sz, i32, ctypes.POINTER(ctypes.c_double)]
        L.asd_profile_prefill.argtypes = [vp, vp, i32, ctypes.POINTER(PrefillTimes)]
        L.asd_time_step_class.argtypes = [vp, i32, i32, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        _lib = L
    return _lib


def make_config(shape, max_seq: int, page_tokens: int = 64, max_rows: int = MAX_ROWS, debug_flags: int = 0,
                debug_tune: str | None = None) -> Config:
    """Config from any object with the shape fields (n_layers, d_model, ..., dtype, rms_eps, rope_theta)."""
    return Config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                  shape.vocab, max_seq, page_tokens, max_rows, shape.dtype, shape.rms_eps, shape.rope_theta,
                  debug_flags, None if debug_tune is None else debug_tune.encode())


def arena_bytes(cfg: Config) -> int:
    return int(lib().asd_arena_bytes(ctypes.byref(cfg)))


def admg(c_attn, alpha: float, m: int, n: int, use_cs: bool = True) -> np.ndarray:
    """Algorithm 1 on the host: skip mask [2L] from the attention sublayers' ACS."""
    c = np.ascontiguousarray(c_attn, dtype=np.float32)
    mask = np.zeros(2 * c.size, dtype=np.uint8)
    rc = lib().asd_admg(c.ctypes.data, c.size, alpha, m, n, int(use_cs), mask.ctypes.data)
    if rc:
        raise AsdError(rc, "asd_admg: invalid argument")
    return mask


def admg2(c_all, alpha: float, m: int, n: int, use_cs: bool = True, alpha_mlp: float = 0.0, use_cs_mlp: bool = False) -> np.ndarray:
    """Algorithm 1 plus CS thresholding of the MLP sublayers, from all 2L ACS values (attention, MLP interleaved)."""
    c = np.ascontiguousarray(c_all, dtype=np.float32)
    mask = np.zeros(c.size, dtype=np.uint8)
    rc = lib().asd_admg2(c.ctypes.data, c.size // 2, alpha, m, n, int(use_cs), alpha_mlp, int(use_cs_mlp), mask.ctypes.data)
    if rc:
        raise AsdError(rc, "asd_admg2: invalid argument")
    return mask


def _ptr(a):
    return None if a is None else a.ctypes.data


class Engine:
    """One engine on the current CUDA/HIP device; owns a torch uint8 arena it lends to the library."""

    def __init__(self, cfg: Config, device: str = "cuda:0", arena_fill: int | None = None):
        """arena_fill: byte value the arena is filled with before the library sees it (tests: every region the
        library reads must have been written by the library first); None leaves the allocator's bytes."""
        import torch
        self._torch = torch
        self.cfg = cfg
        need = arena_bytes(cfg)
        if need == 0:
            raise AsdError(E_INVAL, "invalid configuration")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.arena = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        if arena_fill is not None:
            self.arena.fill_(arena_fill)
            torch.cuda.synchronize(self.device)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        # a stream of its own (default priority): graph capture is not allowed on the legacy default stream
        self.stream = torch.cuda.Stream(self.device)
        h = ctypes.c_void_p()
        rc = lib().asd_create(ctypes.byref(cfg), base, need, self.stream.cuda_stream, ctypes.byref(h))
        if rc:
            raise AsdError(rc, lib().asd_last_error(None).decode())
        self._h = h
        self.L2 = 2 * cfg.n_layers

    def close(self):
        if getattr(self, "_h", None):
            lib().asd_destroy(self._h)
            self._h = None
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown: module globals may already be gone
            pass

    def _ck(self, rc: int):
        if rc:
            raise AsdError(rc, lib().asd_last_error(self._h).decode())

    # ---- weights
    def set_weight(self, tensor: int, layer: int, arr: np.ndarray):
        a = np.ascontiguousarray(arr)
        self._ck(lib().asd_set_weight(self._h, tensor, layer, a.ctypes.data, a.nbytes, 0))

    def get_weight(self, tensor: int, layer: int, shape, dtype) -> np.ndarray:
        out = np.empty(shape, dtype=dtype)
        self._ck(lib().asd_get_weight(self._h, tensor, layer, out.ctypes.data, out.nbytes))
        return out

    def load(self, tensors):
        for t, l, a in tensors:
            self.set_weight(t, l, a)
        return self

    def init_synthetic(self, seed: int):
        self._ck(lib().asd_init_synthetic(self._h, seed))
        return self

    def load_weights_file(self, path: str):
        self._ck(lib().asd_load_weights_file(self._h, path.encode()))
        return self

    # ---- cache
    def set_page_table(self, table):
        t = np.ascontiguousarray(table, dtype=np.int32)
        self._ck(lib().asd_set_page_table(self._h, t.ctypes.data, t.size))

    def get_kv(self, layer: int, pos0: int, n: int):
        """(K, V) of positions pos0 .. pos0+n-1 of one layer: float32 [n, n_kv_heads, head_dim], the stored values widened."""
        k = np.empty((n, self.cfg.n_kv_heads, self.cfg.head_dim), dtype=np.float32)
        v = np.empty_like(k)
        self._ck(lib().asd_get_kv(self._h, layer, pos0, n, k.ctypes.data, v.ctypes.data))
        return k, v

    def reset(self):
        self._ck(lib().asd_reset(self._h))

    def truncate(self, n: int):
        self._ck(lib().asd_truncate(self._h, n))

    @property
    def kv_len(self) -> int:
        return int(lib().asd_kv_len(self._h))

    # ---- passes
    def forward(self, tokens, pos0: int, skip=None, commit: bool = True, want_logits: bool = True):
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        n = tok.size
        logits = np.empty((n, self.cfg.vocab), dtype=np.float32) if want_logits else None
        cos = np.empty(self.L2, dtype=np.float32)
        cos_rows = np.empty((n, self.L2), dtype=np.float32)
        am = np.empty(n, dtype=np.int32)
        sk = None if skip is None else np.ascontiguousarray(skip, dtype=np.uint8)
        self._ck(lib().asd_forward(self._h, tok.ctypes.data, n, pos0, _ptr(sk), int(commit), _ptr(logits),
                                   cos.ctypes.data, cos_rows.ctypes.data, am.ctypes.data))
        return {"logits": logits, "cos": cos, "cos_rows": cos_rows, "argmax": am}

    def forward_noalloc(self, d_tokens, pos0: int, skip=None, commit: bool = True, d_logits=None, d_cos=None, d_argmax=None):
        """asd_forward_noalloc: tokens and outputs are device tensors (int32 [n], float32 [n, V], float32 [2L], int32 [n]);
        enqueues on the engine's stream and returns without synchronising."""
        sk = None if skip is None else np.ascontiguousarray(skip, dtype=np.uint8)
        ptr = lambda t: None if t is None else t.data_ptr()
        self._ck(lib().asd_forward_noalloc(self._h, d_tokens.data_ptr(), d_tokens.numel(), pos0, _ptr(sk), int(commit),
                                           ptr(d_logits), ptr(d_cos), ptr(d_argmax)))

    def check(self):
        """Synchronise the engine's stream and raise if a kernel flagged an error since the last pass started."""
        self._ck(lib().asd_check(self._h))

    def prefill(self, tokens, want_logits: bool = False, chunked: bool = False):
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        first = ctypes.c_int32()
        cos = np.empty(self.L2, dtype=np.float32)
        lg = np.empty(self.cfg.vocab, dtype=np.float32) if want_logits else None
        fn = lib().asd_prefill_chunked if chunked else lib().asd_prefill
        self._ck(fn(self._h, tok.ctypes.data, tok.size, ctypes.byref(first), cos.ctypes.data, _ptr(lg)))
        return int(first.value), cos, lg

    @staticmethod
    def _params(draft_len, alpha=0.985, m=3, n=2, use_cs=True, fixed_mask=None, use_graphs=True, refresh=False,
                alpha_mlp=0.0, use_cs_mlp=False, exit_mode=0, gamma0=0.0, ar0=1.0, ar_target=0.9, eps=0.01, beta1=0.5,
                beta2=0.9, temperature=0.0, seed=0, sample_index0=0):
        fm = None if fixed_mask is None else np.ascontiguousarray(fixed_mask, dtype=np.uint8)
        mode = 1 if fm is not None else (2 if refresh else 0)
        gp = GenParams(alpha, m, n, int(use_cs), draft_len, mode, _ptr(fm), int(use_graphs), alpha_mlp, int(use_cs_mlp),
                       exit_mode, gamma0, ar0, ar_target, eps, beta1, beta2, temperature, seed, sample_index0)
        return gp, fm

    def decode(self, last_token: int, n_more: int, draft_len: int, **kw):
        """Speculative decode from the current cache; kw: alpha, m, n, use_cs, fixed_mask, use_graphs, refresh
        (mask rebuilt from the running ACS), alpha_mlp / use_cs_mlp, exit_mode, gamma0, ar0, ar_target, eps, beta1, beta2,
        temperature (> 0: sampled decoding by speculative sampling), seed, sample_index0."""
        gp, fm = self._params(draft_len, **kw)
        out = np.empty(n_more, dtype=np.int32)
        st = GenStats()
        mask = np.zeros(self.L2, dtype=np.uint8)
        self._ck(lib().asd_decode(self._h, last_token, n_more, ctypes.byref(gp), out.ctypes.data, ctypes.byref(st),
                                  mask.ctypes.data))
        return out, self._stats(st), mask

    def generate(self, prompt, n_new: int, draft_len: int, **kw):
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        gp, fm = self._params(draft_len, **kw)
        out = np.empty(n_new, dtype=np.int32)
        st = GenStats()
        mask = np.zeros(self.L2, dtype=np.uint8)
        self._ck(lib().asd_generate(self._h, p.ctypes.data, p.size, n_new, ctypes.byref(gp), out.ctypes.data,
                                    ctypes.byref(st), mask.ctypes.data))
        return out, self._stats(st), mask

    def spec_sample(self, q_logits, p_logits, temperature: float, seed: int, index0: int = 0):
        """The sampling kernels on given logits: q [kk, V] draft, p [kk+1, V] full model; returns (drafts, accepted, next)."""
        p = np.ascontiguousarray(p_logits, dtype=np.float32)
        kk = p.shape[0] - 1
        q = np.ascontiguousarray(q_logits, dtype=np.float32).reshape(kk, p.shape[1]) if kk else None
        drafts = np.zeros(max(kk, 1), dtype=np.int32)
        a, nxt = ctypes.c_int32(), ctypes.c_int32()
        self._ck(lib().asd_spec_sample(self._h, _ptr(q), p.ctypes.data, kk, temperature, seed, index0, drafts.ctypes.data,
                                       ctypes.byref(a), ctypes.byref(nxt)))
        return drafts[:kk], int(a.value), int(nxt.value)

    @staticmethod
    def _stats(st: GenStats) -> dict:
        return {k: getattr(st, k) for k in ("cycles", "drafted", "accepted", "emitted", "ms_prefill", "ms_decode",
                                            "mask_changes", "gamma", "ar", "ms_draft", "ms_verify", "ms_other",
                                            "bytes_draft", "bytes_verify")}

    # ---- measurement
    def time_pass(self, n_rows: int, skip=None, reps: int = 20, use_graph: bool = True):
        sk = None if skip is None else np.ascontiguousarray(skip, dtype=np.uint8)
        ms, by = ctypes.c_double(), ctypes.c_double()
        self._ck(lib().asd_time_pass(self._h, n_rows, _ptr(sk), reps, int(use_graph), ctypes.byref(ms), ctypes.byref(by)))
        return ms.value, by.value

    def profile_forward(self, n_rows: int, skip=None) -> dict:
        sk = None if skip is None else np.ascontiguousarray(skip, dtype=np.uint8)
        kt = KernelTimes()
        self._ck(lib().asd_profile_forward(self._h, n_rows, _ptr(sk), ctypes.byref(kt)))
        out = {name: {"ms": kt.ms[i], "launches": kt.launches[i], "bytes": kt.bytes[i]}
               for i, name in enumerate(KERNEL_CLASSES)}
        out["ms_total"] = kt.ms_total
        return out

    def profile_prefill(self, tokens) -> dict:
        """Per-class GPU time of the prompt pass in blocks (event pair around every launch); resets the cache."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        pt = PrefillTimes()
        self._ck(lib().asd_profile_prefill(self._h, tok.ctypes.data, tok.size, ctypes.byref(pt)))
        out = {name: {"ms": pt.ms[i], "launches": pt.launches[i], "flops": pt.flops[i]} for i, name in enumerate(PREFILL_CLASSES)}
        out["ms_total"] = pt.ms_total
        return out

    def time_step_class(self, name: str, n_rows: int = 1, reps: int = 10):
        """(average microseconds per launch, algorithmic bytes per launch) of one kernel class launched back to back."""
        us, by = ctypes.c_double(), ctypes.c_double()
        self._ck(lib().asd_time_step_class(self._h, KERNEL_CLASSES.index(name), n_rows, reps, ctypes.byref(us), ctypes.byref(by)))
        return us.value, by.value

    def copy_bench(self, nbytes: int, reps: int = 10) -> float:
        ms = ctypes.c_double()
        self._ck(lib().asd_copy_bench(self._h, nbytes, reps, ctypes.byref(ms)))
        return ms.value
