"""Seeded synthetic inputs shared by the CPU oracle and the HIP engine.

Nothing here belongs to the decoding method: this module only produces the
random-init weights, per-sublayer output scales and prompts that stand in for
trained checkpoints and dataset prompts, plus the table of model shapes used
by the tests and the benchmark.  The generator itself is `synth.c` (compiled
with gcc on first use); its header comment states the counter-based recipe.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
_SRC_PATH = os.path.join(_HERE, "synth.c")

# Tensor identifiers (also the tensor ids of the engine's C ABI).
T_EMBED, T_ATTN_NORM, T_WQ, T_WK, T_WV, T_WO = 0, 1, 2, 3, 4, 5
T_MLP_NORM, T_WG, T_WU, T_WD, T_FINAL_NORM, T_LM_HEAD = 6, 7, 8, 9, 10, 11
T_PROMPT, T_SCALES = 100, 101

DT_F32, DT_BF16 = 0, 1
WEIGHT_STD = 0.02


def build(force: bool = False) -> str:
    """Compile synth.c into libsynth.so (gcc, OpenMP)."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC_PATH):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, _SRC_PATH, "-lm"])
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        L.synth_constant.restype = ctypes.c_float
        L.synth_constant.argtypes = [ctypes.c_double]
        L.synth_uniform.restype = ctypes.c_double
        L.synth_uniform.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint64]
        fill = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_float]
        L.synth_fill_f32.argtypes = fill
        L.synth_fill_bf16.argtypes = fill
        L.synth_sublayer_scales.argtypes = [ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p]
        L.synth_prompt.argtypes = [ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        _lib = L
    return _lib


@dataclass(frozen=True)
class Shape:
    """Llama-style decoder shape (dtype: DT_F32 or DT_BF16 storage of weights and KV)."""
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: int
    prompt_len: int
    n_new: int
    draft_len: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    def with_(self, **kw) -> "Shape":
        return replace(self, **kw)

    @property
    def q_dim(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim


# The five workload configurations (shapes, prompt length, new tokens, draft length).
SHAPES = {
    "tiny": Shape("tiny", 4, 256, 4, 4, 64, 688, 1024, DT_F32, 32, 32, 4),
    "7b": Shape("7b", 32, 4096, 32, 32, 128, 11008, 32000, DT_BF16, 512, 256, 4),
    "13b": Shape("13b", 40, 5120, 40, 40, 128, 13824, 32000, DT_BF16, 1024, 512, 6),
    "7b-long": Shape("7b-long", 32, 4096, 32, 32, 128, 11008, 32000, DT_BF16, 8192, 256, 6),
    "70b": Shape("70b", 80, 8192, 64, 8, 128, 28672, 32000, DT_BF16, 2048, 256, 8),
}


def tensor_shape(s: Shape, tensor: int):
    return {
        T_EMBED: (s.vocab, s.d_model), T_LM_HEAD: (s.vocab, s.d_model),
        T_WQ: (s.q_dim, s.d_model), T_WK: (s.kv_dim, s.d_model), T_WV: (s.kv_dim, s.d_model),
        T_WO: (s.d_model, s.q_dim), T_WG: (s.d_ffn, s.d_model), T_WU: (s.d_ffn, s.d_model),
        T_WD: (s.d_model, s.d_ffn),
        T_ATTN_NORM: (s.d_model,), T_MLP_NORM: (s.d_model,), T_FINAL_NORM: (s.d_model,),
    }[tensor]


GLOBAL_TENSORS = (T_EMBED, T_FINAL_NORM, T_LM_HEAD)
LAYER_TENSORS = (T_ATTN_NORM, T_WQ, T_WK, T_WV, T_WO, T_MLP_NORM, T_WG, T_WU, T_WD)
NORM_TENSORS = (T_ATTN_NORM, T_MLP_NORM, T_FINAL_NORM)


def sublayer_scales(seed: int, n_layers: int) -> np.ndarray:
    """2L log-uniform [1e-3, 1] factors; index 2l scales W_o of layer l, 2l+1 scales W_d."""
    out = np.empty(2 * n_layers, dtype=np.float64)
    lib().synth_sublayer_scales(seed, n_layers, out.ctypes.data)
    return out


def tensor_constant(s: Shape, seed: int, tensor: int, layer: int, scales=None) -> float:
    """The single fp32 multiplier of a matrix tensor (std 0.02, times the sublayer scale for W_o / W_d)."""
    std = WEIGHT_STD
    if tensor in (T_WO, T_WD):
        sc = sublayer_scales(seed, s.n_layers) if scales is None else scales
        std *= float(sc[2 * layer + (0 if tensor == T_WO else 1)])
    return float(lib().synth_constant(std))


def tensor(s: Shape, seed: int, tensor_id: int, layer: int = 0, gain_std: float = 0.0, scales=None) -> np.ndarray:
    """One tensor in its storage form: fp32 array, or uint16 array of bf16 bit patterns.

    Norm gains are fp32 ones (or 1 + gain_std * z when a test wants non-trivial gains).
    """
    shp = tensor_shape(s, tensor_id)
    n = int(np.prod(shp))
    if tensor_id in NORM_TENSORS:
        g = np.ones(n, dtype=np.float32)
        if gain_std > 0.0:
            z = np.empty(n, dtype=np.float32)
            lib().synth_fill_f32(z.ctypes.data, 0, n, seed, tensor_id, layer, lib().synth_constant(gain_std))
            g = (g + z).astype(np.float32)
        return g
    cst = tensor_constant(s, seed, tensor_id, layer, scales)
    if s.dtype == DT_BF16:
        out = np.empty(n, dtype=np.uint16)
        lib().synth_fill_bf16(out.ctypes.data, 0, n, seed, tensor_id, layer, cst)
    else:
        out = np.empty(n, dtype=np.float32)
        lib().synth_fill_f32(out.ctypes.data, 0, n, seed, tensor_id, layer, cst)
    return out.reshape(shp)


def all_tensors(s: Shape, seed: int, gain_std: float = 0.0):
    """Yield (tensor_id, layer, array) for every tensor of the model, one at a time."""
    scales = sublayer_scales(seed, s.n_layers)
    for t in GLOBAL_TENSORS:
        yield t, 0, tensor(s, seed, t, 0, gain_std, scales)
    for l in range(s.n_layers):
        for t in LAYER_TENSORS:
            yield t, l, tensor(s, seed, t, l, gain_std, scales)


def prompt(seed: int, n: int, vocab: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    lib().synth_prompt(seed, n, vocab, out.ctypes.data)
    return out


T_SAMPLING = 102      # stream id of the uniforms drawn by sampled decoding


def sampling_uniform(seed: int, index: int, purpose: int) -> float:
    """Uniform in [0, 1) of the sampling stream for output index `index` (purpose 0 draft, 1 accept test, 2 token draw)."""
    return float(lib().synth_uniform(seed, T_SAMPLING, 0, 3 * index + purpose))


def bf16_to_f32(a: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 values (exact)."""
    return (a.astype(np.uint32) << 16).view(np.float32)


def as_f64(a: np.ndarray) -> np.ndarray:
    """Storage form -> float64 values (exact)."""
    return (bf16_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)


def fixed_keep_mask(n_layers: int, period: int) -> np.ndarray:
    """Skip mask [2L] (1 = skip) keeping both sublayers of layer i iff i % period == 0."""
    m = np.ones(2 * n_layers, dtype=np.uint8)
    for i in range(0, n_layers, period):
        m[2 * i] = m[2 * i + 1] = 0
    return m
