"""Seeded synthetic inputs (numpy uint16 arrays holding bf16 bit patterns).

Serves both the CPU oracle's tests and the GPU harness; contains no operator
arithmetic.  Tensor ids are fixed per role so a tensor can be regenerated
anywhere from (seed, role) alone.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libvte_inputs.so")
_lib = None

# tensor roles -> ids (arbitrary but frozen)
T_X, T_GAMMA, T_BETA, T_W, T_XB = 1, 2, 3, 4, 5
T_EMB, T_WQKV, T_WO, T_WGU, T_WD, T_WLM, T_TOK0 = 10, 11, 12, 13, 14, 15, 16
T_GEMM_A, T_GEMM_B = 20, 21


def build(force=False):
    src = os.path.join(_HERE, "gen.cpp")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-pthread",
                               "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        L = ctypes.CDLL(_LIB_PATH)
        u64, i64, dbl, i32, vp = ctypes.c_uint64, ctypes.c_int64, ctypes.c_double, ctypes.c_int, ctypes.c_void_p
        L.vte_gen_normal_bf16.argtypes = [u64, u64, i64, i64, dbl, dbl, vp, i32]
        L.vte_gen_uniform_bf16.argtypes = [u64, u64, i64, dbl, dbl, vp, i32]
        L.vte_gen_int_bf16.argtypes = [u64, u64, i64, i32, i32, i32, vp, i32]
        L.vte_gen_tokens.argtypes = [u64, u64, i64, i64, vp]
        for f in (L.vte_gen_normal_bf16, L.vte_gen_uniform_bf16, L.vte_gen_int_bf16, L.vte_gen_tokens):
            f.restype = None
        _lib = L
    return _lib


def _threads():
    return max(1, min(16, os.cpu_count() or 1))


def normal_bf16(seed, tensor, shape, mean=0.0, std=1.0, out=None):
    n = int(np.prod(shape))
    a = np.empty(n, dtype=np.uint16) if out is None else out.reshape(-1)
    _load().vte_gen_normal_bf16(seed, tensor, 0, n, mean, std, a.ctypes.data, _threads())
    return a.reshape(shape)


def uniform_bf16(seed, tensor, shape, lo, hi):
    n = int(np.prod(shape))
    a = np.empty(n, dtype=np.uint16)
    _load().vte_gen_uniform_bf16(seed, tensor, n, lo, hi, a.ctypes.data, _threads())
    return a.reshape(shape)


def int_bf16(seed, tensor, shape, lo, hi, scale_pow2=0):
    """Integers in [lo, hi] (|v| < 256) times 2**scale_pow2: exact in bf16."""
    n = int(np.prod(shape))
    a = np.empty(n, dtype=np.uint16)
    _load().vte_gen_int_bf16(seed, tensor, n, lo, hi, scale_pow2, a.ctypes.data, _threads())
    return a.reshape(shape)


def tokens(seed, tensor, n, vocab):
    a = np.empty(n, dtype=np.int32)
    _load().vte_gen_tokens(seed, tensor, n, vocab, a.ctypes.data)
    return a


def bf16_bits(values):
    """float array whose values are exactly representable in bf16 -> bit patterns."""
    f = np.ascontiguousarray(values, dtype=np.float32)
    u = f.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "value not exactly representable in bf16"
    return (u >> 16).astype(np.uint16)


def bf16_to_f32(bits):
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


# ---- the workloads of the benchmark configurations -----------------------------

def rmsnorm_case(seed=0, rows=8, cols=1024):
    """x ~ N(0,1), gamma ~ U(0.5,1.5)."""
    return (normal_bf16(seed, T_X, (rows, cols)), uniform_bf16(seed, T_GAMMA, (cols,), 0.5, 1.5))


def layernorm_case(seed=0, rows=8, cols=1024):
    x, g = rmsnorm_case(seed, rows, cols)
    return x, g, normal_bf16(seed, T_BETA, (cols,), 0.0, 0.5)


def gemv_case(seed=0, B=1, N=4096, K=4096, w_std=None, w_tensor=T_W):
    """W ~ N(0, 1/K) (std K**-0.5) unless w_std is given, X ~ N(0,1)."""
    std = K ** -0.5 if w_std is None else w_std
    return normal_bf16(seed, w_tensor, (N, K), 0.0, std), normal_bf16(seed, T_XB, (B, K))


class DecodeShapes:
    """Llama-8B-shaped single-layer chain; `scale` shrinks every dimension for tests."""

    def __init__(self, D=4096, Nqkv=6144, F=14336, V=128256):
        self.D, self.Nqkv, self.F, self.V = D, Nqkv, F, V

    def weight_bytes(self):
        D, Nq, F, V = self.D, self.Nqkv, self.F, self.V
        return 2 * (Nq * D + D * D + 2 * F * D + D * F + V * D)


def decode_weights(seed, shp, with_embedding=True):
    """bf16 weights ~ N(0, 0.02), E ~ N(0,1), gamma ~ U(0.5,1.5)."""
    D, Nq, F, V = shp.D, shp.Nqkv, shp.F, shp.V
    w = {
        "gamma": uniform_bf16(seed, T_GAMMA, (D,), 0.5, 1.5),
        "Wqkv": normal_bf16(seed, T_WQKV, (Nq, D), 0.0, 0.02),
        "Wo": normal_bf16(seed, T_WO, (D, D), 0.0, 0.02),
        "Wgu": normal_bf16(seed, T_WGU, (2 * F, D), 0.0, 0.02),
        "Wd": normal_bf16(seed, T_WD, (D, F), 0.0, 0.02),
        "Wlm": normal_bf16(seed, T_WLM, (V, D), 0.0, 0.02),
    }
    if with_embedding:
        w["E"] = normal_bf16(seed, T_EMB, (V, D), 0.0, 1.0)
    return w


def embedding_rows(seed, shp, toks):
    """Rows E[toks] of the N(0,1) embedding table without materialising the table."""
    out = np.empty((len(toks), shp.D), dtype=np.uint16)
    for i, t in enumerate(toks):
        _load().vte_gen_normal_bf16(seed, T_EMB, int(t) * shp.D, shp.D, 0.0, 1.0, out[i].ctypes.data, 1)
    return out
