"""ctypes front end of the CPU oracle (oracle/vte_oracle.cpp).  TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
It never imports the HIP library or its binding.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    src = os.path.join(_HERE, "vte_oracle.cpp")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
                               "-pthread", "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.orc_silu.restype = ctypes.c_double
        _lib.orc_silu.argtypes = [ctypes.c_double]
    return _lib


def hardware_threads():
    return int(_load().orc_hardware_threads())


def default_threads():
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, n)


def _u16(a):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return a, ctypes.c_void_p(a.ctypes.data)


def _i64(v):
    return ctypes.c_int64(int(v))


def bf16_to_f64(bits):
    a, p = _u16(bits)
    out = np.empty(a.shape, dtype=np.float64)
    _load().orc_bf16_to_f64(p, _i64(a.size), ctypes.c_void_p(out.ctypes.data))
    return out


def f64_to_bf16(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    _load().orc_f64_to_bf16(ctypes.c_void_p(x.ctypes.data), _i64(x.size), ctypes.c_void_p(out.ctypes.data))
    return out


def rmsnorm(x, gamma, eps=1e-6, threads=None):
    x, px = _u16(x)
    g, pg = _u16(gamma)
    rows, cols = x.shape
    assert g.shape == (cols,)
    out = np.empty((rows, cols), dtype=np.float64)
    _load().orc_rmsnorm(px, pg, _i64(rows), _i64(cols), ctypes.c_double(eps),
                        ctypes.c_void_p(out.ctypes.data), threads or default_threads())
    return out


def layernorm(x, gamma, beta, eps=1e-6, threads=None):
    x, px = _u16(x)
    g, pg = _u16(gamma)
    b, pb = _u16(beta)
    rows, cols = x.shape
    out = np.empty((rows, cols), dtype=np.float64)
    _load().orc_layernorm(px, pg, pb, _i64(rows), _i64(cols), ctypes.c_double(eps),
                          ctypes.c_void_p(out.ctypes.data), threads or default_threads())
    return out


def _gemv_like(fn, W, X, threads):
    W, pw = _u16(W)
    X, px = _u16(X)
    N, K = W.shape
    B, K2 = X.shape
    assert K == K2
    out = np.empty((B, N), dtype=np.float64)
    fn(pw, px, _i64(B), _i64(N), _i64(K), ctypes.c_void_p(out.ctypes.data), threads or default_threads())
    return out


def gemv(W, X, threads=None):
    return _gemv_like(_load().orc_gemv, W, X, threads)


def gemv_reverse(W, X, threads=None):
    return _gemv_like(_load().orc_gemv_reverse, W, X, threads)


def gemv_abs(W, X, threads=None):
    return _gemv_like(_load().orc_gemv_abs, W, X, threads)


def gemv_silu_mul(W, X, threads=None):
    W, pw = _u16(W)
    X, px = _u16(X)
    N2, K = W.shape
    B = X.shape[0]
    Nh = N2 // 2
    out = np.empty((B, Nh), dtype=np.float64)
    _load().orc_gemv_silu_mul(pw, px, _i64(B), _i64(Nh), _i64(K), ctypes.c_void_p(out.ctypes.data),
                              threads or default_threads())
    return out


def silu(g):
    return float(_load().orc_silu(float(g)))


def argmax(logits):
    lg = np.ascontiguousarray(logits, dtype=np.float64)
    B, V = lg.shape
    tok = np.empty(B, dtype=np.int32)
    margin = np.empty(B, dtype=np.float64)
    _load().orc_argmax(ctypes.c_void_p(lg.ctypes.data), _i64(B), _i64(V), ctypes.c_void_p(tok.ctypes.data),
                       ctypes.c_void_p(margin.ctypes.data))
    return tok, margin


def lmhead_argmax(W, H, want_logits=True, threads=None):
    W, pw = _u16(W)
    H, ph = _u16(H)
    V, K = W.shape
    B = H.shape[0]
    logits = np.empty((B, V), dtype=np.float64) if want_logits else None
    tok = np.empty(B, dtype=np.int32)
    margin = np.empty(B, dtype=np.float64)
    _load().orc_lmhead_argmax(pw, ph, _i64(B), _i64(V), _i64(K),
                              ctypes.c_void_p(logits.ctypes.data) if want_logits else None,
                              ctypes.c_void_p(tok.ctypes.data), ctypes.c_void_p(margin.ctypes.data),
                              threads or default_threads())
    return logits, tok, margin


def softmax_prob(logits, tok):
    """Softmax probability of tok[b] under logits[b, :] (float32 values taken as exact), in double."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    tk = np.ascontiguousarray(tok, dtype=np.int32)
    B, V = lg.shape
    out = np.empty(B, dtype=np.float64)
    _load().orc_softmax_prob(ctypes.c_void_p(lg.ctypes.data), ctypes.c_void_p(tk.ctypes.data), _i64(B), _i64(V),
                             ctypes.c_void_p(out.ctypes.data))
    return out


def gather(E, tok):
    E, pe = _u16(E)
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    B, K = tok.shape[0], E.shape[1]
    out = np.empty((B, K), dtype=np.uint16)
    _load().orc_gather(pe, ctypes.c_void_p(tok.ctypes.data), _i64(B), _i64(K), ctypes.c_void_p(out.ctypes.data))
    return out


def gemm_rows(A, Bm, rows, threads=None):
    """C[rows, :] of C = A @ Bm.T (A [M,K], Bm [N,K])."""
    A, pa = _u16(A)
    Bm, pb = _u16(Bm)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    N, K = Bm.shape
    out = np.empty((rows.size, N), dtype=np.float64)
    _load().orc_gemm_rows(pa, pb, _i64(N), _i64(K), ctypes.c_void_p(rows.ctypes.data), _i64(rows.size),
                          ctypes.c_void_p(out.ctypes.data), threads or default_threads())
    return out


def gemm_cols(A, Bm, cols, threads=None):
    """C[:, cols].T of C = A @ Bm.T, shape [len(cols), M]."""
    A, pa = _u16(A)
    Bm, pb = _u16(Bm)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    M, K = A.shape
    out = np.empty((cols.size, M), dtype=np.float64)
    _load().orc_gemm_cols(pa, pb, _i64(M), _i64(K), ctypes.c_void_p(cols.ctypes.data), _i64(cols.size),
                          ctypes.c_void_p(out.ctypes.data), threads or default_threads())
    return out


def decode_step(w, tok, shp, eps=1e-6, want_logits=False, threads=None):
    """One step of the chain; returns dict of bf16 intermediates, logits (opt), next tokens, margins."""
    B = len(tok)
    D, Nq, F, V = shp.D, shp.Nqkv, shp.F, shp.V
    tok = np.ascontiguousarray(tok, dtype=np.int32)
    keep = {k: np.ascontiguousarray(w[k], dtype=np.uint16) for k in ("E", "gamma", "Wqkv", "Wo", "Wgu", "Wd", "Wlm")}
    assert keep["E"].shape == (V, D) and keep["Wqkv"].shape == (Nq, D) and keep["Wgu"].shape == (2 * F, D)
    assert keep["Wd"].shape == (D, F) and keep["Wlm"].shape == (V, D) and keep["Wo"].shape == (D, D)
    o = {
        "h0": np.empty((B, D), np.uint16), "n": np.empty((B, D), np.uint16),
        "qkv": np.empty((B, Nq), np.uint16), "o": np.empty((B, D), np.uint16),
        "act": np.empty((B, F), np.uint16), "d": np.empty((B, D), np.uint16),
    }
    logits = np.empty((B, V), np.float64) if want_logits else None
    nxt = np.empty(B, np.int32)
    margin = np.empty(B, np.float64)
    P = lambda a: ctypes.c_void_p(a.ctypes.data)
    _load().orc_decode_step(P(keep["E"]), P(keep["gamma"]), P(keep["Wqkv"]), P(keep["Wo"]), P(keep["Wgu"]),
                            P(keep["Wd"]), P(keep["Wlm"]), P(tok), _i64(B), _i64(D), _i64(Nq), _i64(F), _i64(V),
                            ctypes.c_double(eps), P(o["h0"]), P(o["n"]), P(o["qkv"]), P(o["o"]), P(o["act"]),
                            P(o["d"]), P(logits) if want_logits else None, P(nxt), P(margin),
                            threads or default_threads())
    o["logits"], o["next"], o["margin"] = logits, nxt, margin
    return o
