"""ctypes binding of libvte.so: one Python function per C entry point of
include/vte.h, same names, argument marshalling only.  Device buffers are torch
CUDA tensors (or raw integer addresses); every step of the path runs in the
library's kernels.  There is no fallback: if the library is missing, loading
raises.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvte.so")

VTE_OK, VTE_EINVAL, VTE_ENOMEM, VTE_EHIP, VTE_EBUSY, VTE_ENOTREADY, VTE_EINCOMPAT, VTE_ESTATE, VTE_ETIMEOUT = \
    0, -1, -2, -3, -4, -5, -6, -7, -8
VTE_BACKEND_HIP, VTE_BACKEND_FAKE = 0, 1
VTE_MODE_STRICT, VTE_MODE_PIPELINED = 0, 1
VTE_LAYOUT_STRIPED = 0
VTE_REMAINDERS_NONE, VTE_REMAINDERS_ALL, VTE_REMAINDERS_PER_LEVEL = 0, 1, 2
VTE_PCTX_NODE, VTE_PCTX_REMAINDER = 0, 1
VTE_PCTX_IDLE, VTE_PCTX_LEASED, VTE_PCTX_DRAINING, VTE_PCTX_RESERVED = 0, 1, 2, 3
VTE_EPI_NONE, VTE_EPI_SILU_MUL = 0, 1
VTE_CLASS_LATENCY, VTE_CLASS_BEST_EFFORT = 0, 1
VTE_POLICY_WIDEST, VTE_POLICY_QUEUE_STATE, VTE_POLICY_TPUT_PLAN, VTE_POLICY_TPOT_FIRST = 0, 1, 2, 3
VTE_GEMV_DOT2, VTE_GEMV_MFMA, VTE_GEMV_MFMA_ROWS = 0, 1, 2
(VTE_K_RMSNORM, VTE_K_LAYERNORM, VTE_K_GEMV, VTE_K_LMHEAD, VTE_K_GATHER, VTE_K_GEMM, VTE_K_GEMV_SPLITK,
 VTE_K_LMHEAD_SPLITK, VTE_K_RMSNORM_RESHAPED, VTE_K_ARGMAX_FINISH, VTE_K_RMSNORM_GATHER,
 VTE_K_RMSNORM_GATHER_ARGMAX, VTE_K_MEMCPY, VTE_K_MEMSET, VTE_K_SOFTMAX_PROB, VTE_K_GEMV_SPLIT,
 VTE_K_GEMV_SPLIT_FINISH, VTE_K_GEMV_NORM) = range(1, 19)


class VteError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("vte error %d: %s" % (code, msg))
        self.code = code


class vte_pool_cfg(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("backend", "total_cus", "leaf_cus", "layout", "with_remainders", "mode",
                                        "lookahead", "stats_capacity")] + [("device_timing_mask", C.c_uint),
                                                                           ("dispatch_pipes", C.c_int),
                                                                          ("device_timing_stride", C.c_int)]


class vte_pctx_info(C.Structure):
    _fields_ = [("id", C.c_int), ("kind", C.c_int), ("width", C.c_int), ("level", C.c_int), ("parent", C.c_int),
                ("child", C.c_int * 2), ("remainder", C.c_int), ("state", C.c_int), ("gate_open", C.c_int),
                ("outstanding", C.c_int), ("reserved_for", C.c_int), ("mask", C.c_uint32 * 8), ("pipe", C.c_int)]


class vte_desc_view(C.Structure):
    _fields_ = [("kernel", C.c_int), ("grid", C.c_uint32 * 3), ("block", C.c_uint32 * 3), ("lds_bytes", C.c_uint32),
                ("arg_bytes", C.c_uint32), ("hash", C.c_uint64), ("profile_key", C.c_uint64), ("bytes", C.c_uint64),
                ("flops", C.c_uint64)]


class vte_gemv_plan(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("batch_tile", "rows", "ksteps", "prefetch", "max_waves", "groups", "kind")]


class vte_ready_op(C.Structure):
    _fields_ = [("token", C.c_uint64), ("vstream", C.c_int), ("klass", C.c_int), ("pinned_pctx", C.c_int),
                ("age", C.c_uint64), ("pred_pctx", C.c_int), ("desc", vte_desc_view)]


class vte_pool_view(C.Structure):
    _fields_ = [("count", C.c_int), ("pctx", C.POINTER(vte_pctx_info)), ("ready_by_class", C.c_int * 2),
                ("inflight_by_class", C.c_int * 2)]


class vte_hint(C.Structure):
    _fields_ = [("vstream", C.c_int), ("want_width", C.c_int), ("ready_in_s", C.c_double), ("deadline_in_s", C.c_double)]


class vte_prepare_plan(C.Structure):
    _fields_ = [("target_pctx", C.c_int), ("reserve", C.c_int), ("n_close", C.c_int), ("close", C.c_int * 32)]


PICK_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.POINTER(vte_ready_op), C.c_int, C.POINTER(vte_pool_view))
SELECT_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.POINTER(vte_ready_op), C.POINTER(C.c_int), C.c_int,
                        C.POINTER(vte_pool_view))
PREPARE_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.POINTER(vte_hint), C.POINTER(vte_pool_view),
                         C.POINTER(vte_prepare_plan))


class vte_policy_vtbl(C.Structure):
    _fields_ = [("pick", PICK_FN), ("select", SELECT_FN), ("prepare", PREPARE_FN)]


class vte_op_record(C.Structure):
    _fields_ = [("token", C.c_uint64), ("vstream", C.c_int), ("klass", C.c_int), ("kernel", C.c_int),
                ("pctx", C.c_int), ("width", C.c_int), ("t_submit", C.c_double), ("t_ready", C.c_double),
                ("t_bound", C.c_double), ("t_done", C.c_double), ("gpu_seconds", C.c_double),
                ("gpu_begin", C.c_double), ("gpu_end", C.c_double)]


class vte_stats_t(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("submitted", "completed", "leases_opened", "leases_reused",
                                           "lease_conflicts", "stale_proposals", "submit_failures", "gates_closed",
                                           "reservations", "completion_records", "failed")]


class vte_tpot_info(C.Structure):
    _fields_ = [("tpot_seconds", C.c_double), ("ops_per_token", C.c_int), ("standing_pctx", C.c_int),
                ("escalated_pctx", C.c_int), ("at_risk", C.c_int), ("tokens_done", C.c_uint64),
                ("deadline_misses", C.c_uint64), ("escalations", C.c_uint64)]


class vte_fake_log_entry(C.Structure):
    _fields_ = [("token", C.c_uint64), ("pctx", C.c_int), ("desc_hash", C.c_uint64), ("waited_on_pctx", C.c_int)]


# every symbol include/vte.h declares
EXPORTS = [
    "vte_last_error", "vte_last_hip_error", "vte_pool_cfg_default", "vte_init", "vte_shutdown", "vte_pool_count",
    "vte_pool_info", "vte_pool_find", "vte_pool_conflict", "vte_pctx_native_stream", "vte_desc_rmsnorm",
    "vte_desc_rmsnorm_gather", "vte_desc_rmsnorm_gather_argmax",
    "vte_desc_layernorm", "vte_desc_gemv", "vte_lmhead_workspace_bytes", "vte_desc_lmhead_argmax", "vte_desc_argmax_finish",
    "vte_desc_gemv_strided", "vte_gemv_default_plan", "vte_desc_gemv_planned", "vte_desc_lmhead_argmax_planned", "vte_desc_gather",
    "vte_desc_gemm", "vte_splitk_workspace_bytes", "vte_desc_gemv_splitk", "vte_desc_lmhead_argmax_splitk",
    "vte_desc_rmsnorm_reshaped", "vte_desc_info", "vte_desc_args", "vte_desc_destroy", "vte_bind_and_launch",
    "vte_vstream_create", "vte_vstream_destroy", "vte_vstream_id", "vte_vstream_pin", "vte_submit",
    "vte_submit_after", "vte_token_query", "vte_token_wait", "vte_vstream_sync", "vte_device_sync",
    "vte_pctx_close_gate", "vte_pctx_reserve", "vte_pctx_unreserve", "vte_set_policy", "vte_set_builtin_policy",
    "vte_hint_submit", "vte_profile_measure", "vte_profile_measure_on", "vte_profile_set", "vte_profile_get", "vte_stats", "vte_stats_read",
    "vte_stats_reset", "vte_fake_complete", "vte_fake_set_autocomplete", "vte_fake_fail_next_submits",
    "vte_fake_log", "vte_dispatcher_quiesce", "vte_now", "vte_vstream_set_tpot", "vte_vstream_tpot_info", "vte_submit_batch", "vte_pool_creation_order", "vte_desc_memcpy", "vte_desc_memset32",
    "vte_event_record", "vte_vstream_wait_event", "vte_desc_softmax_prob",
    "vte_static_scratch_bytes", "vte_lmhead_argmax_static", "vte_fake_complete_error",
    "vte_gemv_fixed_split", "vte_desc_gemv_split", "vte_desc_gemv_split_finish", "vte_set_device_timing",
    "vte_desc_gemv_rmsnorm_gather", "vte_desc_gemv_rmsnorm_gather_argmax",
]

_lib = None


def load():
    """Loads libvte.so.  Raises if it has not been built: there is no other path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s not found: run `python -m paper_2603_15042_amd.build` first" % LIB_PATH)
        # torch ships its own HIP runtime: it has to be in the process first, so that the
        # library binds to that copy and both see the same device state
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(L, name).restype = C.c_int
        L.vte_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != VTE_OK:
        raise VteError(rc, load().vte_last_error().decode())
    return rc


def _ptr(t):
    """torch tensor / int / None -> void*"""
    if t is None:
        return C.c_void_p(None)
    if isinstance(t, int):
        return C.c_void_p(t)
    if hasattr(t, "data_ptr"):
        return C.c_void_p(t.data_ptr())
    raise TypeError("expected a tensor or an address")


def vte_last_error():
    return load().vte_last_error().decode()


def vte_last_hip_error():
    return load().vte_last_hip_error()


def vte_pool_cfg_default():
    cfg = vte_pool_cfg()
    _check(load().vte_pool_cfg_default(C.byref(cfg)))
    return cfg


def vte_init(device=0, cfg=None):
    ctx = C.c_void_p()
    _check(load().vte_init(C.byref(ctx), int(device), C.byref(cfg) if cfg is not None else None))
    return ctx


def vte_shutdown(ctx):
    _check(load().vte_shutdown(ctx))


def vte_pool_count(ctx):
    n = C.c_int()
    _check(load().vte_pool_count(ctx, C.byref(n)))
    return n.value


def vte_pool_info(ctx, pctx_id):
    info = vte_pctx_info()
    _check(load().vte_pool_info(ctx, int(pctx_id), C.byref(info)))
    return info


def vte_pool_creation_order(ctx):
    arr = (C.c_int * 64)()
    n = C.c_int()
    _check(load().vte_pool_creation_order(ctx, arr, 64, C.byref(n)))
    return [arr[i] for i in range(min(n.value, 64))]


def vte_pool_find(ctx, kind, width, index=0):
    out = C.c_int()
    _check(load().vte_pool_find(ctx, int(kind), int(width), int(index), C.byref(out)))
    return out.value


def vte_pool_conflict(ctx, a, b):
    out = C.c_int()
    _check(load().vte_pool_conflict(ctx, int(a), int(b), C.byref(out)))
    return bool(out.value)


def vte_pctx_native_stream(ctx, pctx_id):
    s = C.c_void_p()
    _check(load().vte_pctx_native_stream(ctx, int(pctx_id), C.byref(s)))
    return s.value


def _desc_call(fn, *args):
    d = C.c_void_p()
    _check(fn(*args, C.byref(d)))
    return d


def vte_desc_rmsnorm(ctx, x, gamma, y, rows, cols, eps):
    return _desc_call(load().vte_desc_rmsnorm, ctx, _ptr(x), _ptr(gamma), _ptr(y), int(rows), int(cols), C.c_float(eps))


def vte_desc_rmsnorm_gather(ctx, E, tok, gamma, y, h_or_null, B, V, cols, eps):
    return _desc_call(load().vte_desc_rmsnorm_gather, ctx, _ptr(E), _ptr(tok), _ptr(gamma), _ptr(y), _ptr(h_or_null),
                      int(B), int(V), int(cols), C.c_float(eps))


def vte_desc_rmsnorm_gather_argmax(ctx, E, lmhead, tok_out_or_null, gamma, y, h_or_null, V, cols, eps):
    return _desc_call(load().vte_desc_rmsnorm_gather_argmax, ctx, _ptr(E), lmhead, _ptr(tok_out_or_null), _ptr(gamma),
                      _ptr(y), _ptr(h_or_null), int(V), int(cols), C.c_float(eps))


def vte_desc_gemv_rmsnorm_gather(ctx, W, E, tok, gamma, Y, h_or_null, n_or_null, B, V, N, K, eps):
    return _desc_call(load().vte_desc_gemv_rmsnorm_gather, ctx, _ptr(W), _ptr(E), _ptr(tok), _ptr(gamma), _ptr(Y),
                      _ptr(h_or_null), _ptr(n_or_null), int(B), int(V), int(N), int(K), C.c_float(eps))


def vte_desc_gemv_rmsnorm_gather_argmax(ctx, W, E, lmhead, tok_out_or_null, gamma, Y, h_or_null, n_or_null, V, N, K, eps):
    return _desc_call(load().vte_desc_gemv_rmsnorm_gather_argmax, ctx, _ptr(W), _ptr(E), lmhead, _ptr(tok_out_or_null),
                      _ptr(gamma), _ptr(Y), _ptr(h_or_null), _ptr(n_or_null), int(V), int(N), int(K), C.c_float(eps))


def vte_desc_layernorm(ctx, x, gamma, beta, y, rows, cols, eps):
    return _desc_call(load().vte_desc_layernorm, ctx, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), int(rows), int(cols),
                      C.c_float(eps))


def vte_desc_rmsnorm_reshaped(ctx, x, gamma, y, rows, cols, eps, active_cus):
    return _desc_call(load().vte_desc_rmsnorm_reshaped, ctx, _ptr(x), _ptr(gamma), _ptr(y), int(rows), int(cols),
                      C.c_float(eps), int(active_cus))


def vte_gemv_default_plan(B, N, K, epilogue=VTE_EPI_NONE, S=1):
    p = vte_gemv_plan()
    _check(load().vte_gemv_default_plan(int(B), int(N), int(K), int(epilogue), int(S), C.byref(p)))
    return p


def vte_desc_gemv(ctx, W, X, Y, B, N, K, epilogue=VTE_EPI_NONE):
    return _desc_call(load().vte_desc_gemv, ctx, _ptr(W), _ptr(X), _ptr(Y), int(B), int(N), int(K), int(epilogue))


def vte_desc_gemv_strided(ctx, W, X, ldx, Y, ldy, B, N, K, epilogue=VTE_EPI_NONE):
    return _desc_call(load().vte_desc_gemv_strided, ctx, _ptr(W), _ptr(X), int(ldx), _ptr(Y), int(ldy), int(B), int(N),
                      int(K), int(epilogue))


def vte_desc_gemv_planned(ctx, W, X, Y, B, N, K, epilogue, plan):
    return _desc_call(load().vte_desc_gemv_planned, ctx, _ptr(W), _ptr(X), _ptr(Y), int(B), int(N), int(K),
                      int(epilogue), C.byref(plan))


def vte_splitk_workspace_bytes(B, N, S):
    n = C.c_size_t()
    _check(load().vte_splitk_workspace_bytes(int(B), int(N), int(S), C.byref(n)))
    return n.value


def vte_desc_gemv_splitk(ctx, W, X, Y, workspace, B, N, K, epilogue, S):
    return _desc_call(load().vte_desc_gemv_splitk, ctx, _ptr(W), _ptr(X), _ptr(Y), _ptr(workspace), int(B), int(N),
                      int(K), int(epilogue), int(S))


def vte_gemv_fixed_split(B, N, K, epilogue=VTE_EPI_NONE):
    S = C.c_int()
    _check(load().vte_gemv_fixed_split(int(B), int(N), int(K), int(epilogue), C.byref(S)))
    return S.value


def vte_desc_gemv_split(ctx, W, X, ldx, workspace, B, N, K, epilogue, S, plan=None):
    return _desc_call(load().vte_desc_gemv_split, ctx, _ptr(W), _ptr(X), int(ldx), _ptr(workspace), int(B), int(N), int(K),
                      int(epilogue), int(S), C.byref(plan) if plan is not None else None)


def vte_desc_gemv_split_finish(ctx, split_desc, Y, ldy=0):
    return _desc_call(load().vte_desc_gemv_split_finish, ctx, split_desc, _ptr(Y), int(ldy))


def vte_lmhead_workspace_bytes(B, V, K):
    n = C.c_size_t()
    _check(load().vte_lmhead_workspace_bytes(int(B), int(V), int(K), C.byref(n)))
    return n.value


def vte_desc_lmhead_argmax(ctx, W, H, tok, logits_or_null, workspace, B, V, K):
    return _desc_call(load().vte_desc_lmhead_argmax, ctx, _ptr(W), _ptr(H), _ptr(tok), _ptr(logits_or_null),
                      _ptr(workspace), int(B), int(V), int(K))


def vte_desc_argmax_finish(ctx, lmhead_desc):
    return _desc_call(load().vte_desc_argmax_finish, ctx, lmhead_desc)


def vte_desc_lmhead_argmax_planned(ctx, W, H, tok, logits_or_null, workspace, B, V, K, plan):
    return _desc_call(load().vte_desc_lmhead_argmax_planned, ctx, _ptr(W), _ptr(H), _ptr(tok), _ptr(logits_or_null),
                      _ptr(workspace), int(B), int(V), int(K), C.byref(plan))


def vte_desc_lmhead_argmax_splitk(ctx, W, H, tok, logits_or_null, workspace, partials, B, V, K, S):
    return _desc_call(load().vte_desc_lmhead_argmax_splitk, ctx, _ptr(W), _ptr(H), _ptr(tok), _ptr(logits_or_null),
                      _ptr(workspace), _ptr(partials), int(B), int(V), int(K), int(S))


def vte_desc_gather(ctx, E, tok, H, B, V, K):
    return _desc_call(load().vte_desc_gather, ctx, _ptr(E), _ptr(tok), _ptr(H), int(B), int(V), int(K))


def vte_desc_softmax_prob(ctx, logits, tok, prob, B, V):
    return _desc_call(load().vte_desc_softmax_prob, ctx, _ptr(logits), _ptr(tok), _ptr(prob), int(B), int(V))


def vte_desc_memcpy(ctx, dst, src, nbytes):
    return _desc_call(load().vte_desc_memcpy, ctx, _ptr(dst), _ptr(src), C.c_size_t(nbytes))


def vte_desc_memset32(ctx, dst, value, nbytes):
    return _desc_call(load().vte_desc_memset32, ctx, _ptr(dst), C.c_uint32(value), C.c_size_t(nbytes))


def vte_event_record(vs):
    tok = C.c_uint64()
    _check(load().vte_event_record(vs, C.byref(tok)))
    return tok.value


def vte_vstream_wait_event(vs, event):
    _check(load().vte_vstream_wait_event(vs, C.c_uint64(event)))


def vte_desc_gemm(ctx, A, Bm, Cm, M, N, K):
    return _desc_call(load().vte_desc_gemm, ctx, _ptr(A), _ptr(Bm), _ptr(Cm), int(M), int(N), int(K))


def vte_desc_info(desc):
    v = vte_desc_view()
    _check(load().vte_desc_info(desc, C.byref(v)))
    return v


def vte_desc_args(desc, cap=160):
    buf = C.create_string_buffer(cap)
    _check(load().vte_desc_args(desc, buf, C.c_size_t(cap)))
    return buf.raw[:vte_desc_info(desc).arg_bytes]


def vte_desc_destroy(desc):
    _check(load().vte_desc_destroy(desc))


def vte_bind_and_launch(ctx, desc, pctx_id):
    tok = C.c_uint64()
    _check(load().vte_bind_and_launch(ctx, desc, int(pctx_id), C.byref(tok)))
    return tok.value


def vte_vstream_create(ctx, klass=VTE_CLASS_LATENCY):
    vs = C.c_void_p()
    _check(load().vte_vstream_create(ctx, int(klass), C.byref(vs)))
    return vs


def vte_vstream_destroy(vs):
    _check(load().vte_vstream_destroy(vs))


def vte_vstream_id(vs):
    i = C.c_int()
    _check(load().vte_vstream_id(vs, C.byref(i)))
    return i.value


def vte_vstream_pin(vs, pctx_id):
    _check(load().vte_vstream_pin(vs, int(pctx_id)))


def vte_submit(vs, desc):
    tok = C.c_uint64()
    _check(load().vte_submit(vs, desc, C.byref(tok)))
    return tok.value


def desc_array(descs):
    """A C array of descriptor handles for vte_submit_batch (build once, submit many times)."""
    return (C.c_void_p * len(descs))(*[d if isinstance(d, int) else d.value for d in descs])


def vte_submit_batch(vs, arr):
    """arr: desc_array(...).  Returns the token of the last op."""
    tok = C.c_uint64()
    _check(load().vte_submit_batch(vs, arr, len(arr), C.byref(tok)))
    return tok.value


def vte_submit_after(vs, desc, deps):
    tok = C.c_uint64()
    arr = (C.c_uint64 * len(deps))(*deps)
    _check(load().vte_submit_after(vs, desc, arr, len(deps), C.byref(tok)))
    return tok.value


def vte_token_query(ctx, token):
    d = C.c_int()
    _check(load().vte_token_query(ctx, C.c_uint64(token), C.byref(d)))
    return bool(d.value)


def vte_token_wait(ctx, token):
    _check(load().vte_token_wait(ctx, C.c_uint64(token)))


def vte_vstream_sync(vs):
    _check(load().vte_vstream_sync(vs))


def vte_device_sync(ctx):
    _check(load().vte_device_sync(ctx))


def vte_pctx_close_gate(ctx, pctx_id):
    _check(load().vte_pctx_close_gate(ctx, int(pctx_id)))


def vte_pctx_reserve(ctx, pctx_id, vs):
    _check(load().vte_pctx_reserve(ctx, int(pctx_id), vs))


def vte_pctx_unreserve(ctx, pctx_id):
    _check(load().vte_pctx_unreserve(ctx, int(pctx_id)))


def vte_set_policy(ctx, vtbl, user=None):
    """vtbl: a vte_policy_vtbl the caller keeps alive (with its callbacks), or None."""
    _check(load().vte_set_policy(ctx, C.byref(vtbl) if vtbl is not None else None, user))


def vte_set_device_timing(ctx, mask, stride):
    _check(load().vte_set_device_timing(ctx, C.c_uint(mask), int(stride)))


def vte_set_builtin_policy(ctx, which, slack=0.1, keep_free_cus=0):
    _check(load().vte_set_builtin_policy(ctx, int(which), C.c_double(slack), int(keep_free_cus)))


def vte_vstream_set_tpot(vs, tpot_seconds, ops_per_token):
    _check(load().vte_vstream_set_tpot(vs, C.c_double(tpot_seconds), int(ops_per_token)))


def vte_vstream_tpot_info(vs):
    out = vte_tpot_info()
    _check(load().vte_vstream_tpot_info(vs, C.byref(out)))
    return out


def vte_hint_submit(ctx, hint):
    _check(load().vte_hint_submit(ctx, C.byref(hint)))


def vte_profile_measure(ctx, desc, warmup=3, reps=10):
    _check(load().vte_profile_measure(ctx, desc, int(warmup), int(reps)))


def vte_profile_measure_on(ctx, desc, pctx_id, warmup=3, reps=10):
    s = C.c_double()
    _check(load().vte_profile_measure_on(ctx, desc, int(pctx_id), int(warmup), int(reps), C.byref(s)))
    return s.value


def vte_profile_set(ctx, key, width, seconds):
    _check(load().vte_profile_set(ctx, C.c_uint64(key), int(width), C.c_double(seconds)))


def vte_profile_get(ctx, key, width):
    s = C.c_double()
    _check(load().vte_profile_get(ctx, C.c_uint64(key), int(width), C.byref(s)))
    return s.value


def vte_stats(ctx):
    s = vte_stats_t()
    _check(load().vte_stats(ctx, C.byref(s)))
    return s


def vte_stats_read(ctx, cap=65536):
    arr = (vte_op_record * cap)()
    n = C.c_int()
    _check(load().vte_stats_read(ctx, arr, cap, C.byref(n)))
    return [arr[i] for i in range(n.value)]


def vte_stats_reset(ctx):
    _check(load().vte_stats_reset(ctx))


def vte_fake_complete(ctx, token):
    _check(load().vte_fake_complete(ctx, C.c_uint64(token)))


def vte_fake_complete_error(ctx, token):
    _check(load().vte_fake_complete_error(ctx, C.c_uint64(token)))


def vte_fake_set_autocomplete(ctx, on):
    _check(load().vte_fake_set_autocomplete(ctx, int(on)))


def vte_fake_fail_next_submits(ctx, n):
    _check(load().vte_fake_fail_next_submits(ctx, int(n)))


def vte_fake_log(ctx, cap=4096):
    arr = (vte_fake_log_entry * cap)()
    n = C.c_int()
    _check(load().vte_fake_log(ctx, arr, cap, C.byref(n)))
    return [arr[i] for i in range(n.value)]


def vte_dispatcher_quiesce(ctx):
    _check(load().vte_dispatcher_quiesce(ctx))


def vte_now(ctx):
    s = C.c_double()
    _check(load().vte_now(ctx, C.byref(s)))
    return s.value


def vte_static_scratch_bytes():
    n = C.c_size_t()
    _check(load().vte_static_scratch_bytes(C.byref(n)))
    return n.value


def vte_lmhead_argmax_static(hip_stream, W, H, tok, logits_or_null, B, V, K):
    """hip_stream: a hipStream_t as an integer (0 / None = the null stream)."""
    _check(load().vte_lmhead_argmax_static(C.c_void_p(hip_stream or None), _ptr(W), _ptr(H), _ptr(tok),
                                           _ptr(logits_or_null), int(B), int(V), int(K)))
