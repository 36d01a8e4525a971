"""Harness around the C ABI: device buffers (torch, plumbing only), the decode
chain as a list of immutable descriptors, bit-level comparison helpers.

Nothing here computes any part of the method: tensors are moved, descriptors are
built and submitted, outputs are compared.
"""
import numpy as np
import torch

from . import inputs, vte

WIDTHS = (32, 64, 128, 256)


def to_dev(bits_or_array):
    """numpy uint16 (bf16 bits) / int32 / float32 -> torch tensor on cuda:0 (same bits)."""
    a = np.ascontiguousarray(bits_or_array)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def dev_empty(shape, dtype=torch.int16):
    return torch.empty(shape, dtype=dtype, device="cuda")


def dev_zeros_bytes(nbytes):
    return torch.zeros((nbytes + 3) // 4, dtype=torch.int32, device="cuda")


def to_bits(t):
    """torch int16 tensor -> numpy uint16 bit patterns."""
    return t.detach().cpu().numpy().view(np.uint16)


def mismatched_bits(a, b):
    """(elements that differ, bits that differ) between two same-shape raw arrays."""
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    ua = a.view(np.uint16 if a.dtype.itemsize == 2 else np.uint32)
    ub = b.view(ua.dtype)
    x = ua ^ ub
    nbits = int(np.unpackbits(x.view(np.uint8)).sum())
    return int(np.count_nonzero(x)), nbits


def make_ctx(mode=vte.VTE_MODE_PIPELINED, lookahead=32, device=0):
    cfg = vte.vte_pool_cfg_default()
    cfg.mode = mode
    cfg.lookahead = lookahead
    torch.cuda.init()
    torch.zeros(1, device="cuda")  # make sure the primary context exists before streams are created
    return vte.vte_init(device, cfg)


def pctx_of_width(ctx, width, index=0):
    """First pCtx of this width: a tree node if there is one, else a remainder."""
    try:
        return vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, width, index)
    except vte.VteError:
        return vte.vte_pool_find(ctx, vte.VTE_PCTX_REMAINDER, width, index)


def run_on(ctx, desc, pctx_id):
    tok = vte.vte_bind_and_launch(ctx, desc, pctx_id)
    vte.vte_token_wait(ctx, tok)


class DecodeChain:
    """The Llama-shaped single-layer decode chain as immutable descriptors:
    gather, RMSNorm, QKV, O (on the Q slice of QKV), gate/up+SiLU, down, LM head, argmax finish
    (eight launches; seven with fused_gather).  splitk=S builds the reshaped variant of every
    GEMV instead (the negative control).  fused_argmax adds the step-boundary descriptor that
    finishes the previous step's token, gathers and normalises in one launch: a burst is then
    first step (7 launches, no finish) + later steps (6 launches each) + one finish at the end.
    fused_qkv (with fused_argmax; hidden size 4096, batch <= 16) folds that boundary into the QKV launch:
    5 launches per step.  With want_logits the fused launch also stores the gathered and the normalised
    rows, so that snapshot() shows the same buffers as the other forms."""

    def __init__(self, ctx, weights_dev, shp, B, eps=1e-6, want_logits=False, splitk=None, rms_active_cus=None,
                 feedback=False, fused_gather=False, fused_argmax=False, fixed_split=True, fused_qkv=False):
        self.ctx, self.shp, self.B = ctx, shp, B
        D, Nq, F, V = shp.D, shp.Nqkv, shp.F, shp.V
        w = self.w = weights_dev
        self.tok = torch.zeros(B, dtype=torch.int32, device="cuda")
        self.h0, self.n = dev_empty((B, D)), dev_empty((B, D))
        self.qkv, self.o = dev_empty((B, Nq)), dev_empty((B, D))
        self.act, self.d = dev_empty((B, F)), dev_empty((B, D))
        # feedback: the LM head writes the token buffer the next step's gather reads (free-running decode)
        self.next = self.tok if feedback else torch.zeros(B, dtype=torch.int32, device="cuda")
        self.logits = torch.zeros((B, V), dtype=torch.float32, device="cuda") if want_logits else None
        self.ws = dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, D))
        self.extra = []
        d = self.desc = {}
        if fused_gather:  # gather folded into the norm launch (h0 still written, for inspection)
            d["rmsnorm"] = vte.vte_desc_rmsnorm_gather(ctx, w["E"], self.tok, w["gamma"], self.n, self.h0, B, V, D, eps)
        else:
            d["gather"] = vte.vte_desc_gather(ctx, w["E"], self.tok, self.h0, B, V, D)
        if fused_gather:
            pass
        elif rms_active_cus is None:
            d["rmsnorm"] = vte.vte_desc_rmsnorm(ctx, self.h0, w["gamma"], self.n, B, D, eps)
        else:
            d["rmsnorm"] = vte.vte_desc_rmsnorm_reshaped(ctx, self.h0, w["gamma"], self.n, B, D, eps, rms_active_cus)
        self.alg_bytes = {}  # algorithmic bytes of the projections that run as a split + finish pair
        if splitk is None:
            def proj(name, W, X, ldx, Y, N, K, epi=vte.VTE_EPI_NONE):
                """One projection: a single launch, or where the shape asks for it (narrow output, batch
                above 32) the shape-derived K split and its finish launch."""
                S = vte.vte_gemv_fixed_split(B, N, K, epi) if fixed_split else 1
                if S > 1:
                    ws = dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S))
                    self.extra.append(ws)
                    d[name] = vte.vte_desc_gemv_split(ctx, W, X, ldx, ws, B, N, K, epi, S)
                    d[name + "_fin"] = vte.vte_desc_gemv_split_finish(ctx, d[name], Y)
                    n_out = N // 2 if epi == vte.VTE_EPI_SILU_MUL else N
                    self.alg_bytes[name] = 2 * N * K + 2 * B * K + 2 * B * n_out
                    self.alg_bytes[name + "_fin"] = 0
                elif ldx != K:
                    d[name] = vte.vte_desc_gemv_strided(ctx, W, X, ldx, Y, N, B, N, K, epi)
                else:
                    d[name] = vte.vte_desc_gemv(ctx, W, X, Y, B, N, K, epi)
            proj("qkv", w["Wqkv"], self.n, D, self.qkv, Nq, D)
            # the O projection consumes the Q slice (first D columns) of qkv in place
            proj("o", w["Wo"], self.qkv, Nq, self.o, D, D)
            proj("gateup", w["Wgu"], self.o, D, self.act, 2 * F, D, vte.VTE_EPI_SILU_MUL)
            proj("down", w["Wd"], self.act, F, self.d, D, F)
            d["lmhead"] = vte.vte_desc_lmhead_argmax(ctx, w["Wlm"], self.d, self.next, self.logits, self.ws, B, V, D)
        else:
            S = splitk
            self.q = dev_empty((B, D))

            def ws(n):
                t = dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, n, S))
                self.extra.append(t)
                return t
            d["qkv"] = vte.vte_desc_gemv_splitk(ctx, w["Wqkv"], self.n, self.qkv, ws(Nq), B, Nq, D, 0, S)
            # split-K has no strided form: Q is the first D rows of Wqkv applied again, into its own buffer
            d["q"] = vte.vte_desc_gemv_splitk(ctx, w["Wqkv"], self.n, self.q, ws(D), B, D, D, 0, S)
            d["o"] = vte.vte_desc_gemv_splitk(ctx, w["Wo"], self.q, self.o, ws(D), B, D, D, 0, S)
            d["gateup"] = vte.vte_desc_gemv_splitk(ctx, w["Wgu"], self.o, self.act, ws(2 * F), B, 2 * F, D,
                                                   vte.VTE_EPI_SILU_MUL, S)
            d["down"] = vte.vte_desc_gemv_splitk(ctx, w["Wd"], self.act, self.d, ws(D), B, D, F, 0, S)
            d["lmhead"] = vte.vte_desc_lmhead_argmax_splitk(ctx, w["Wlm"], self.d, self.next, self.logits, self.ws,
                                                            ws(V), B, V, D, S)
        d["argmax"] = vte.vte_desc_argmax_finish(ctx, d["lmhead"])
        self.order = [k for k in ("gather", "rmsnorm", "qkv", "qkv_fin", "q", "o", "o_fin", "gateup", "gateup_fin", "down", "down_fin",
                                  "lmhead", "argmax") if k in d]
        self.fused_argmax = fused_argmax
        if fused_argmax:
            d["boundary"] = vte.vte_desc_rmsnorm_gather_argmax(ctx, w["E"], d["lmhead"], self.next, w["gamma"], self.n,
                                                               self.h0, V, D, eps)
            body = [k for k in self.order if k not in ("gather", "rmsnorm", "argmax")]
            self.order_first = [k for k in self.order if k != "argmax"]
            self.order_next = ["boundary"] + body
            if fused_qkv:
                keep = (self.h0, self.n) if want_logits else (None, None)
                d["qkv_first"] = vte.vte_desc_gemv_rmsnorm_gather(ctx, w["Wqkv"], w["E"], self.tok, w["gamma"], self.qkv,
                                                                  keep[0], keep[1], B, V, Nq, D, eps)
                d["qkv_next"] = vte.vte_desc_gemv_rmsnorm_gather_argmax(ctx, w["Wqkv"], w["E"], d["lmhead"], self.next,
                                                                        w["gamma"], self.qkv, keep[0], keep[1], V, Nq, D, eps)
                rest = [k for k in body if k not in ("qkv", "qkv_fin")]
                self.order_first = ["qkv_first"] + rest
                self.order_next = ["qkv_next"] + rest
            self.bytes_per_step = sum(self.alg_bytes.get(k, vte.vte_desc_info(d[k]).bytes) for k in self.order_next if k != "q")
        else:
            self.bytes_per_step = sum(self.alg_bytes.get(k, vte.vte_desc_info(d[k]).bytes) for k in self.order if k != "q")

    def set_tokens(self, toks):
        self.tok.copy_(torch.from_numpy(np.ascontiguousarray(toks, dtype=np.int32)))
        torch.cuda.synchronize()

    def submit_step(self, vs):
        """Submits one step (8 launches) to a vstream; returns the last token."""
        last = 0
        for k in self.order:
            last = vte.vte_submit(vs, self.desc[k])
        return last

    def submit_burst(self, vs, steps):
        """Submits `steps` free-running steps; with fused_argmax the step boundary is one launch
        and the last token is finished by one extra launch at the end.  Returns the last token."""
        last = 0
        if not self.fused_argmax:
            for _ in range(steps):
                last = self.submit_step(vs)
            return last
        # handed over as batches (one call per 32 steps): a Python loop of single submissions takes 5 us per
        # launch, longer than the boundary launch runs, and starves the first step of a burst
        if steps > 0:
            vte.vte_submit_batch(vs, self._batch(0))
        rest = steps - 1
        while rest > 0:
            n = min(rest, 32)
            vte.vte_submit_batch(vs, self._batch(n))
            rest -= n
        return vte.vte_submit(vs, self.desc["argmax"])

    def _batch(self, n):
        """desc_array of a burst's first step (n = 0) or of n later steps, built once."""
        cache = self.__dict__.setdefault("_batches", {})
        if n not in cache:
            ks = self.order_first if n == 0 else self.order_next * n
            cache[n] = vte.desc_array([self.desc[k] for k in ks])
        return cache[n]

    def run_step_on(self, pctx_ids):
        """One step with every launch bound explicitly: pctx_ids is an id or one id per launch."""
        if isinstance(pctx_ids, int):
            pctx_ids = [pctx_ids] * len(self.order)
        for k, p in zip(self.order, pctx_ids):
            run_on(self.ctx, self.desc[k], p)

    def advance(self):
        """tok <- next (device copy on torch's stream, ordered by the caller's syncs)."""
        self.tok.copy_(self.next)
        torch.cuda.synchronize()

    def snapshot(self):
        torch.cuda.synchronize()
        out = {k: to_bits(getattr(self, k)) for k in ("h0", "n", "qkv", "o", "act", "d")}
        out["next"] = self.next.cpu().numpy().copy()
        if self.logits is not None:
            out["logits"] = self.logits.cpu().numpy().copy()
        return out

    def close(self):
        for dd in self.desc.values():
            vte.vte_desc_destroy(dd)
        self.desc = {}


class LayeredDecode:
    """L copies of the decode layer (RMSNorm, QKV, O on the Q slice, gate/up+SiLU, down), each with its
    own weights, between one embedding gather and one LM head + greedy token that feeds back into the
    token buffer: 5L + 2 launches per step.  Every batch is built at a fixed batch size B, so a row's
    result does not depend on which other rows share the launch.  Activation buffers are per instance,
    weights are shared between instances."""

    def __init__(self, ctx, layers_dev, head_dev, shp, B, eps=1e-6):
        self.ctx, self.shp, self.B, self.L = ctx, shp, B, len(layers_dev)
        D, Nq, F, V = shp.D, shp.Nqkv, shp.F, shp.V
        self.tok = torch.zeros(B, dtype=torch.int32, device="cuda")
        self.n, self.qkv, self.o = dev_empty((B, D)), dev_empty((B, Nq)), dev_empty((B, D))
        self.act, self.d = dev_empty((B, F)), dev_empty((B, D))
        self.ws = dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, D))
        ds = self.descs = []
        for l, w in enumerate(layers_dev):
            if l == 0:
                ds.append(vte.vte_desc_rmsnorm_gather(ctx, head_dev["E"], self.tok, w["gamma"], self.n, None, B, V, D, eps))
            else:
                ds.append(vte.vte_desc_rmsnorm(ctx, self.d, w["gamma"], self.n, B, D, eps))
            ds.append(vte.vte_desc_gemv(ctx, w["Wqkv"], self.n, self.qkv, B, Nq, D))
            ds.append(vte.vte_desc_gemv_strided(ctx, w["Wo"], self.qkv, Nq, self.o, D, B, D, D))
            ds.append(vte.vte_desc_gemv(ctx, w["Wgu"], self.o, self.act, B, 2 * F, D, vte.VTE_EPI_SILU_MUL))
            ds.append(vte.vte_desc_gemv(ctx, w["Wd"], self.act, self.d, B, D, F))
        lm = vte.vte_desc_lmhead_argmax(ctx, head_dev["Wlm"], self.d, self.tok, None, self.ws, B, V, D)
        ds.append(lm)
        ds.append(vte.vte_desc_argmax_finish(ctx, lm))
        self.step = vte.desc_array(ds)
        self.ops_per_step = len(ds)
        self.bytes_per_step = sum(vte.vte_desc_info(d).bytes for d in ds)

    def distinct_descs(self):
        """One descriptor per distinct profile key (kernel and shape), in chain order."""
        seen, out = set(), []
        for d in self.descs:
            k = vte.vte_desc_info(d).profile_key
            if k not in seen:
                seen.add(k)
                out.append(d)
        return out

    def submit_step(self, vs):
        return vte.vte_submit_batch(vs, self.step)

    def close(self):
        for d in self.descs:
            vte.vte_desc_destroy(d)
        self.descs = []


def upload_weights(weights_np):
    return {k: to_dev(v) for k, v in weights_np.items()}
