"""The paper's experiments on this path, on one MI355X, through the C ABI.

    python -m paper_2603_15042_amd.experiments determinism [--trials 1000] [--replays 100]
    python -m paper_2603_15042_amd.experiments cotenancy   [--seconds 3] [--gap-ms 60]
    python -m paper_2603_15042_amd.experiments gemm | operators | overhead | ramp

determinism  Sec. 7.1 "Determinism Protocol" / Sec. 7.2: matched-input trials of a reduction
             (RMSNorm 8x1024) and a GEMV (4096x4096, batch 1/4/8) with only the physical
             allocation varied (random pCtx per trial, a GEMM co-tenant on the complement),
             against the reshaping treatment (threads per row / split-K derived from the CU
             count); the co-tenant's GEMM at a compute-bound and an HBM-bound shape; then one
             decode state replayed with both treatments.
cotenancy    the mixed training-inference setting (Sec. 7.3.2) in synthetic form: a stream of
             8192^3 bf16 GEMMs as best-effort tenant, bursts of 128 decode steps at batch 8 as
             latency tenant; solo, fixed 128/128 split, and late-bound with lookahead hints.
Prints one JSON object.  Plumbing only: every number comes from launches of the library's
descriptors.
"""
import argparse
import json
import sys
import time

import numpy as np
import torch

from . import harness as H
from . import inputs, vte


def _rand_pctx(rng, ctx):
    return int(rng.integers(0, vte.vte_pool_count(ctx)))


def _complement_launch(ctx, gemm_desc, pctx):
    """Starts the co-tenant GEMM on the widest pCtx that does not overlap `pctx` (if there is one)."""
    best, bw = -1, 0
    for i in range(vte.vte_pool_count(ctx)):
        if not vte.vte_pool_conflict(ctx, i, pctx):
            w = vte.vte_pool_info(ctx, i).width
            if w > bw:
                best, bw = i, w
    if best < 0:
        return None
    try:
        return vte.vte_bind_and_launch(ctx, gemm_desc, best)
    except vte.VteError:
        return None


ALL_SECTIONS = ("rmsnorm", "gemv", "gemv_wide", "gemm", "replay")


def determinism(trials, replays, seed0=0, sections=ALL_SECTIONS):
    ctx = H.make_ctx(vte.VTE_MODE_STRICT)
    rng = np.random.default_rng(seed0)
    out = {}
    M = 2048
    gA = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, M)))
    gB = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (M, M)))
    gC = H.dev_empty((M, M))
    gemm = vte.vte_desc_gemm(ctx, gA, gB, gC, M, M, M)
    p256 = H.pctx_of_width(ctx, 256)
    widths = (32, 64, 128, 256)

    # ---- operator 1: the reduction (RMSNorm 8 x 1024) -------------------------------------------
    print("determinism: RMSNorm 8x1024, %d trials" % trials, file=sys.stderr, flush=True)
    if "rmsnorm" not in sections:
        trials_rms = 0
    else:
        trials_rms = trials
    rows, cols = 8, 1024
    dx, dg, dy = H.dev_empty((rows, cols)), H.dev_empty((cols,)), H.dev_empty((rows, cols))
    fixed = vte.vte_desc_rmsnorm(ctx, dx, dg, dy, rows, cols, 1e-6)
    resh = {w: vte.vte_desc_rmsnorm_reshaped(ctx, dx, dg, dy, rows, cols, 1e-6, w) for w in widths}
    r = {"trials": trials_rms, "fixed_mismatched_bits": 0, "fixed_trials_with_mismatch": 0,
         "reshaped_mismatched_bits": 0, "reshaped_trials_with_mismatch": 0, "reshaped_max_abs_diff": 0.0}
    for t in range(trials_rms):
        x, g = inputs.rmsnorm_case(seed=seed0 + t, rows=rows, cols=cols)
        dx.copy_(H.to_dev(x)); dg.copy_(H.to_dev(g))
        torch.cuda.synchronize()
        H.run_on(ctx, fixed, p256)
        ref = H.to_bits(dy).copy()
        p = _rand_pctx(rng, ctx)
        co = _complement_launch(ctx, gemm, p)
        H.run_on(ctx, fixed, p)
        got = H.to_bits(dy).copy()
        if co:
            vte.vte_token_wait(ctx, co)
        e, b = H.mismatched_bits(ref, got)
        r["fixed_mismatched_bits"] += b
        r["fixed_trials_with_mismatch"] += int(b > 0)
        w = widths[int(rng.integers(0, 4))]
        H.run_on(ctx, resh[256], p256)
        ref_r = H.to_bits(dy).copy()
        H.run_on(ctx, resh[w], H.pctx_of_width(ctx, w))
        got_r = H.to_bits(dy).copy()
        e, b = H.mismatched_bits(ref_r, got_r)
        r["reshaped_mismatched_bits"] += b
        r["reshaped_trials_with_mismatch"] += int(b > 0)
        d = np.abs(inputs.bf16_to_f32(ref_r) - inputs.bf16_to_f32(got_r)).max()
        r["reshaped_max_abs_diff"] = max(r["reshaped_max_abs_diff"], float(d))
    if trials_rms:
        out["rmsnorm_8x1024"] = r

    # ---- operator 2: GEMV 4096 x 4096 (fp32 sums kept through the LM-head form) --------------------
    N = K = 4096
    W0 = inputs.normal_bf16(seed0, inputs.T_W, (N, K), 0.0, K ** -0.5)
    dW = H.to_dev(W0)
    for B in ((1, 4, 8) if "gemv" in sections else ()):
        print("determinism: GEMV 4096x4096 batch %d, %d trials" % (B, trials), file=sys.stderr, flush=True)
        dX, dY = H.dev_empty((B, K)), H.dev_empty((B, N))
        tok = torch.zeros(B, dtype=torch.int32, device="cuda")
        lg = torch.zeros((B, N), dtype=torch.float32, device="cuda")
        ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, N, K))
        fixed = vte.vte_desc_gemv(ctx, dW, dX, dY, B, N, K)
        fixed32 = vte.vte_desc_lmhead_argmax(ctx, dW, dX, tok, lg, ws, B, N, K)
        sk, sk32 = {}, {}
        for w in widths:
            S = w // 32
            sk[w] = vte.vte_desc_gemv_splitk(ctx, dW, dX, dY, H.dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S)),
                                             B, N, K, 0, S)
            sk32[w] = vte.vte_desc_lmhead_argmax_splitk(ctx, dW, dX, tok, lg, ws,
                                                        H.dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S)),
                                                        B, N, K, S)
        r = {"trials": trials, "fixed_mismatched_bits_bf16": 0, "fixed_mismatched_bits_fp32": 0,
             "reshaped_mismatched_bits_bf16": 0, "reshaped_mismatched_bits_fp32": 0,
             "reshaped_trials_with_mismatch_bf16": 0, "reshaped_trials_with_mismatch_fp32": 0,
             "reshaped_max_abs_diff_fp32": 0.0}
        for t in range(trials):
            X = inputs.normal_bf16(seed0 + t, inputs.T_XB, (B, K))
            dX.copy_(H.to_dev(X))
            torch.cuda.synchronize()
            H.run_on(ctx, fixed, p256); ref = H.to_bits(dY).copy()
            H.run_on(ctx, fixed32, p256); ref32 = lg.cpu().numpy().copy()
            p = _rand_pctx(rng, ctx)
            co = _complement_launch(ctx, gemm, p)
            H.run_on(ctx, fixed, p); got = H.to_bits(dY).copy()
            H.run_on(ctx, fixed32, p); got32 = lg.cpu().numpy().copy()
            if co:
                vte.vte_token_wait(ctx, co)
            r["fixed_mismatched_bits_bf16"] += H.mismatched_bits(ref, got)[1]
            r["fixed_mismatched_bits_fp32"] += H.mismatched_bits(ref32, got32)[1]
            w = widths[int(rng.integers(0, 4))]
            pw = H.pctx_of_width(ctx, w)
            H.run_on(ctx, sk[w], pw); got = H.to_bits(dY).copy()
            H.run_on(ctx, sk32[w], pw); got32 = lg.cpu().numpy().copy()
            b16, b32 = H.mismatched_bits(ref, got)[1], H.mismatched_bits(ref32, got32)[1]
            r["reshaped_mismatched_bits_bf16"] += b16
            r["reshaped_mismatched_bits_fp32"] += b32
            r["reshaped_trials_with_mismatch_bf16"] += int(b16 > 0)
            r["reshaped_trials_with_mismatch_fp32"] += int(b32 > 0)
            r["reshaped_max_abs_diff_fp32"] = max(r["reshaped_max_abs_diff_fp32"], float(np.abs(ref32 - got32).max()))
        out["gemv_4096x4096_B%d" % B] = r

    # ---- operator 2b: the wide batches (fixed structure only: there is no split-K baseline above batch 32) ----
    for B, Nw in (((32, 4096), (64, 4096), (64, 32064)) if "gemv_wide" in sections else ()):
        print("determinism: GEMV %dx4096 batch %d, %d trials" % (Nw, B, trials), file=sys.stderr, flush=True)
        dWw = dW if Nw == N else H.to_dev(inputs.normal_bf16(seed0 + 7, inputs.T_W, (Nw, K), 0.0, K ** -0.5))
        dX, dY = H.dev_empty((B, K)), H.dev_empty((B, Nw))
        tok = torch.zeros(B, dtype=torch.int32, device="cuda")
        lg = torch.zeros((B, Nw), dtype=torch.float32, device="cuda")
        ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, Nw, K))
        fixed = vte.vte_desc_gemv(ctx, dWw, dX, dY, B, Nw, K)
        fixed32 = vte.vte_desc_lmhead_argmax(ctx, dWw, dX, tok, lg, ws, B, Nw, K)
        plan = vte.vte_gemv_default_plan(B, Nw, K, 0, 1)
        r = {"trials": trials, "plan_kind": int(plan.kind), "plan_batch_tile": int(plan.batch_tile),
             "fixed_mismatched_bits_bf16": 0, "fixed_mismatched_bits_fp32": 0}
        for t in range(trials):
            X = inputs.normal_bf16(seed0 + t, inputs.T_XB, (B, K))
            dX.copy_(H.to_dev(X))
            torch.cuda.synchronize()
            H.run_on(ctx, fixed, p256); ref = H.to_bits(dY).copy()
            H.run_on(ctx, fixed32, p256); ref32 = lg.cpu().numpy().copy()
            p = _rand_pctx(rng, ctx)
            co = _complement_launch(ctx, gemm, p)
            H.run_on(ctx, fixed, p); got = H.to_bits(dY).copy()
            H.run_on(ctx, fixed32, p); got32 = lg.cpu().numpy().copy()
            if co:
                vte.vte_token_wait(ctx, co)
            r["fixed_mismatched_bits_bf16"] += H.mismatched_bits(ref, got)[1]
            r["fixed_mismatched_bits_fp32"] += H.mismatched_bits(ref32, got32)[1]
        out["gemv_%dx4096_B%d" % (Nw, B)] = r
        vte.vte_desc_destroy(fixed); vte.vte_desc_destroy(fixed32)

    # ---- operator 3: the co-tenant's own GEMM, at a compute-bound and at an HBM-bound shape -----------
    for (gm, gn, gk) in (((4096, 4096, 4096), (32768, 256, 8192)) if "gemm" in sections else ()):
        ntr = max(1, trials // 5)
        print("determinism: GEMM %dx%dx%d, %d trials" % (gm, gn, gk, ntr), file=sys.stderr, flush=True)
        tA = H.to_dev(inputs.normal_bf16(seed0, inputs.T_GEMM_A, (gm, gk)))
        tB = H.to_dev(inputs.normal_bf16(seed0, inputs.T_GEMM_B, (gn, gk)))
        tC = H.dev_empty((gm, gn))
        dg_ = vte.vte_desc_gemm(ctx, tA, tB, tC, gm, gn, gk)
        H.run_on(ctx, dg_, p256)
        ref = H.to_bits(tC).copy()
        r = {"trials": ntr, "fixed_mismatched_bits": 0, "fixed_trials_with_mismatch": 0}
        for t in range(ntr):
            p = _rand_pctx(rng, ctx)
            co = _complement_launch(ctx, gemm, p)
            tC.fill_(0x7FC1)
            H.run_on(ctx, dg_, p)
            got = H.to_bits(tC)
            if co:
                vte.vte_token_wait(ctx, co)
            b = H.mismatched_bits(ref, got)[1]
            r["fixed_mismatched_bits"] += b
            r["fixed_trials_with_mismatch"] += int(b > 0)
        out["gemm_%dx%dx%d" % (gm, gn, gk)] = r
        vte.vte_desc_destroy(dg_)
        del tA, tB, tC

    # ---- decoding level: one state replayed (reduced vocabulary keeps it short) ------------------------
    if "replay" not in sections or replays < 1:
        vte.vte_shutdown(ctx)
        return out
    print("determinism: decode state replay, %d replays" % replays, file=sys.stderr, flush=True)
    shp = inputs.DecodeShapes(D=4096, Nqkv=6144, F=14336, V=32064)
    w = inputs.decode_weights(seed0, shp)
    wd = H.upload_weights(w)
    B = 8
    tok0 = inputs.tokens(seed0, inputs.T_TOK0, B, shp.V)
    base = H.DecodeChain(ctx, wd, shp, B, want_logits=True)
    base.set_tokens(tok0)
    base.run_step_on(p256)
    # the replay also records the softmax probability of the greedy token (Sec. 7.2)
    prob = torch.zeros(B, dtype=torch.float32, device="cuda")
    d_prob = vte.vte_desc_softmax_prob(ctx, base.logits, base.next, prob, B, shp.V)
    H.run_on(ctx, d_prob, p256)
    p0 = prob.cpu().numpy().copy()
    s0 = base.snapshot()
    chains = {S: H.DecodeChain(ctx, wd, shp, B, want_logits=True, splitk=S, rms_active_cus=32 * S) for S in (1, 2, 4, 8)}
    r = {"replays": replays, "fixed_logit_mismatched_bits": 0, "fixed_token_flips": 0,
         "reshaped_logit_mismatched_bits": 0, "reshaped_token_flips": 0, "reshaped_max_logit_diff": 0.0,
         "reshaped_replays_with_logit_drift": 0, "fixed_prob_mismatched_bits": 0, "reshaped_max_prob_diff": 0.0,
         "greedy_token_prob_min": float(p0.min()), "greedy_token_prob_max": float(p0.max())}
    probs_r = {S: torch.zeros(B, dtype=torch.float32, device="cuda") for S in chains}
    d_prob_r = {S: vte.vte_desc_softmax_prob(ctx, chains[S].logits, chains[S].next, probs_r[S], B, shp.V) for S in chains}
    chains[1].set_tokens(tok0)
    chains[1].run_step_on(H.pctx_of_width(ctx, 32))
    s1 = chains[1].snapshot()
    r["split1_equals_fixed"] = bool(np.array_equal(s1["logits"].view(np.uint32), s0["logits"].view(np.uint32)))
    for t in range(replays):
        if t % 20 == 0:
            print("determinism: replay %d" % t, file=sys.stderr, flush=True)
        ids = [_rand_pctx(rng, ctx) for _ in base.order]
        base.set_tokens(tok0)
        base.run_step_on(ids)
        H.run_on(ctx, d_prob, _rand_pctx(rng, ctx))
        s = base.snapshot()
        r["fixed_prob_mismatched_bits"] += H.mismatched_bits(p0, prob.cpu().numpy())[1]
        r["fixed_logit_mismatched_bits"] += H.mismatched_bits(s0["logits"], s["logits"])[1]
        r["fixed_token_flips"] += int(np.count_nonzero(s0["next"] != s["next"]))
        S = (1, 2, 4, 8)[int(rng.integers(0, 4))]
        c = chains[S]
        c.set_tokens(tok0)
        c.run_step_on(H.pctx_of_width(ctx, 32 * S))
        H.run_on(ctx, d_prob_r[S], H.pctx_of_width(ctx, 32 * S))
        s = c.snapshot()
        r["reshaped_max_prob_diff"] = max(r["reshaped_max_prob_diff"], float(np.abs(probs_r[S].cpu().numpy() - p0).max()))
        b = H.mismatched_bits(s0["logits"], s["logits"])[1]
        r["reshaped_logit_mismatched_bits"] += b
        r["reshaped_replays_with_logit_drift"] += int(b > 0)
        r["reshaped_token_flips"] += int(np.count_nonzero(s0["next"] != s["next"]))
        r["reshaped_max_logit_diff"] = max(r["reshaped_max_logit_diff"], float(np.abs(s0["logits"] - s["logits"]).max()))
    top2 = np.sort(s0["logits"], axis=1)[:, -2:]
    r["min_top2_margin_of_state"] = float((top2[:, 1] - top2[:, 0]).min())
    out["decode_state_replay_B8_V32064"] = r
    vte.vte_shutdown(ctx)
    return out


# ----------------------------------------------------------------------------------------------------
def step_latencies(recs, first_kernel, last_kernel):
    """Device-clock latency of every decode step in `recs` (op records with timed first and last
    launches): end of the step's last kernel minus begin of its first.  Seconds."""
    out, begin = [], None
    for r in sorted((r for r in recs if r.klass == vte.VTE_CLASS_LATENCY), key=lambda r: r.token):
        if r.kernel == first_kernel and r.gpu_begin >= 0:
            begin = r.gpu_begin
        elif r.kernel == last_kernel and r.gpu_end >= 0 and begin is not None:
            out.append(r.gpu_end - begin)
            begin = None
    return out


def overlap_of_tenants(recs, first_kernel, last_kernel):
    """From the device-clock intervals of the timed launches: how many best-effort launches ran on
    fewer than all CUs while a decode step was in progress on another pCtx (spatial sharing), and
    how many ran on the whole device (then the tenants can only have alternated in time)."""
    steps, begin, pctx = [], None, -1
    for r in sorted((r for r in recs if r.klass == vte.VTE_CLASS_LATENCY), key=lambda r: r.token):
        if r.kernel == first_kernel and r.gpu_begin >= 0:
            begin, pctx = r.gpu_begin, r.pctx
        elif r.kernel == last_kernel and r.gpu_end >= 0 and begin is not None:
            steps.append((begin, r.gpu_end, pctx))
            begin = None
    side_by_side = whole_device = 0
    widths = set()
    shared_step = [False] * len(steps)
    for r in recs:
        if r.klass != vte.VTE_CLASS_BEST_EFFORT or r.gpu_begin < 0:
            continue
        hit = False
        for i, (b, e, p) in enumerate(steps):
            if b < r.gpu_end and r.gpu_begin < e and p != r.pctx:
                hit = shared_step[i] = True
        if hit:
            side_by_side += 1
            widths.add(int(r.width))
        elif r.width >= 256:
            whole_device += 1
    return {"best_effort_launches_beside_a_decode_step": side_by_side, "their_widths": sorted(widths),
            "best_effort_launches_alone_on_256": whole_device,
            "decode_steps": len(steps), "decode_steps_beside_a_best_effort_launch": int(sum(shared_step))}


def cotenancy(seconds, gap_ms, steps_per_burst=128, lead_ms=3.0, shared=None, modes=("fixed", "late", "late_nohint")):
    """shared: optional dict with the config-3 weights already made ("w", "wd", "shp") and the GEMM
    operands ("gA", "gB", "gC")."""
    shared = shared or {}
    shp = shared.get("shp") or inputs.DecodeShapes()
    w = shared.get("w") or inputs.decode_weights(0, shp)
    B, M = 8, 8192
    cfg = vte.vte_pool_cfg_default()
    cfg.mode = vte.VTE_MODE_PIPELINED
    cfg.lookahead = 16
    # device-clock begin of every step's first launch and end of its last, and the co-tenant's launches
    cfg.device_timing_mask = (1 << vte.VTE_K_RMSNORM_GATHER) | (1 << vte.VTE_K_ARGMAX_FINISH) | (1 << vte.VTE_K_GEMM)
    torch.zeros(1, device="cuda")
    ctx = vte.vte_init(0, cfg)
    wd = shared.get("wd") or H.upload_weights(w)
    ch = H.DecodeChain(ctx, wd, shp, B, feedback=True, fused_gather=True)
    gA = shared["gA"] if "gA" in shared else H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, M)))
    gB = shared["gB"] if "gB" in shared else H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (M, M)))
    gC = shared["gC"] if "gC" in shared else H.dev_empty((M, M))
    gemm = vte.vte_desc_gemm(ctx, gA, gB, gC, M, M, M)
    tok0 = inputs.tokens(0, inputs.T_TOK0, B, shp.V)
    lat = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
    be = vte.vte_vstream_create(ctx, vte.VTE_CLASS_BEST_EFFORT)
    a128 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 0)
    b128 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 1)

    # width profiles of every recurring launch (Sec. 5 "Performance Profiles")
    prof = {}
    for k in ch.order:
        vte.vte_profile_measure(ctx, ch.desc[k], 2, 5)
        key = vte.vte_desc_info(ch.desc[k]).profile_key
        prof[k] = {wd_: round(vte.vte_profile_get(ctx, key, wd_) * 1e6, 2) for wd_ in (32, 64, 128, 192, 224, 256)}
    vte.vte_profile_measure(ctx, gemm, 1, 3)
    key = vte.vte_desc_info(gemm).profile_key
    prof["gemm"] = {wd_: round(vte.vte_profile_get(ctx, key, wd_) * 1e6, 1) for wd_ in (32, 64, 128, 192, 224, 256)}

    def run(mode, with_gemm=True, with_decode=True):
        """mode: 'solo' | 'fixed' | 'late' | 'late_nohint'.  Returns dict of raw measurements."""
        vte.vte_device_sync(ctx)
        vte.vte_stats_reset(ctx)
        # a hint of the mode before may have been submitted and not used (the run ended before its burst): its
        # reservation would keep the GEMM off the full device for this whole mode
        for i in range(vte.vte_pool_count(ctx)):
            if vte.vte_pool_info(ctx, i).reserved_for == vte.vte_vstream_id(lat):
                vte.vte_pctx_unreserve(ctx, i)
        vte.vte_vstream_pin(lat, a128 if mode == "fixed" else -1)
        vte.vte_vstream_pin(be, b128 if mode == "fixed" else -1)
        # slack 0.4: beside the GEMM the decode chain takes the narrowest pCtx whose profiled chain time is within
        # 40 % of the best one on offer.  The chain's times step by 1.17 (224 or 192 CUs against 256), 1.26 (128
        # against 256), 1.72 (64 against 128) and 1.83 (32 against 64): 0.4 sits between the steps; 0.7, used before,
        # sat on the 1.72 one, and a noisy profile then parked whole bursts on 64 CUs
        vte.vte_set_builtin_policy(ctx, vte.VTE_POLICY_QUEUE_STATE if mode.startswith("late") else vte.VTE_POLICY_WIDEST,
                                   0.4, 128 if mode.startswith("late") else 0)
        ch.set_tokens(tok0)
        gemm_q, gemm_done = [], 0
        bursts, burst_times, burst_tokens = 0, [], []
        t_start = time.perf_counter()
        next_burst = t_start + 0.005
        hinted = False
        state, tail, t_burst0 = "idle", 0, 0.0
        while True:
            now = time.perf_counter()
            if now - t_start > seconds and state == "idle":
                break
            if with_gemm:
                while gemm_q and vte.vte_token_query(ctx, gemm_q[0]):
                    gemm_q.pop(0)
                    gemm_done += 1
                while len(gemm_q) < 2:
                    gemm_q.append(vte.vte_submit(be, gemm))
            if with_decode:
                if state == "idle":
                    if mode == "late" and not hinted and now >= next_burst - lead_ms * 1e-3:
                        vte.vte_hint_submit(ctx, vte.vte_hint(vte.vte_vstream_id(lat), 128, lead_ms * 1e-3, 0.0))
                        hinted = True
                    if now >= next_burst:
                        t_burst0 = time.perf_counter()
                        for _ in range(steps_per_burst):
                            tail = ch.submit_step(lat)
                        state = "busy"
                elif vte.vte_token_query(ctx, tail):
                    burst_times.append(time.perf_counter() - t_burst0)
                    bursts += 1
                    burst_tokens.append(ch.tok.cpu().numpy().tolist())   # outside the timed burst
                    state = "idle"
                    if hinted:
                        for i in range(vte.vte_pool_count(ctx)):
                            if vte.vte_pool_info(ctx, i).reserved_for == vte.vte_vstream_id(lat):
                                vte.vte_pctx_unreserve(ctx, i)
                        hinted = False
                    next_burst = time.perf_counter() + gap_ms * 1e-3
            time.sleep(0.0001)
        elapsed = time.perf_counter() - t_start
        for t in gemm_q:
            vte.vte_token_wait(ctx, t)
        vte.vte_device_sync(ctx)
        recs = vte.vte_stats_read(ctx)
        # first-step latency of each burst: submit of its first op to completion of its first argmax
        lat_recs = sorted((r for r in recs if r.klass == vte.VTE_CLASS_LATENCY), key=lambda r: r.token)
        first_lat = []
        per = len(ch.order)
        for i in range(0, len(lat_recs) - per + 1, per * steps_per_burst):
            first_lat.append(lat_recs[i + per - 1].t_done - lat_recs[i].t_submit)
        gw = [r.width for r in recs if r.klass == vte.VTE_CLASS_BEST_EFFORT]
        dw = [r.width for r in recs if r.klass == vte.VTE_CLASS_LATENCY]
        sl = step_latencies(recs, vte.VTE_K_RMSNORM_GATHER, vte.VTE_K_ARGMAX_FINISH)
        ov = overlap_of_tenants(recs, vte.VTE_K_RMSNORM_GATHER, vte.VTE_K_ARGMAX_FINISH) if with_gemm and with_decode else None
        return {"elapsed_s": elapsed, "steps_timed": len(sl),
                # per step on the device clock: begin of the step's first kernel to end of its last
                "step_latency_ms_p50": float(np.percentile(sl, 50) * 1e3) if sl else None,
                "step_latency_ms_p99": float(np.percentile(sl, 99) * 1e3) if sl else None,
                "step_latency_ms_max": float(np.max(sl) * 1e3) if sl else None,
                "overlap": ov, "gemm_done": gemm_done, "gemm_per_s": gemm_done / elapsed, "bursts": bursts,
                "burst_ms_mean": float(np.mean(burst_times) * 1e3) if burst_times else None,
                "burst_ms_max": float(np.max(burst_times) * 1e3) if burst_times else None,
                "step_ms_mean": float(np.mean(burst_times) * 1e3 / steps_per_burst) if burst_times else None,
                "burst_step_ms_p99": float(np.percentile(burst_times, 99) * 1e3 / steps_per_burst) if burst_times else None,
                "first_step_ms_mean": float(np.mean(first_lat) * 1e3) if first_lat else None,
                "first_step_ms_max": float(np.max(first_lat) * 1e3) if first_lat else None,
                "gemm_widths": {str(k): int(v) for k, v in zip(*np.unique(gw, return_counts=True))} if gw else {},
                "decode_widths": {str(k): int(v) for k, v in zip(*np.unique(dw, return_counts=True))} if dw else {},
                "burst_tokens": burst_tokens}

    res = {"profiles_us": prof, "gap_ms": gap_ms, "steps_per_burst": steps_per_burst, "lead_ms": lead_ms}
    res["solo_gemm"] = run("solo", with_decode=False)
    res["solo_decode"] = run("solo", with_gemm=False)
    for mode in modes:
        res[mode] = run(mode)
    g0 = res["solo_gemm"]["gemm_per_s"]
    d0 = res["solo_decode"]["burst_ms_mean"]
    for mode in modes:
        r = res[mode]
        r["norm_gemm"] = r["gemm_per_s"] / g0
        r["norm_decode"] = d0 / r["burst_ms_mean"] if r["burst_ms_mean"] else None
        r["aggregate_normalized_throughput"] = r["norm_gemm"] + (r["norm_decode"] or 0.0)
    # the token stream is a function of the start tokens and the number of steps run alone:
    # whatever widths a mode used, the tokens after burst i must equal the solo run's
    ref = res["solo_decode"]["burst_tokens"]
    for mode in modes:
        got = res[mode]["burst_tokens"]
        m = min(len(ref), len(got))
        res[mode]["bursts_compared"] = m
        res[mode]["bursts_with_token_mismatch"] = sum(int(ref[i] != got[i]) for i in range(m))
    for mode in ("solo_gemm", "solo_decode") + tuple(modes):
        bt = res[mode].pop("burst_tokens")
        res[mode]["final_tokens"] = bt[-1] if bt else None
    res["gemm_tflops_solo"] = 2 * M ** 3 * g0 / 1e12
    vte.vte_shutdown(ctx)
    return res


def config1_latency(ctx, launches=200):
    """BASELINE config 1: the fixed-structure RMSNorm 8 x 1024 (x ~ N(0,1), gamma ~ U(0.5,1.5), eps 1e-6,
    seed 0) launched explicitly on one pCtx of every width: host-clock latency of bind + launch +
    completion per launch (microseconds), and the bits against the 256-CU run."""
    x, g = inputs.rmsnorm_case(seed=0, rows=8, cols=1024)
    dx, dg, dy = H.to_dev(x), H.to_dev(g), H.dev_empty((8, 1024))
    d = vte.vte_desc_rmsnorm(ctx, dx, dg, dy, 8, 1024, 1e-6)
    out, ref = {}, None
    for width in (256, 224, 192, 128, 64, 32):
        p = H.pctx_of_width(ctx, width)
        for _ in range(10):
            H.run_on(ctx, d, p)
        ts = []
        for _ in range(launches):
            t0 = time.perf_counter()
            vte.vte_token_wait(ctx, vte.vte_bind_and_launch(ctx, d, p))
            ts.append(time.perf_counter() - t0)
        bits = H.to_bits(dy).copy()
        ref = bits if ref is None else ref
        out[str(width)] = {"p50_us": round(float(np.percentile(ts, 50)) * 1e6, 2), "p95_us": round(float(np.percentile(ts, 95)) * 1e6, 2),
                           "mismatched_bits_vs_256": H.mismatched_bits(ref, bits)[1]}
    vte.vte_desc_destroy(d)
    return out


def gemm_widths(reps, M=8192):
    """The co-tenant GEMM alone on one pCtx of every width: device time per launch (the profiling target)."""
    torch.zeros(1, device="cuda")
    ctx = H.make_ctx()
    gA = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, M)))
    gB = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (M, M)))
    gC = H.dev_empty((M, M))
    d = vte.vte_desc_gemm(ctx, gA, gB, gC, M, M, M)
    out = {"M": M, "reps": reps, "widths": {}}
    for width in (256, 224, 192, 128, 64, 32):
        # as many warm-up launches as timed ones: at full width the clock settles only after about
        # fifteen back-to-back launches (a burst of six averages 15 % slower than the steady state)
        t = vte.vte_profile_measure_on(ctx, d, H.pctx_of_width(ctx, width), reps, reps)
        out["widths"][str(width)] = {"ms": t * 1e3, "TFLOP/s": 2.0 * M ** 3 / t / 1e12, "pct_of_2.5_PFLOP/s": 2.0 * M ** 3 / t / 2.5e13}
    vte.vte_shutdown(ctx)
    return out


def operators_by_width(reps):
    """The metric's bandwidth-bound operators alone on one pCtx of every width, `reps` launches each, in a fixed
    order (width-major: 256, 224, 192, 128, 64, 32; per width RMSNorm 32768x4096, GEMV 4096x4096 batch 8 over 8
    weight buffers in rotation, LM head 128256x4096 batch 8): the target of the per-width kernel trace.
    Inputs as BASELINE states them: x ~ N(0,1), gamma ~ U(0.5,1.5), weights ~ N(0, 1/K)."""
    torch.zeros(1, device="cuda")
    ctx = H.make_ctx()
    rows, cols, N, V, B = 32768, 4096, 4096, 128256, 8
    x = H.to_dev(inputs.normal_bf16(0, inputs.T_X, (rows, cols)))
    y = torch.empty_like(x)
    g = H.to_dev(inputs.uniform_bf16(0, inputs.T_GAMMA, (cols,), 0.5, 1.5))
    d_norm = vte.vte_desc_rmsnorm(ctx, x, g, y, rows, cols, 1e-6)
    Ws = [H.to_dev(inputs.normal_bf16(i, inputs.T_W, (N, cols), 0.0, cols ** -0.5)) for i in range(8)]
    X = H.to_dev(inputs.normal_bf16(0, inputs.T_XB, (B, cols)))
    Y = torch.empty((B, N), dtype=torch.int16, device="cuda")
    d_gemv = [vte.vte_desc_gemv(ctx, W_, X, Y, B, N, cols) for W_ in Ws]
    Wlm = H.to_dev(inputs.normal_bf16(0, inputs.T_WLM, (V, cols), 0.0, 0.02))
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, cols))
    d_lm = vte.vte_desc_lmhead_argmax(ctx, Wlm, X, tok, None, ws, B, V, cols)
    out = {"reps": reps, "order": ["rmsnorm_32768x4096", "gemv_4096x4096_B8", "lmhead_128256x4096_B8"], "widths": {}}
    for width in (256, 224, 192, 128, 64, 32):
        p = H.pctx_of_width(ctx, width)
        r = {}
        t = vte.vte_profile_measure_on(ctx, d_norm, p, 0, reps)
        r["rmsnorm_32768x4096"] = {"us": t * 1e6, "GB/s": vte.vte_desc_info(d_norm).bytes / t / 1e9}
        ts = [vte.vte_profile_measure_on(ctx, d_gemv[i % 8], p, 0, 1) for i in range(reps)]
        t = float(np.median(ts))
        r["gemv_4096x4096_B8"] = {"us": t * 1e6, "GB/s": vte.vte_desc_info(d_gemv[0]).bytes / t / 1e9}
        t = vte.vte_profile_measure_on(ctx, d_lm, p, 0, reps)
        r["lmhead_128256x4096_B8"] = {"us": t * 1e6, "GB/s": vte.vte_desc_info(d_lm).bytes / t / 1e9}
        out["widths"][str(width)] = r
    vte.vte_shutdown(ctx)
    return out


def overhead(launches):
    """Dispatch overhead in kind (Sec. 7.5): the paper's probe is a BF16 GEMM of shape (512, 8192, 28672).
    Native = the same descriptor launched back to back on the 256-CU stream by the backend itself (no
    dispatcher); STRICT / PIPELINED = the same launches through a virtual stream and the dispatcher;
    on-demand = what creating the pool's CU-masked streams costs (they are pre-created once)."""
    out = {"launches": launches}
    M, N, K = 512, 8192, 28672
    res = {}
    for mode, name in ((vte.VTE_MODE_STRICT, "strict"), (vte.VTE_MODE_PIPELINED, "pipelined")):
        t0 = time.perf_counter()
        ctx = H.make_ctx(mode, lookahead=32)
        t_init = time.perf_counter() - t0
        gA = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, K)))
        gB = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (N, K)))
        gC = H.dev_empty((M, N))
        d = vte.vte_desc_gemm(ctx, gA, gB, gC, M, N, K)
        root = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 256)
        native = vte.vte_profile_measure_on(ctx, d, root, 10, launches)
        vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
        vte.vte_set_builtin_policy(ctx, vte.VTE_POLICY_WIDEST)
        arr = vte.desc_array([d] * launches)
        vte.vte_token_wait(ctx, vte.vte_submit_batch(vs, vte.desc_array([d] * 10)))
        t = time.perf_counter()
        vte.vte_token_wait(ctx, vte.vte_submit_batch(vs, arr))
        through = (time.perf_counter() - t) / launches
        # a short kernel shows the per-launch cost itself
        x = H.dev_empty((8, 4096)); g = H.dev_empty((4096,)); y = H.dev_empty((8, 4096))
        dn = vte.vte_desc_rmsnorm(ctx, x, g, y, 8, 4096, 1e-6)
        native_s = vte.vte_profile_measure_on(ctx, dn, root, 10, launches)
        arr_s = vte.desc_array([dn] * launches)
        vte.vte_token_wait(ctx, vte.vte_submit_batch(vs, vte.desc_array([dn] * 10)))
        t = time.perf_counter()
        vte.vte_token_wait(ctx, vte.vte_submit_batch(vs, arr_s))
        through_s = (time.perf_counter() - t) / launches
        res[name] = {"gemm_native_us": native * 1e6, "gemm_through_runtime_us": through * 1e6,
                     "gemm_overhead_pct": 100 * (through / native - 1),
                     "norm_native_us": native_s * 1e6, "norm_through_runtime_us": through_s * 1e6,
                     "pool_creation_ms": t_init * 1e3, "pool_streams": vte.vte_pool_count(ctx),
                     "per_stream_creation_ms": t_init * 1e3 / vte.vte_pool_count(ctx)}
        vte.vte_shutdown(ctx)
    out.update(res)
    out["pools"] = overhead_pools(launches)
    return out


def overhead_pools(launches):
    """The pool arms of the same study: the bounded hierarchical pool (tree + one remainder per level,
    17 queues) against a flat one that pre-creates every node's remainder as well (27 queues, more
    than the device keeps resident at once).  Per arm: end-to-end latency of one GEMM (host clock
    around launch + wait; median and p95) bound explicitly to the 256-CU pCtx and submitted through
    a STRICT virtual stream, and what creating the pool takes in time, device memory and host RSS."""
    import psutil
    proc = psutil.Process()
    M, N, K = 512, 8192, 28672
    gA = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, K)))
    gB = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (N, K)))
    gC = H.dev_empty((M, N))
    arms = {}
    for name, rem in (("hierarchical", vte.VTE_REMAINDERS_PER_LEVEL), ("flat", vte.VTE_REMAINDERS_ALL)):
        cfg = vte.vte_pool_cfg_default()
        cfg.mode = vte.VTE_MODE_STRICT
        cfg.with_remainders = rem
        torch.cuda.synchronize()
        free0, rss0 = torch.cuda.mem_get_info()[0], proc.memory_info().rss
        t0 = time.perf_counter()
        ctx = vte.vte_init(0, cfg)
        t_init = time.perf_counter() - t0
        free1, rss1 = torch.cuda.mem_get_info()[0], proc.memory_info().rss
        d = vte.vte_desc_gemm(ctx, gA, gB, gC, M, N, K)
        root = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 256)
        vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
        vte.vte_set_builtin_policy(ctx, vte.VTE_POLICY_WIDEST)
        lat = {"explicit": [], "vstream": []}
        for i in range(10 + launches):
            t = time.perf_counter()
            vte.vte_token_wait(ctx, vte.vte_bind_and_launch(ctx, d, root))
            t1 = time.perf_counter()
            vte.vte_token_wait(ctx, vte.vte_submit(vs, d))
            t2 = time.perf_counter()
            if i >= 10:
                lat["explicit"].append(t1 - t)
                lat["vstream"].append(t2 - t1)
        arm = {"queues": vte.vte_pool_count(ctx), "creation_ms": t_init * 1e3,
               "device_bytes": int(free0 - free1), "host_rss_bytes": int(rss1 - rss0)}
        for k, v in lat.items():
            v.sort()
            arm[k + "_median_us"] = v[len(v) // 2] * 1e6
            arm[k + "_p95_us"] = v[min(len(v) - 1, int(0.95 * len(v)))] * 1e6
            arm[k + "_max_us"] = v[-1] * 1e6
        arms[name] = arm
        vte.vte_shutdown(ctx)
    return arms


RAMP_POINTS = ("entry", "first weights requested", "all first loads issued (weights, then X)", "X (its first block) arrived and turned",
               "first block of weights multiplied", "wave's share of the stream through", "all waves of the workgroup through",
               "sums added, outputs stored")
RAMP_SLOTS = (0, 7, 1, 2, 3, 4, 5, 6)   # the stamp slot (csrc/gemv_mfma_kernel.h) behind each point, in the order of the timeline


def ramp(batches=(8, 16), N=4096, K=4096, width=256, bursts=9):
    """Where the time of one small GEMV launch goes (BASELINE config 2: 4096 x 4096; the matrix-core
    kind, batch 3 to 16).  Needs the trace build of the library (`python -m paper_2603_15042_amd.build
    --trace`), whose kernels stamp the device's 100 MHz clock per wave (csrc/trace_stamps.h): 128
    launches back to back on a stream pinned to one pCtx, 32 weight buffers in rotation; reported are,
    for the last launch of a burst, the stamps of all waves relative to the first wave's entry (each
    statistic the median over several bursts), and the time per launch of the burst (which also holds
    the gap between launches)."""
    import ctypes as C
    L = vte.load()
    if not hasattr(L, "vte_trace_stamps_read"):
        raise RuntimeError("ramp needs the trace build: python -m paper_2603_15042_amd.build --trace, then run with "
                           "the ramp command first on the command line (it selects libvte_trace.so before the library loads)")
    ctx = H.make_ctx(vte.VTE_MODE_PIPELINED, lookahead=64)
    Ws = [H.to_dev(inputs.normal_bf16(i, inputs.T_W, (N, K), 0.0, K ** -0.5)) for i in range(32)]
    out = {"shape": [N, K], "width": width, "points": list(RAMP_POINTS), "batches": {}}
    for B in batches:
        X = H.to_dev(inputs.normal_bf16(0, inputs.T_XB, (B, K)))
        Y = torch.empty((B, N), dtype=torch.int16, device="cuda")
        ds = [vte.vte_desc_gemv(ctx, W_, X, Y, B, N, K) for W_ in Ws]
        info = vte.vte_desc_info(ds[0])
        v = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
        vte.vte_vstream_pin(v, H.pctx_of_width(ctx, width))
        vte.vte_token_wait(ctx, vte.vte_submit_batch(v, vte.desc_array(ds)))
        wgs, waves = info.grid[0], info.block[0] // 64
        per_launch, tables = [], []
        for burst in range(bursts):
            tb = time.perf_counter()
            vte.vte_token_wait(ctx, vte.vte_submit_batch(v, vte.desc_array(ds * 4)))
            per_launch.append((time.perf_counter() - tb) / (4 * len(ds)))
            torch.cuda.synchronize()
            buf = np.zeros(1024 * 8 * 8, dtype=np.uint64)
            rc = L.vte_trace_stamps_read(buf.ctypes.data_as(C.c_void_p), C.c_size_t(buf.size))
            if rc != 0:
                raise RuntimeError("vte_trace_stamps_read: HIP error %d" % rc)
            st = buf.reshape(1024, 8, 8).astype(np.int64)[:min(wgs, 1024), :waves][:, :, list(RAMP_SLOTS)]
            rel = (st - st[:, :, 0].min()) * 0.01                 # us after the first wave's entry
            tables.append([[float(f(rel[:, :, i])) for f in (np.min, lambda c: np.percentile(c, 10), np.median,
                                                             lambda c: np.percentile(c, 90), np.max)] for i in range(len(RAMP_POINTS))])
        vte.vte_vstream_destroy(v)
        med = np.median(np.array(tables), axis=0)                 # per statistic, the median over the bursts' last launches
        rows = {name: dict(zip(("min", "p10", "median", "p90", "max"), (round(float(x), 2) for x in med[i]))) for i, name in enumerate(RAMP_POINTS)}
        t = float(np.median(per_launch)) * 1e6
        out["batches"][str(B)] = {"workgroups": int(wgs), "waves_per_workgroup": int(waves), "bursts": bursts,
                                  "us_per_launch_back_to_back": round(t, 2), "us_after_first_entry": rows,
                                  "last_wave_done_to_next_launch_entry_us": round(t - float(med[len(RAMP_POINTS) - 1][4]), 2)}
        for d in ds:
            vte.vte_desc_destroy(d)
    vte.vte_shutdown(ctx)
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    d = sub.add_parser("determinism")
    d.add_argument("--trials", type=int, default=1000)
    d.add_argument("--replays", type=int, default=100)
    c = sub.add_parser("cotenancy")
    c.add_argument("--seconds", type=float, default=3.0)
    c.add_argument("--gap-ms", type=float, default=60.0)
    g = sub.add_parser("gemm")
    g.add_argument("--reps", type=int, default=5)
    ov = sub.add_parser("overhead")
    ov.add_argument("--launches", type=int, default=200)
    o = sub.add_parser("operators")
    o.add_argument("--reps", type=int, default=8)
    sub.add_parser("ramp")
    a = ap.parse_args(argv)
    if a.cmd == "ramp":                       # the trace build, selected before anything loads the library
        import os
        vte.LIB_PATH = os.path.join(os.path.dirname(vte.LIB_PATH), "libvte_trace.so")
        print(json.dumps(ramp()))
        return
    if a.cmd == "determinism":
        out = determinism(a.trials, a.replays)
    elif a.cmd == "gemm":
        out = gemm_widths(a.reps)
    elif a.cmd == "operators":
        out = operators_by_width(a.reps)
    elif a.cmd == "overhead":
        out = overhead(a.launches)
    else:
        out = cotenancy(a.seconds, a.gap_ms)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
