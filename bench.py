"""Benchmark of the decode hot path on one MI355X.

A step is one pass of the Llama-8B-shaped decode chain at batch 8 (greedy-token
finish + embedding gather + RMSNorm in one launch, QKV, O, gate/up+SiLU, down,
LM head: six immutable descriptors per step submitted to a virtual stream and
late-bound by the dispatcher), on synthetic weights resident in HBM.  Prints
one JSON line.  Outside the timed region it also measures, each under its own
key: the chain and the single operators of the metric on pCtxs of every width
(bits compared across widths), the other batch sizes, the strict binding mode,
co-tenancy with the 8192^3 GEMM against a fixed 128/128 split, the determinism
protocol at a reduced trial count, the launch latency of the 8 x 1024 RMSNorm,
and the CPU oracle on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
WIDTHS = (256, 224, 192, 128, 64, 32)


def _committed_counter_traffic():
    """HBM bytes per LM-head launch as counted by rocprofv3 for the committed profile (not measured
    in this run): (bytes, file) or (None, None)."""
    name = os.path.join("profiles", "decode_chain_b8_hbm_counters.txt")
    try:
        for line in open(os.path.join(ROOT, name)):
            if line.startswith("lmhead_traffic_bytes_per_launch="):
                return int(line.split("=")[1]), name
    except OSError:
        pass
    return None, None


def _log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


class _section:
    """One of the measurements behind the headline: announced on stderr; if it raises, the error goes into
    out["errors"] and the run goes on, so that the JSON line with the metric is printed whatever happens
    to the extras."""

    def __init__(self, out, name):
        self.out, self.name = out, name

    def __enter__(self):
        _log(self.name)

    def __exit__(self, et, ev, tb):
        if et is None or not issubclass(et, Exception):
            return False
        self.out.setdefault("errors", {})[self.name] = "%s: %s" % (et.__name__, ev)
        _log("FAILED %s: %s: %s" % (self.name, et.__name__, ev))
        return True


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--settle-steps", type=int, default=400,
                    help="steps of the same chain run before the warm-up, untimed: a device that comes out of idle (weights "
                         "were being generated and uploaded) runs its first 25 ms or so about 2 %% slower, which a short "
                         "--warmup would leave inside the timed region")
    ap.add_argument("--mode", choices=("pipelined", "strict"), default="pipelined")
    ap.add_argument("--lookahead", type=int, default=64, help="launches bound ahead of the oldest unfinished one (pipelined binding)")
    ap.add_argument("--timing-stride", type=int, default=8,
                    help="in the metric's pass every n-th LM-head launch carries a HIP event pair (a timed launch idles "
                         "its stream for a few us on either side); the roofline's kernel time comes from a second pass "
                         "over the same steps with every LM-head launch timed")
    ap.add_argument("--no-kernel-timing", action="store_true", help="do not bracket the LM head with device events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-width-sweep", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip strict / co-tenancy / determinism / config-1 latency")
    ap.add_argument("--cotenancy-seconds", type=float, default=2.0)
    ap.add_argument("--determinism-trials", type=int, default=50)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three 1 GiB device-to-device copies (a known-size reference for HBM byte counters)")
    ap.add_argument("--small", action="store_true", help="reduced shapes (debugging only; not a valid result)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2603_15042_amd import harness as H, inputs, vte
    if not os.path.exists(vte.LIB_PATH):
        from paper_2603_15042_amd import build as b
        b.build()

    shp = inputs.DecodeShapes(D=1024, Nqkv=1536, F=3584, V=32064) if a.small else inputs.DecodeShapes()
    B = a.batch
    t0 = time.time()
    w = inputs.decode_weights(0, shp)
    tok0 = inputs.tokens(0, inputs.T_TOK0, B, shp.V)
    gen_s = time.time() - t0

    stride = max(1, a.timing_stride)
    cfg = vte.vte_pool_cfg_default()
    cfg.mode = vte.VTE_MODE_PIPELINED if a.mode == "pipelined" else vte.VTE_MODE_STRICT
    cfg.lookahead = a.lookahead
    cfg.device_timing_mask = 0 if a.no_kernel_timing else 1 << vte.VTE_K_LMHEAD
    cfg.device_timing_stride = stride
    torch.zeros(1, device="cuda")
    ctx = vte.vte_init(0, cfg)
    wd = H.upload_weights(w)
    ch = H.DecodeChain(ctx, wd, shp, B, feedback=True, fused_gather=True, fused_argmax=True)
    vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)

    def run(chain, steps, vstream):
        chain.submit_burst(vstream, steps)
        vte.vte_vstream_sync(vstream)

    ch.set_tokens(tok0)
    if a.settle_steps > 0:
        run(ch, a.settle_steps, vs)
        ch.set_tokens(tok0)
    run(ch, a.warmup, vs)
    vte.vte_device_sync(ctx)
    torch.cuda.synchronize()
    vte.vte_stats_reset(ctx)
    t1 = time.perf_counter()
    run(ch, a.steps, vs)
    vte.vte_device_sync(ctx)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    recs = vte.vte_stats_read(ctx)
    st = vte.vte_stats(ctx)
    lm_metric = [r.gpu_seconds for r in recs if r.kernel == vte.VTE_K_LMHEAD and r.gpu_seconds > 0]
    lm_bytes = vte.vte_desc_info(ch.desc["lmhead"]).bytes
    step_bytes = ch.bytes_per_step
    value = step_bytes * a.steps / dt / 1e9
    tokens_end = ch.tok.cpu().numpy().copy()
    # The dominant kernel's duration: the same steps once more, every LM-head launch bracketed by a HIP event
    # pair on its own dispatch and stream (at least 16 launches).  Kept out of the metric's pass because a
    # timed launch idles its stream for a few us on either side; the metric's pass carries a thin sample
    # (every --timing-stride-th launch) as a cross-check that the kernel runs the same in both.
    lm, dt_timed, n_timed = lm_metric, float("nan"), 0
    if not a.no_kernel_timing:
        n_timed = min(max(a.steps, 16), 200)
        vte.vte_set_device_timing(ctx, 1 << vte.VTE_K_LMHEAD, 1)
        vte.vte_stats_reset(ctx)
        t2 = time.perf_counter()
        run(ch, n_timed, vs)
        vte.vte_device_sync(ctx)
        torch.cuda.synchronize()
        dt_timed = time.perf_counter() - t2
        lm = [r.gpu_seconds for r in vte.vte_stats_read(ctx) if r.kernel == vte.VTE_K_LMHEAD and r.gpu_seconds > 0]
        vte.vte_set_device_timing(ctx, 0, 0)          # the sections below time whole chains from the host
    lm_avg = float(np.mean(lm)) if lm else float("nan")
    if a.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.int8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    traffic, traffic_file = _committed_counter_traffic()
    out = {
        "metric": "GEMV/RMSNorm HBM GB/s (% peak) per CU width; bit mismatches across widths (=0)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(dt / a.steps * 1e3, 4), "settle_steps_before_warmup": a.settle_steps,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "Llama-8B-shaped decode chain (gather+RMSNorm 4096 -> QKV 4096x6144 -> O 4096x4096 -> "
                               "gate/up 4096x2x14336 SiLU -> down 14336x4096 -> LM head 4096x128256 -> argmax), "
                               "batch %d, 6 launches per step (the argmax finish of a step is fused into the gather+RMSNorm "
                               "launch of the next; 7 in the first step, one finish after the last), full width "
                               "(256 CUs), %s binding" % (B, a.mode),
                   "batch": B, "bytes_per_step": int(step_bytes), "small_shapes": bool(a.small)},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "launches": int(st.completed), "completion_records": int(st.completion_records),
        "roofline": {"bound": "hbm", "kernel": "lm-head GEMV + argmax", "achieved": round(lm_bytes / lm_avg / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(lm_bytes / lm_avg / 1e9 / HBM_PEAK_GBS, 4),
                     "avg_kernel_us": round(lm_avg * 1e6, 2), "launches_timed": len(lm),
                     "timed_in": "a second pass over the same steps (%d) with a HIP event pair on every LM-head launch, on the "
                                 "CU-masked stream it was bound to; %.4f ms per step with the events" % (n_timed, dt_timed / max(n_timed, 1) * 1e3),
                     "metric_pass_sample": {"timing_stride": stride, "launches_timed": len(lm_metric),
                                            "avg_kernel_us": round(float(np.mean(lm_metric)) * 1e6, 2) if lm_metric else None},
                     # HBM bytes per launch as rocprofv3 counted them for the committed profile of this kernel and
                     # workload; not collected in this run (counters need the profiler)
                     "traffic": traffic, "traffic_source": traffic_file,
                     "algorithmic_bytes_per_launch": int(lm_bytes)},
    }

    # ---- per CU width: throughput and bit mismatches (outside the timed region) -------------
    if not a.no_width_sweep:
        with _section(out, "chain per width"):
            per_width, mism = {}, 0
            ref_snap = None
            for width in WIDTHS:
                p = H.pctx_of_width(ctx, width)
                v = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
                vte.vte_vstream_pin(v, p)
                ch.set_tokens(tok0)
                n = max(16, a.steps // 8)
                run(ch, 4, v)
                ch.set_tokens(tok0)
                t = time.perf_counter()
                run(ch, n, v)
                e = time.perf_counter() - t
                snap = ch.snapshot()
                snap["tok"] = ch.tok.cpu().numpy().copy()
                if ref_snap is None:
                    ref_snap = snap
                else:
                    for k in ("n", "qkv", "o", "act", "d"):
                        mism += H.mismatched_bits(ref_snap[k], snap[k])[1]
                    mism += H.mismatched_bits(ref_snap["tok"].astype(np.uint32), snap["tok"].astype(np.uint32))[1]
                gbs = step_bytes * n / e / 1e9
                per_width[str(width)] = {"GB/s": round(gbs, 1), "pct_peak": round(100 * gbs / HBM_PEAK_GBS, 2),
                                         "ms_per_step": round(e / n * 1e3, 4), "steps": n}
                vte.vte_vstream_destroy(v)
            out["per_width"] = per_width
            out["bit_mismatches_across_widths"] = int(mism)

    # ---- the metric's single operators per CU width (outside the timed region) ----
    shared = {"w": w, "wd": wd, "shp": shp}
    if not a.no_width_sweep and not a.small:
        with _section(out, "operators per width"):
            ops = {}
            rows, cols = 32768, 4096                       # RMSNorm at a size HBM has to serve: 256 MiB in, 256 MiB out
            x = H.to_dev(inputs.normal_bf16(0, inputs.T_X, (rows, cols)))           # x ~ N(0,1)
            gam = H.to_dev(inputs.uniform_bf16(0, inputs.T_GAMMA, (cols,), 0.5, 1.5))  # gamma ~ U(0.5,1.5)
            y = torch.empty_like(x)
            d = vte.vte_desc_rmsnorm(ctx, x, gam, y, rows, cols, 1e-6)
            r = {}
            for width in WIDTHS:
                t = vte.vte_profile_measure_on(ctx, d, H.pctx_of_width(ctx, width), 2, 6)
                r[str(width)] = {"GB/s": round(rows * cols * 4 / t / 1e9, 1), "pct_peak": round(rows * cols * 4 / t / 1e9 / 80, 2)}
            ops["rmsnorm_32768x4096"] = r
            vte.vte_desc_destroy(d)
            del x, y
            N = K = 4096                                   # GEMV 4096x4096 (BASELINE config 2): W ~ N(0, 1/K), X ~ N(0,1);
            Ws = [H.to_dev(inputs.normal_bf16(i, inputs.T_W, (N, K), 0.0, K ** -0.5)) for i in range(32)]  # 32 buffers in rotation (1 GiB > caches)
            for b2 in (1, 4, 8):
                X = H.to_dev(inputs.normal_bf16(0, inputs.T_XB, (b2, K)))
                Y = torch.empty((b2, N), dtype=torch.int16, device="cuda")
                plans = {"default": None}
                if b2 == 8:                                # the dot-product plan beside the matrix-core default
                    pl = vte.vte_gemv_plan()
                    pl.batch_tile, pl.rows, pl.ksteps, pl.prefetch, pl.max_waves, pl.groups, pl.kind = 8, 2, 4, 0, 8, 8, vte.VTE_GEMV_DOT2
                    plans["dot2_plan"] = pl
                for pname, pl in plans.items():
                    ds = [vte.vte_desc_gemv(ctx, W_, X, Y, b2, N, K) if pl is None else
                          vte.vte_desc_gemv_planned(ctx, W_, X, Y, b2, N, K, vte.VTE_EPI_NONE, pl) for W_ in Ws]
                    r = {}
                    for width in WIDTHS:
                        # 128 launches back to back on a virtual stream pinned to the pCtx, each on the next weight
                        # buffer; wall time per launch (a single launch between two events would add their cost)
                        v = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
                        vte.vte_vstream_pin(v, H.pctx_of_width(ctx, width))
                        vte.vte_token_wait(ctx, vte.vte_submit_batch(v, vte.desc_array(ds)))
                        burst = vte.desc_array(ds * 4)
                        tb = time.perf_counter()
                        vte.vte_token_wait(ctx, vte.vte_submit_batch(v, burst))
                        t = (time.perf_counter() - tb) / (4 * len(ds))
                        vte.vte_vstream_destroy(v)
                        r[str(width)] = {"GB/s": round(N * K * 2 / t / 1e9, 1), "pct_peak": round(N * K * 2 / t / 1e9 / 80, 2),
                                         "us": round(t * 1e6, 2)}
                    ops["gemv_4096x4096_B%d" % b2 + ("" if pl is None else "_" + pname)] = r
                    for dd in ds:
                        vte.vte_desc_destroy(dd)
            del Ws
            torch.cuda.empty_cache()
            M = 8192                                       # the co-tenant: bf16 MFMA GEMM 8192^3, N(0,1) inputs
            gA = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, M)))
            gB = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (M, M)))
            gC = H.dev_empty((M, M))
            shared.update(gA=gA, gB=gB, gC=gC)
            d = vte.vte_desc_gemm(ctx, gA, gB, gC, M, M, M)
            r = {}
            for width in WIDTHS:
                # steady state: the first dozen back-to-back launches at full width run through a clock transient
                # (0.84 ms, up to 1.05 ms around the fourth, 0.82 ms from the sixteenth on), so they are warm-up
                t = vte.vte_profile_measure_on(ctx, d, H.pctx_of_width(ctx, width), 20 if width >= 128 else 3, 20 if width >= 128 else 4)
                r[str(width)] = {"TFLOP/s": round(2.0 * M ** 3 / t / 1e12, 1), "pct_mfma_peak": round(2.0 * M ** 3 / t / 1e12 / 25.0, 2),
                                 "ms": round(t * 1e3, 3)}
            ops["gemm_8192_bf16"] = r
            ops["gemm_8192_bf16"]["roofline"] = {"bound": "mfma", "achieved": r["256"]["TFLOP/s"], "peak": 2500.0, "unit": "TFLOP/s",
                                                 "frac": round(r["256"]["TFLOP/s"] / 2500.0, 4)}
            vte.vte_desc_destroy(d)
            out["per_operator"] = ops

    # ---- other batch sizes of the same chain, full width (outside the timed region) -------------
    if not a.no_width_sweep:
        with _section(out, "chain per batch"):
            per_batch = {}
            for b2 in (1, 2, 4, 16, 32, 64):
                c2 = H.DecodeChain(ctx, wd, shp, b2, feedback=True, fused_gather=True, fused_argmax=True)
                c2.set_tokens(inputs.tokens(0, inputs.T_TOK0, b2, shp.V))
                n = max(50, a.steps // 4)
                run(c2, 20, vs)
                t = time.perf_counter()
                run(c2, n, vs)
                e = time.perf_counter() - t
                gbs = c2.bytes_per_step * n / e / 1e9
                per_batch[str(b2)] = {"GB/s": round(gbs, 1), "pct_peak": round(100 * gbs / HBM_PEAK_GBS, 2),
                                      "ms_per_step": round(e / n * 1e3, 4)}
                c2.close()
            out["per_batch"] = per_batch

    out["final_tokens_checksum"] = int(tokens_end.astype(np.int64).sum())
    vte.vte_vstream_destroy(vs)
    ch.close()
    vte.vte_shutdown(ctx)      # one pool of queues at a time: more than ~22 live compute queues get time-sliced

    if not a.no_extras:
        from paper_2603_15042_amd import experiments as E
        # ---- strict binding (readiness before binding, literally): same chain, same steps -------
        with _section(out, "strict binding"):
            cfg2 = vte.vte_pool_cfg_default()
            cfg2.mode = vte.VTE_MODE_STRICT
            ctx2 = vte.vte_init(0, cfg2)
            ch2 = H.DecodeChain(ctx2, wd, shp, B, feedback=True, fused_gather=True, fused_argmax=True)
            vs2 = vte.vte_vstream_create(ctx2, vte.VTE_CLASS_LATENCY)
            n = max(100, min(a.steps, 400))
            ch2.set_tokens(tok0)
            run(ch2, 30, vs2)
            ch2.set_tokens(tok0)
            t = time.perf_counter()
            run(ch2, n, vs2)
            e = time.perf_counter() - t
            strict_tok = ch2.tok.cpu().numpy().copy()
            out["strict"] = {"ms_per_step": round(e / n * 1e3, 4), "GB/s": round(step_bytes * n / e / 1e9, 1),
                             "pct_peak": round(100 * step_bytes * n / e / 1e9 / HBM_PEAK_GBS, 2), "steps": n}
            # the same chain with the step boundary in the QKV launch's prologue (five launches per step, the
            # same bits): a loss of about 2 % under pipelined binding, where a launch boundary is free, and a
            # gain under strict binding, where each boundary is a host round trip
            if B <= 16 and shp.D == 4096:
                ch5 = H.DecodeChain(ctx2, wd, shp, B, feedback=True, fused_gather=True, fused_argmax=True, fused_qkv=True)
                ch5.set_tokens(tok0)
                run(ch5, 30, vs2)
                ch5.set_tokens(tok0)
                t = time.perf_counter()
                run(ch5, n, vs2)
                e5 = time.perf_counter() - t
                out["strict"]["five_launches_per_step"] = {
                    "ms_per_step": round(e5 / n * 1e3, 4), "GB/s": round(ch5.bytes_per_step * n / e5 / 1e9, 1),
                    "pct_peak": round(100 * ch5.bytes_per_step * n / e5 / 1e9 / HBM_PEAK_GBS, 2),
                    "tokens_equal_six_launches": bool(np.array_equal(strict_tok, ch5.tok.cpu().numpy()))}
                ch5.close()
            # the pipelined chain of the timed region, from the same tokens, after the same number of steps
            vte.vte_vstream_destroy(vs2)
            # ---- BASELINE config 1: launch latency of the 8 x 1024 RMSNorm per width -------------------
            _log("config 1 latency")
            out["config1_rmsnorm_8x1024"] = E.config1_latency(ctx2, 200)
            ch2.close()
            vte.vte_shutdown(ctx2)
            cfg3 = vte.vte_pool_cfg_default()
            cfg3.mode = vte.VTE_MODE_PIPELINED
            cfg3.lookahead = a.lookahead
            ctx3 = vte.vte_init(0, cfg3)
            ch3 = H.DecodeChain(ctx3, wd, shp, B, feedback=True, fused_gather=True, fused_argmax=True)
            vs3 = vte.vte_vstream_create(ctx3, vte.VTE_CLASS_LATENCY)
            ch3.set_tokens(tok0)
            run(ch3, 30, vs3)
            ch3.set_tokens(tok0)
            run(ch3, n, vs3)
            out["strict"]["tokens_equal_pipelined"] = bool(np.array_equal(strict_tok, ch3.tok.cpu().numpy()))
            if B <= 16 and shp.D == 4096:   # the five-launch chain under pipelined binding, beside the six-launch one
                res5 = {}
                for name, fq in (("six_launches", False), ("five_launches", True)):
                    c = ch3 if not fq else H.DecodeChain(ctx3, wd, shp, B, feedback=True, fused_gather=True, fused_argmax=True, fused_qkv=True)
                    c.set_tokens(tok0)
                    run(c, 100, vs3)
                    t = time.perf_counter()
                    run(c, n, vs3)
                    e6 = time.perf_counter() - t
                    res5[name] = {"ms_per_step": round(e6 / n * 1e3, 4), "GB/s": round(c.bytes_per_step * n / e6 / 1e9, 1)}
                    if fq:
                        c.close()
                out["boundary_in_qkv_launch_pipelined"] = res5
            vte.vte_vstream_destroy(vs3)
            ch3.close()
            vte.vte_shutdown(ctx3)

        # ---- co-tenancy (BASELINE config 4): decode bursts beside the 8192^3 GEMM -----------------
        if not a.small:
            with _section(out, "co-tenancy"):
                r = E.cotenancy(a.cotenancy_seconds, 60.0, shared=shared, modes=("fixed", "late", "late_nohint"))
                keep = ("gemm_per_s", "norm_gemm", "norm_decode", "aggregate_normalized_throughput", "bursts", "bursts_compared",
                        "bursts_with_token_mismatch", "step_ms_mean", "step_latency_ms_p50", "step_latency_ms_p99", "steps_timed",
                        "first_step_ms_mean", "gemm_widths", "decode_widths", "overlap")
                out["cotenancy"] = {
                    "seconds_per_mode": a.cotenancy_seconds, "gemm_tflops_solo": round(r["gemm_tflops_solo"], 1),
                    "solo_decode": {k: r["solo_decode"].get(k) for k in ("step_ms_mean", "step_latency_ms_p50", "step_latency_ms_p99", "bursts")},
                    "fixed_128_128": {k: r["fixed"].get(k) for k in keep},
                    "late_bound": {k: r["late"].get(k) for k in keep},                    # with a 3 ms arrival hint per burst
                    "late_bound_no_hint": {k: r["late_nohint"].get(k) for k in keep},  # the policy alone
                    "late_bound_beats_fixed_split": bool(r["late"]["aggregate_normalized_throughput"] > r["fixed"]["aggregate_normalized_throughput"]),
                }
        for k in ("gA", "gB", "gC"):
            shared.pop(k, None)
        torch.cuda.empty_cache()

        # ---- determinism protocol at a reduced trial count -----------------------------------------
        with _section(out, "determinism"):
            dres = E.determinism(a.determinism_trials, 0, sections=("rmsnorm", "gemv"))
            fixed_bits = sum(v.get("fixed_mismatched_bits", 0) + v.get("fixed_mismatched_bits_bf16", 0) + v.get("fixed_mismatched_bits_fp32", 0)
                             for v in dres.values())
            out["determinism"] = {"trials_per_operator": a.determinism_trials, "fixed_mismatched_bits": int(fixed_bits),
                                  "reshaped_trials_that_drift": {k: int(v.get("reshaped_trials_with_mismatch", v.get("reshaped_trials_with_mismatch_fp32", 0)))
                                                                 for k, v in dres.items()},
                                  "reshaped_trials_that_drift_in_bf16": {k: int(v.get("reshaped_trials_with_mismatch", v.get("reshaped_trials_with_mismatch_bf16", 0)))
                                                                         for k, v in dres.items()}}

    # ---- the oracle timed on the host cores (a baseline for scale only) -----------------------
    if not a.no_cpu_baseline:
        with _section(out, "cpu baseline"):
            import oracle
            thr = oracle.default_threads()
            t = time.perf_counter()
            tok_c, n_cpu, first = tok0, 0, None
            while True:                                   # free-running oracle decode, about 10 s of CPU work
                o = oracle.decode_step(w, tok_c, shp, threads=thr)
                first = first if first is not None else o["next"].copy()
                tok_c = o["next"]
                n_cpu += 1
                ct = time.perf_counter() - t
                if ct > 8.0 or n_cpu >= 64:
                    break
            cpu = {"value": round(step_bytes * n_cpu / ct / 1e9, 3), "unit": "GB/s", "cores": thr, "kind": "oracle",
                   "sample": "%d free-running decode steps at batch %d (whole chain, double precision), %.1f s" % (n_cpu, B, ct),
                   "hardware_threads": oracle.hardware_threads()}

            def timed(fn, reps=1):
                tb = time.perf_counter()
                for _ in range(reps):
                    fn()
                return (time.perf_counter() - tb) / reps
            t1c = timed(lambda: oracle.decode_step(w, tok0, shp, threads=1))
            cpu["one_core"] = {"value": round(step_bytes / t1c / 1e9, 4), "unit": "GB/s", "sample": "1 decode step at batch %d, %.1f s" % (B, t1c)}
            if not a.small:
                per_op = {}
                x8, g8 = inputs.rmsnorm_case(seed=0, rows=8, cols=1024)
                per_op["rmsnorm_8x1024_us"] = round(timed(lambda: oracle.rmsnorm(x8, g8, threads=thr), 20) * 1e6, 1)
                xs = inputs.normal_bf16(0, inputs.T_X, (2048, 4096))
                per_op["rmsnorm_2048x4096_ms (a 1/16 sample of 32768x4096)"] = round(timed(lambda: oracle.rmsnorm(xs, w["gamma"], threads=thr)) * 1e3, 2)
                Wc, _ = inputs.gemv_case(seed=0, B=1, N=4096, K=4096)
                for b2 in (1, 4, 8):
                    Xc = inputs.normal_bf16(0, inputs.T_XB, (b2, 4096))
                    per_op["gemv_4096x4096_B%d_ms" % b2] = round(timed(lambda: oracle.gemv(Wc, Xc, threads=thr), 3) * 1e3, 2)
                for b2 in (1, 16):
                    tb2 = inputs.tokens(0, inputs.T_TOK0, b2, shp.V)
                    per_op["decode_step_B%d_ms" % b2] = round(timed(lambda: oracle.decode_step(w, tb2, shp, threads=thr)) * 1e3, 1)
                per_op["decode_step_B%d_ms" % B] = round(ct / n_cpu * 1e3, 1)
                Ag = inputs.normal_bf16(0, inputs.T_GEMM_A, (1024, 1024))
                Bg = inputs.normal_bf16(0, inputs.T_GEMM_B, (1024, 1024))
                per_op["gemm_1024^3_ms"] = round(timed(lambda: oracle.gemm_rows(Ag, Bg, np.arange(1024), threads=thr)) * 1e3, 1)
                cpu["per_operator_all_cores"] = per_op
            out["cpu_baseline"] = cpu
            # the GPU chain from the same start tokens must pick the oracle's tokens, at every batch the sweep timed
            ctx4 = vte.vte_init(0, cfg)
            vs4 = vte.vte_vstream_create(ctx4, vte.VTE_CLASS_LATENCY)
            match = {}
            for b2 in ((1, 2, 4, 8, 16) if not a.small else (B,)):
                c4 = H.DecodeChain(ctx4, wd, shp, b2, feedback=True, fused_gather=True, fused_argmax=True)
                tb2 = inputs.tokens(0, inputs.T_TOK0, b2, shp.V)
                c4.set_tokens(tb2)
                run(c4, 1, vs4)
                ref = first if b2 == B else oracle.decode_step(w, tb2, shp, threads=thr)["next"]
                match[str(b2)] = bool(np.array_equal(c4.tok.cpu().numpy(), ref))
                c4.close()
            vte.vte_vstream_destroy(vs4)
            vte.vte_shutdown(ctx4)
            out["first_step_tokens_match_oracle"] = match[str(B)]
            out["first_step_tokens_match_oracle_per_batch"] = match
    out["gen_seconds"] = round(gen_s, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
