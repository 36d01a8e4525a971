"""Benchmark of the decode hot path on one MI355X.

A step is one pass of the Llama-8B-shaped decode chain at batch 8 (greedy-token
finish + embedding gather + RMSNorm in one launch, QKV, O, gate/up+SiLU, down,
LM head: six immutable descriptors per step submitted to a virtual stream and
late-bound by the dispatcher), on synthetic weights resident in HBM.  Prints
one JSON line.  Outside the timed region it also times the single operators of
the metric (RMSNorm, GEMV) on pCtxs of every width.
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


def _counter_traffic():
    """HBM bytes per LM-head launch from the committed rocprofv3 counter summary (None if absent)."""
    path = os.path.join(ROOT, "profiles", "decode_chain_b8_hbm_counters.txt")
    try:
        for line in open(path):
            if line.startswith("lmhead_traffic_bytes_per_launch="):
                return int(line.split("=")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--mode", choices=("pipelined", "strict"), default="pipelined")
    ap.add_argument("--lookahead", type=int, default=64, help="launches bound ahead of the oldest unfinished one (pipelined binding)")
    ap.add_argument("--timing-stride", type=int, default=8,
                    help="time every n-th LM-head launch of the run (1 = each; a timed launch idles its stream for a few us)")
    ap.add_argument("--no-kernel-timing", action="store_true", help="do not bracket the LM head with device events")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-width-sweep", action="store_true")
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

    cfg = vte.vte_pool_cfg_default()
    cfg.mode = vte.VTE_MODE_PIPELINED if a.mode == "pipelined" else vte.VTE_MODE_STRICT
    cfg.lookahead = a.lookahead
    cfg.device_timing_mask = 0 if a.no_kernel_timing else 1 << vte.VTE_K_LMHEAD
    cfg.device_timing_stride = a.timing_stride
    torch.zeros(1, device="cuda")
    ctx = vte.vte_init(0, cfg)
    wd = H.upload_weights(w)
    ch = H.DecodeChain(ctx, wd, shp, B, feedback=True, fused_gather=True, fused_argmax=True)
    vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)

    def run(steps, vstream):
        ch.submit_burst(vstream, steps)
        vte.vte_vstream_sync(vstream)

    ch.set_tokens(tok0)
    run(a.warmup, vs)
    vte.vte_device_sync(ctx)
    torch.cuda.synchronize()
    vte.vte_stats_reset(ctx)
    t1 = time.perf_counter()
    run(a.steps, vs)
    vte.vte_device_sync(ctx)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    recs = vte.vte_stats_read(ctx)
    st = vte.vte_stats(ctx)
    lm = [r.gpu_seconds for r in recs if r.kernel == vte.VTE_K_LMHEAD and r.gpu_seconds > 0]
    lm_bytes = vte.vte_desc_info(ch.desc["lmhead"]).bytes
    lm_avg = float(np.mean(lm)) if lm else float("nan")
    step_bytes = ch.bytes_per_step
    value = step_bytes * a.steps / dt / 1e9
    tokens_end = ch.tok.cpu().numpy().copy()
    if a.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.int8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {
        "metric": "GEMV/RMSNorm HBM GB/s (% peak) per CU width; bit mismatches across widths (=0)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(dt / a.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
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
                     "avg_kernel_us": round(lm_avg * 1e6, 2), "launches_timed": len(lm), "timing_stride": a.timing_stride, "traffic": _counter_traffic(),
                     "algorithmic_bytes_per_launch": int(lm_bytes)},
    }

    # ---- per CU width: throughput and bit mismatches (outside the timed region) -------------
    if not a.no_width_sweep:
        per_width, mism = {}, 0
        ref_snap = None
        for width in (256, 128, 64, 32):
            p = H.pctx_of_width(ctx, width)
            v = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
            vte.vte_vstream_pin(v, p)
            ch.set_tokens(tok0)
            n = max(8, a.steps // 8)
            run(4, v)
            ch.set_tokens(tok0)
            t = time.perf_counter()
            run(n, v)
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
                                     "ms_per_step": round(e / n * 1e3, 4)}
            vte.vte_vstream_destroy(v)
        out["per_width"] = per_width
        out["bit_mismatches_across_widths"] = int(mism)

    # ---- the metric's single operators per CU width (outside the timed region) ----
    if not a.no_width_sweep and not a.small:
        ops = {}
        rows, cols = 32768, 4096                       # RMSNorm at a size HBM has to serve: 256 MiB in, 256 MiB out
        x = torch.randint(-3000, 3000, (rows, cols), dtype=torch.int16, device="cuda")
        y = torch.empty_like(x)
        d = vte.vte_desc_rmsnorm(ctx, x, wd["gamma"], y, rows, cols, 1e-6)
        r = {}
        for width in (256, 128, 64, 32):
            t = vte.vte_profile_measure_on(ctx, d, H.pctx_of_width(ctx, width), 2, 6)
            r[str(width)] = {"GB/s": round(rows * cols * 4 / t / 1e9, 1), "pct_peak": round(rows * cols * 4 / t / 1e9 / 80, 2)}
        ops["rmsnorm_32768x4096"] = r
        vte.vte_desc_destroy(d)
        del x, y
        N = K = 4096                                   # GEMV 4096x4096, 32 weight buffers in rotation (1 GiB > caches)
        Ws = [torch.randint(-3000, 3000, (N, K), dtype=torch.int16, device="cuda") for _ in range(32)]
        for b2 in (1, 4, 8):
            X = torch.randint(-3000, 3000, (b2, K), dtype=torch.int16, device="cuda")
            Y = torch.empty((b2, N), dtype=torch.int16, device="cuda")
            ds = [vte.vte_desc_gemv(ctx, W_, X, Y, b2, N, K) for W_ in Ws]
            r = {}
            for width in (256, 128, 64, 32):
                # 128 launches back to back on a virtual stream pinned to the pCtx, each on the next weight
                # buffer; wall time per launch (a single launch between two events would add their cost)
                v = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
                vte.vte_vstream_pin(v, H.pctx_of_width(ctx, width))
                vte.vte_token_wait(ctx, vte.vte_submit_batch(v, vte.desc_array(ds)))
                burst = vte.desc_array(ds * 4)
                t0 = time.perf_counter()
                vte.vte_token_wait(ctx, vte.vte_submit_batch(v, burst))
                t = (time.perf_counter() - t0) / (4 * len(ds))
                vte.vte_vstream_destroy(v)
                r[str(width)] = {"GB/s": round(N * K * 2 / t / 1e9, 1), "pct_peak": round(N * K * 2 / t / 1e9 / 80, 2),
                                 "us": round(t * 1e6, 2)}
            ops["gemv_4096x4096_B%d" % b2] = r
            for dd in ds:
                vte.vte_desc_destroy(dd)
        del Ws
        torch.cuda.empty_cache()
        M = 8192                                       # the co-tenant: bf16 MFMA GEMM 8192^3, N(0,1) inputs
        gA = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, M)))
        gB = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (M, M)))
        gC = H.dev_empty((M, M))
        d = vte.vte_desc_gemm(ctx, gA, gB, gC, M, M, M)
        r = {}
        for width in (256, 128, 64, 32):
            t = vte.vte_profile_measure_on(ctx, d, H.pctx_of_width(ctx, width), 1, 4 if width >= 128 else 2)
            r[str(width)] = {"TFLOP/s": round(2.0 * M ** 3 / t / 1e12, 1), "pct_mfma_peak": round(2.0 * M ** 3 / t / 1e12 / 25.0, 2),
                             "ms": round(t * 1e3, 3)}
        ops["gemm_8192_bf16"] = r
        ops["gemm_8192_bf16"]["roofline"] = {"bound": "mfma", "achieved": r["256"]["TFLOP/s"], "peak": 2500.0, "unit": "TFLOP/s",
                                             "frac": round(r["256"]["TFLOP/s"] / 2500.0, 4)}
        vte.vte_desc_destroy(d)
        del gA, gB, gC
        torch.cuda.empty_cache()
        out["per_operator"] = ops

    # ---- other batch sizes of the same chain, full width (outside the timed region) -------------
    if not a.no_width_sweep:
        per_batch = {}
        for b2 in (1, 4, 16, 32, 64):
            c2 = H.DecodeChain(ctx, wd, shp, b2, feedback=True, fused_gather=True, fused_argmax=True)
            c2.set_tokens(inputs.tokens(0, inputs.T_TOK0, b2, shp.V))
            n = max(50, a.steps // 4)
            c2.submit_burst(vs, 20)
            vte.vte_vstream_sync(vs)
            t = time.perf_counter()
            c2.submit_burst(vs, n)
            vte.vte_vstream_sync(vs)
            e = time.perf_counter() - t
            gbs = c2.bytes_per_step * n / e / 1e9
            per_batch[str(b2)] = {"GB/s": round(gbs, 1), "pct_peak": round(100 * gbs / HBM_PEAK_GBS, 2),
                                  "ms_per_step": round(e / n * 1e3, 4)}
            c2.close()
        out["per_batch"] = per_batch

    # ---- the oracle timed on the host cores (a baseline for scale only) -----------------------
    if not a.no_cpu_baseline:
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
            if ct > 10.0 or n_cpu >= 64:
                break
        out["cpu_baseline"] = {"value": round(step_bytes * n_cpu / ct / 1e9, 3), "unit": "GB/s", "cores": thr,
                               "kind": "oracle",
                               "sample": "%d free-running decode steps at batch %d (whole chain, double precision), "
                                         "%.1f s" % (n_cpu, B, ct)}
        # the GPU chain from the same start tokens must pick the oracle's tokens
        ch.set_tokens(tok0)
        run(1, vs)
        out["first_step_tokens_match_oracle"] = bool(np.array_equal(ch.tok.cpu().numpy(), first))
    out["gen_seconds"] = round(gen_s, 1)
    out["final_tokens_checksum"] = int(tokens_end.astype(np.int64).sum())
    vte.vte_vstream_destroy(vs)
    ch.close()
    vte.vte_shutdown(ctx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
