"""Serving-trace sweep: Poisson decode arrivals on the layered decode chain, co-located
with the training-shaped GEMM, under the policies of Sec. 5 (Sec. 7.3 / 7.4 of the paper use
production traces; this is a seeded synthetic stand-in with the stated distributions).

    python -m paper_2603_15042_amd.serving --rates 5,10,20,40,80 --seconds 20 --layers 32

Requests arrive by a Poisson process, carry a prompt length (it only sizes the host-to-device copy
that precedes the first decode step), an output length and a start token.  Up to 64 run at once,
in chunks of 16 rows (four of them; or two of 32 with --chunk 32, one of 64 with --chunk 64: the
weights are read once per launch whatever its rows), each stepping its own copy of the chain's activations over shared weights; the chunks are
dealt to two virtual streams and take turns on theirs.  Five tenants would be one too many:
the device dispatches from four pipes and queues on one pipe run one kernel at a time, so the sweep
keeps to two decode streams and the co-tenant.  Every launch is built at the chunk size, so a row's arithmetic does not
depend on what shares the launch, and a request's token stream is a function of its start token
alone: every observed transition token -> next token is checked against the same row computed alone
on the full-width pCtx with nothing else running.

Nothing here computes any part of the method; it moves tokens, submits descriptors and reads clocks.
"""
import argparse
import json
import time

import numpy as np
import torch

from . import harness as H, inputs, vte

MAX_ROWS, STREAMS = 64, 2   # at most 64 requests at once, in chunks of 16 (or 32) rows on two virtual streams
WIDTHS = (32, 64, 128, 192, 224, 256)


def make_trace(seed, rate, seconds, vocab):
    """Seeded request list: arrival (s), prompt length, output length, start token."""
    rng = np.random.RandomState(seed)
    t, out = 0.0, []
    while True:
        t += rng.exponential(1.0 / rate)
        if t >= seconds:
            return out
        out.append({"arrival": t, "prompt": int(rng.randint(128, 2049)), "out_len": int(rng.randint(64, 513)),
                    "tok0": int(rng.randint(0, vocab))})


def layer_weights(seed, shp, layers):
    """Distinct weights per layer (same recipe, another seed); one embedding and LM head."""
    head = inputs.decode_weights(seed, shp)
    first = {k: head.pop(k) for k in ("gamma", "Wqkv", "Wo", "Wgu", "Wd")}
    out = [H.upload_weights(first)]
    for l in range(1, layers):
        w = inputs.decode_weights(seed + 1000 * l, shp, with_embedding=False)
        w.pop("Wlm")
        out.append(H.upload_weights(w))
    return out, H.upload_weights(head)


class Server:
    def __init__(self, layers, small=False, lookahead=32, chunk=16):
        assert chunk in (16, 32, 64)
        self.chunk, self.nchunks = chunk, MAX_ROWS // chunk
        self.nstreams = min(STREAMS, self.nchunks)
        self.shp = inputs.DecodeShapes(D=512, Nqkv=768, F=1792, V=4099) if small else inputs.DecodeShapes()
        cfg = vte.vte_pool_cfg_default()
        cfg.mode = vte.VTE_MODE_PIPELINED
        cfg.lookahead = lookahead
        torch.zeros(1, device="cuda")
        self.ctx = ctx = vte.vte_init(0, cfg)
        t0 = time.time()
        self.layers, self.head = layer_weights(0, self.shp, layers)
        self.gen_seconds = time.time() - t0
        self.chains = [H.LayeredDecode(ctx, self.layers, self.head, self.shp, chunk) for _ in range(self.nchunks)]
        M = 1024 if small else 8192
        self.M = M
        gA = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, M)))
        gB = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (M, M)))
        self.gbuf = (gA, gB, H.dev_empty((M, M)))
        self.gemm = vte.vte_desc_gemm(ctx, gA, gB, self.gbuf[2], M, M, M)
        self.vs = [vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY) for _ in range(self.nstreams)]
        self.be = vte.vte_vstream_create(ctx, vte.VTE_CLASS_BEST_EFFORT)
        self.root = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 256)
        # torch work in the serving loop stays off the null stream, which would order itself against
        # every CU-masked stream: token reads and writes go through a non-blocking stream of their own
        self.io_stream = torch.cuda.Stream()
        self.pin_tok = [torch.zeros(chunk, dtype=torch.int32).pin_memory() for _ in range(self.nchunks)]
        self.copy_stream = torch.cuda.Stream()
        self.stage = torch.empty(MAX_ROWS * 2048, dtype=torch.int32, device="cuda")
        self.pinned = torch.zeros(2048, dtype=torch.int32).pin_memory()
        self.next_of = {}      # token -> next token, computed alone at full width
        self.profiles = {}
        for d in self.chains[0].distinct_descs() + [self.gemm]:
            vte.vte_profile_measure(ctx, d, 2, 5)
            v = vte.vte_desc_info(d)
            self.profiles["k%d_%x" % (v.kernel, v.profile_key & 0xffff)] = {
                w: round(vte.vte_profile_get(ctx, v.profile_key, w) * 1e6, 1) for w in WIDTHS}

    def close(self):
        vte.vte_device_sync(self.ctx)
        vte.vte_shutdown(self.ctx)

    def read_tokens(self, c):
        """Chunk c's token buffer -> its pinned host image (the chunk must have no step in flight)."""
        with torch.cuda.stream(self.io_stream):
            self.pin_tok[c].copy_(self.chains[c].tok, non_blocking=True)
        self.io_stream.synchronize()
        return self.pin_tok[c].numpy()

    def write_tokens(self, c, toks=None):
        if toks is not None:
            self.pin_tok[c].numpy()[:] = toks
        with torch.cuda.stream(self.io_stream):
            self.chains[c].tok.copy_(self.pin_tok[c], non_blocking=True)
        self.io_stream.synchronize()

    # -- the reference: each token's successor, the row computed alone at full width --------------
    def reference_next(self, toks):
        todo = sorted({int(t) for t in toks} - set(self.next_of))
        ch, vs = self.chains[0], self.vs[0]
        vte.vte_device_sync(self.ctx)
        vte.vte_set_builtin_policy(self.ctx, vte.VTE_POLICY_WIDEST)
        vte.vte_vstream_pin(vs, self.root)
        CHUNK = self.chunk
        for i in range(0, len(todo), CHUNK):
            part = todo[i:i + CHUNK]
            buf = np.zeros(CHUNK, dtype=np.int32)
            buf[:len(part)] = part
            self.write_tokens(0, buf)
            vte.vte_token_wait(self.ctx, ch.submit_step(vs))
            nxt = self.read_tokens(0).copy()
            for t, n in zip(part, nxt):
                self.next_of[t] = int(n)
        vte.vte_vstream_pin(vs, -1)

    # -- one run of a trace under a policy ---------------------------------------------------------
    def run(self, trace, seconds, mode, tpot_target=0.050, with_gemm=True):
        """mode: 'solo' (no co-tenant, widest) | 'fixed' (decode streams pinned to the quarters of one half, GEMM to the other half)
        | 'tput' (Throughput-Oriented plan) | 'tpot' (TPOT-First).  Chunk c runs on stream c % (number of streams)."""
        ctx = self.ctx
        CHUNK, MAX_CHUNKS = self.chunk, self.nchunks
        vte.vte_device_sync(ctx)
        vte.vte_stats_reset(ctx)
        # fixed split: the decode streams share one half (its quarters; the whole half when there is one stream)
        quarters = ([vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 64, i) for i in range(STREAMS)] if self.nstreams > 1
                    else [vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 0)])
        half1 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 1)
        per_stream = MAX_CHUNKS // self.nstreams
        for i, vs in enumerate(self.vs):
            # a stream's "token" is one chunk step; its chunks alternate, so a request sees per_stream of them per token
            vte.vte_vstream_set_tpot(vs, tpot_target / per_stream if mode == "tpot" else 0.0, self.chains[i].ops_per_step)
            vte.vte_vstream_pin(vs, quarters[i] if mode == "fixed" else -1)
        vte.vte_vstream_pin(self.be, half1 if mode == "fixed" else -1)
        policy = {"solo": vte.VTE_POLICY_WIDEST, "fixed": vte.VTE_POLICY_WIDEST, "tput": vte.VTE_POLICY_TPUT_PLAN,
                  "tpot": vte.VTE_POLICY_TPOT_FIRST}[mode]
        vte.vte_set_builtin_policy(ctx, policy, 0.25, 0)
        with_gemm = with_gemm and mode != "solo"

        reqs = [dict(r, tokens=[], times=[], t_admit=None) for r in trace]
        pending, nxt_arrival = [], 0
        slots = [[-1] * CHUNK for _ in range(MAX_CHUNKS)]
        tail = [0] * MAX_CHUNKS
        busy = [False] * MAX_CHUNKS
        gemm_q, gemm_done, steps = [], 0, 0
        t0 = time.perf_counter()
        while True:
            now = time.perf_counter() - t0
            if now >= seconds and not any(busy):
                break
            while nxt_arrival < len(reqs) and reqs[nxt_arrival]["arrival"] <= now:
                r = reqs[nxt_arrival]
                # the prompt's host-to-device copy: the only thing the prompt length decides here
                with torch.cuda.stream(self.copy_stream):
                    self.stage[:r["prompt"]].copy_(self.pinned[:r["prompt"]], non_blocking=True)
                    r["copied"] = torch.cuda.Event()
                    r["copied"].record()
                pending.append(nxt_arrival)
                nxt_arrival += 1
            if with_gemm:
                while gemm_q and vte.vte_token_query(ctx, gemm_q[0]):
                    gemm_q.pop(0)
                    gemm_done += 1
                while len(gemm_q) < 2 and now < seconds:
                    gemm_q.append(vte.vte_submit(self.be, self.gemm))
            for c in range(MAX_CHUNKS):
                ch = self.chains[c]
                if busy[c]:
                    if not vte.vte_token_query(ctx, tail[c]):
                        continue
                    t_done = time.perf_counter() - t0
                    toks = self.read_tokens(c)
                    for s, ri in enumerate(slots[c]):
                        if ri < 0:
                            continue
                        r = reqs[ri]
                        r["tokens"].append(int(toks[s]))
                        r["times"].append(t_done)
                        if len(r["tokens"]) >= r["out_len"]:
                            slots[c][s] = -1
                    busy[c] = False
                    steps += 1
                if now >= seconds:
                    continue
                new = False
                # fill the lowest chunks first: a chunk admits only while every chunk before it is full
                lower_full = all(ri >= 0 for k in range(c) for ri in slots[k])
                for s in range(CHUNK):
                    if lower_full and slots[c][s] < 0 and pending and reqs[pending[0]]["copied"].query():
                        ri = pending.pop(0)
                        slots[c][s] = ri
                        reqs[ri]["t_admit"] = now
                        self.pin_tok[c].numpy()[s] = reqs[ri]["tok0"]   # the host image holds the step's tokens
                        new = True
                if new:
                    self.write_tokens(c)
                if any(ri >= 0 for ri in slots[c]):
                    tail[c] = ch.submit_step(self.vs[c % self.nstreams])
                    busy[c] = True
            time.sleep(0.00005)
        elapsed = time.perf_counter() - t0
        for t in gemm_q:
            vte.vte_token_wait(ctx, t)
            gemm_done += 1
        vte.vte_device_sync(ctx)
        t_all = time.perf_counter() - t0
        recs = vte.vte_stats_read(ctx)
        info = [vte.vte_vstream_tpot_info(vs) for vs in self.vs]
        for vs in self.vs:
            vte.vte_vstream_set_tpot(vs, 0.0, 0)
        gaps = np.array([b - a for r in reqs for a, b in zip(r["times"], r["times"][1:])])
        first = np.array([r["times"][0] - r["arrival"] for r in reqs if r["times"]])
        req_tpot = np.array([(r["times"][-1] - r["times"][0]) / (len(r["times"]) - 1) for r in reqs if len(r["times"]) > 1])
        dw = [r.width for r in recs if r.klass == vte.VTE_CLASS_LATENCY]
        gw = [r.width for r in recs if r.klass == vte.VTE_CLASS_BEST_EFFORT]
        pct = lambda a, q: float(np.percentile(a, q) * 1e3) if len(a) else None
        return {
            "mode": mode, "elapsed_s": elapsed, "requests": len(reqs), "requests_started": int(len(first)),
            "requests_finished": sum(1 for r in reqs if len(r["tokens"]) >= r["out_len"]),
            "tokens": int(sum(len(r["tokens"]) for r in reqs)), "chunk_steps": steps,
            "tokens_per_s": float(sum(len(r["tokens"]) for r in reqs) / elapsed),
            "tpot_ms_p50": pct(gaps, 50), "tpot_ms_p99": pct(gaps, 99), "tpot_ms_max": pct(gaps, 100),
            "slo_ms": tpot_target * 1e3,
            "slo_violation_rate_tokens": float((gaps > tpot_target).mean()) if len(gaps) else None,
            "slo_violation_rate_requests": float((req_tpot > tpot_target).mean()) if len(req_tpot) else None,
            "first_token_ms_p50": pct(first, 50), "first_token_ms_p99": pct(first, 99),
            "gemm_per_s": gemm_done / t_all if with_gemm else 0.0,
            "gemm_tflops": 2.0 * self.M ** 3 * gemm_done / t_all / 1e12 if with_gemm else 0.0,
            "decode_widths": {str(k): int(v) for k, v in zip(*np.unique(dw, return_counts=True))} if dw else {},
            "gemm_widths": {str(k): int(v) for k, v in zip(*np.unique(gw, return_counts=True))} if gw else {},
            "tpot_first": [{"standing_width": vte.vte_pool_info(ctx, i.standing_pctx).width if i.standing_pctx >= 0 else None,
                            "tokens": int(i.tokens_done), "deadline_misses": int(i.deadline_misses),
                            "escalations": int(i.escalations)} for i in info] if mode == "tpot" else None,
            "timeline": self.timeline(recs, ctx),
            "_reqs": reqs,
        }

    @staticmethod
    def timeline(recs, ctx):
        """Where the launches of each virtual stream spent their time, from the op-record ring (the most
        recent records of the run): per stream the share of its window with nothing in flight, the time
        its ready launches waited for a pCtx (ready -> bound), the width its launches ran on weighted
        by their time in flight, and per pCtx the time it was held (bound -> done, union over launches)."""
        if not recs:
            return None
        out = {"records": len(recs), "streams": {}, "pctx": {}}
        by_vs, by_p = {}, {}
        for r in recs:
            by_vs.setdefault((r.vstream, r.klass), []).append(r)
            by_p.setdefault(r.pctx, []).append(r)
        t_lo, t_hi = min(r.t_submit for r in recs), max(r.t_done for r in recs)

        def union(iv):
            tot, end = 0.0, -1.0
            for a, b in sorted(iv):
                if b <= end:
                    continue
                tot += b - max(a, end)
                end = b
            return tot
        for (vs, klass), rs in sorted(by_vs.items()):
            lo, hi = min(r.t_submit for r in rs), max(r.t_done for r in rs)
            fl = sum(r.t_done - r.t_bound for r in rs)
            w = {}
            for r in rs:
                w[r.width] = w.get(r.width, 0.0) + (r.t_done - r.t_bound)
            out["streams"]["%d (%s)" % (vs, "latency" if klass == vte.VTE_CLASS_LATENCY else "best effort")] = {
                "launches": len(rs), "window_ms": round((hi - lo) * 1e3, 2),
                "share_of_window_with_a_launch_in_flight": round(union([(r.t_bound, r.t_done) for r in rs]) / max(hi - lo, 1e-9), 3),
                "ready_to_bound_wait_ms_total": round(sum(r.t_bound - r.t_ready for r in rs) * 1e3, 2),
                "ready_to_bound_wait_us_mean": round(float(np.mean([r.t_bound - r.t_ready for r in rs])) * 1e6, 2),
                "ready_to_bound_wait_us_p99": round(float(np.percentile([r.t_bound - r.t_ready for r in rs], 99)) * 1e6, 2),
                "time_in_flight_by_width_share": {str(k): round(v / fl, 3) for k, v in sorted(w.items())},
                "mean_width_weighted_by_time_in_flight": round(sum(k * v for k, v in w.items()) / fl, 1)}
        for p, rs in sorted(by_p.items()):
            out["pctx"]["%d (%d CUs)" % (p, vte.vte_pool_info(ctx, p).width)] = {
                "launches": len(rs), "held_share_of_run_window": round(union([(r.t_bound, r.t_done) for r in rs]) / max(t_hi - t_lo, 1e-9), 3),
                "streams": sorted({r.vstream for r in rs})}
        return out

    def check_tokens(self, result):
        """Every transition a run produced against the row computed alone at full width."""
        reqs = result.pop("_reqs")
        seen = set()
        for r in reqs:
            seq = [r["tok0"]] + r["tokens"]
            seen.update(seq[:-1])
        self.reference_next(seen)
        bad = total = 0
        for r in reqs:
            seq = [r["tok0"]] + r["tokens"]
            for a, b in zip(seq, seq[1:]):
                total += 1
                bad += int(self.next_of[a] != b)
        result["transitions_checked"] = total
        result["token_mismatches_vs_solo_full_width"] = bad
        result["distinct_tokens_seen"] = len(seen)
        return result


def sweep(rates, seconds, layers, small=False, modes=("fixed", "tput", "tpot"), seed=0, chunk=16):
    srv = Server(layers, small=small, chunk=chunk)
    out = {"layers": layers, "chunk_rows": chunk, "seconds_per_rate": seconds, "seed": seed, "slo_ms": 50.0, "gen_seconds": srv.gen_seconds,
           "ops_per_step": srv.chains[0].ops_per_step, "bytes_per_step": srv.chains[0].bytes_per_step,
           "profiles_us": srv.profiles, "rates": {}}
    try:
        # the co-tenant alone: normalises its throughput
        t = time.perf_counter()
        n = 0
        vte.vte_set_builtin_policy(srv.ctx, vte.VTE_POLICY_WIDEST)
        while time.perf_counter() - t < 1.0:
            vte.vte_token_wait(srv.ctx, vte.vte_submit(srv.be, srv.gemm))
            n += 1
        out["gemm_solo_per_s"] = n / (time.perf_counter() - t)
        for rate in rates:
            trace = make_trace(seed + int(rate * 1000), rate, seconds, srv.shp.V)
            res = {}
            for mode in ("solo",) + tuple(modes):
                r = srv.check_tokens(srv.run(trace, seconds, mode))
                r["gemm_normalized"] = r["gemm_per_s"] / out["gemm_solo_per_s"]
                res[mode] = r
                print("rate %g %s: tokens/s %.0f tpot p50 %.2f p99 %.2f ms viol %.4f gemm %.2f mism %d widths %s" % (
                    rate, mode, r["tokens_per_s"], r["tpot_ms_p50"] or -1, r["tpot_ms_p99"] or -1,
                    r["slo_violation_rate_tokens"] or 0, r["gemm_normalized"], r["token_mismatches_vs_solo_full_width"],
                    r["decode_widths"]), flush=True)
            out["rates"][str(rate)] = res
    finally:
        srv.close()
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--rates", default="5,10,20,40,80")
    ap.add_argument("--seconds", type=float, default=20.0)
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--small", action="store_true")
    ap.add_argument("--modes", default="fixed,tput,tpot")
    ap.add_argument("--chunk", type=int, default=16, help="rows per launch: 16, 32 or 64")
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    res = sweep([float(x) for x in a.rates.split(",")], a.seconds, a.layers, a.small, tuple(a.modes.split(",")), chunk=a.chunk)
    text = json.dumps(res)
    if a.out:
        with open(a.out, "w") as f:
            f.write(text)
    print(text)


if __name__ == "__main__":
    main()
