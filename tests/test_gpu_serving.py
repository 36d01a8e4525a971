"""Serving sweep at toy size on the GPU: every policy produces the token streams of the solo
full-width run, and a row's result does not depend on what shares its launch."""
import numpy as np
import pytest
import torch

from paper_2603_15042_amd import harness as H, serving, vte

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("chunk", [16, 32, 64])
def test_row_result_is_independent_of_batch_neighbours_and_position(chunk):
    srv = serving.Server(layers=2, small=True, chunk=chunk)
    try:
        rng = np.random.RandomState(3)
        toks = rng.randint(0, srv.shp.V, size=40)
        srv.reference_next(toks)                     # rows grouped 16 at a time in sorted order
        first = dict(srv.next_of)
        srv.next_of.clear()
        for t in toks[::-1]:                         # one row at a time, position 0, neighbours all token 0
            srv.reference_next([t])
        assert srv.next_of == first
    finally:
        srv.close()


@pytest.mark.parametrize("chunk", [16, 32, 64])
def test_serving_policies_reproduce_solo_tokens(chunk):
    out = serving.sweep([60.0], 1.0, layers=2, small=True, modes=("fixed", "tput", "tpot"), chunk=chunk)
    res = out["rates"]["60.0"]
    for mode in ("solo", "fixed", "tput", "tpot"):
        r = res[mode]
        assert r["tokens"] > 0 and r["transitions_checked"] == r["tokens"]
        assert r["token_mismatches_vs_solo_full_width"] == 0, mode
    assert res["tpot"]["tpot_first"][0]["standing_width"] is not None
    assert res["fixed"]["gemm_per_s"] > 0 and res["tput"]["gemm_per_s"] > 0


def test_tpot_first_prepare_escalates_on_the_gpu():
    """TPOT-First's at-risk path on real CU-masked streams (Sec. 5 "TPOT-First", Sec. 4.3 reservation
    and reclamation).  The injected profiles promise that a 32-CU pCtx meets the target with room to
    spare, so the standing pCtx is a leaf; the chain really takes about twice the promised time there
    and a GEMM tenant holds the rest of the device.  The observed slowdown makes the next token's
    predicted completion miss its deadline: Prepare closes the gate of the overlapping best-effort
    lease, reserves the smallest wider pCtx predicted to meet the deadline, and the decode moves
    there -- with every token equal to the run alone on the whole device."""
    import time
    from paper_2603_15042_amd import inputs
    shp = inputs.DecodeShapes(D=1024, Nqkv=1536, F=3584, V=8200)
    w = inputs.decode_weights(5, shp)
    for k in ("Wqkv", "Wo", "Wgu", "Wd"):
        w[k] = inputs.normal_bf16(5, 100 + len(k), w[k].shape, 0.0, 1.5 * w[k].shape[1] ** -0.5)
    B, steps = 8, 300
    tok0 = inputs.tokens(5, inputs.T_TOK0, B, shp.V)
    ctx = H.make_ctx(vte.VTE_MODE_PIPELINED, lookahead=16)
    try:
        wd = H.upload_weights(w)
        ch = H.DecodeChain(ctx, wd, shp, B, feedback=True)
        per_token = len(ch.order)

        def decode(vs, n):
            toks = []
            for s in range(n):
                toks.append(ch.submit_step(vs))
                if s >= 2:
                    vte.vte_token_wait(ctx, toks[s - 2])        # two tokens in flight, like a serving loop
            vte.vte_vstream_sync(vs)

        # alone on the whole device: the reference tokens
        solo = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
        vte.vte_vstream_pin(solo, H.pctx_of_width(ctx, 256))
        ch.set_tokens(tok0)
        decode(solo, steps)
        ref = ch.tok.cpu().numpy().copy()
        # what a token really takes on a 32-CU leaf
        vte.vte_vstream_pin(solo, H.pctx_of_width(ctx, 32))
        ch.set_tokens(tok0)
        decode(solo, 20)
        t0 = time.perf_counter()
        decode(solo, 100)
        t_real32 = (time.perf_counter() - t0) / 100
        vte.vte_vstream_destroy(solo)
        # profiles that promise half of that at 32 CUs and perfect scaling above
        for k in ch.order:
            key = vte.vte_desc_info(ch.desc[k]).profile_key
            for width in (32, 64, 128, 192, 224, 256):
                vte.vte_profile_set(ctx, key, width, 0.5 * t_real32 / per_token * 32.0 / width)
        M = 4096
        A = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, M)))
        Bm = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (M, M)))
        Cm = H.dev_empty((M, M))
        g = vte.vte_desc_gemm(ctx, A, Bm, Cm, M, M, M)
        vte.vte_set_builtin_policy(ctx, vte.VTE_POLICY_TPOT_FIRST, 0.1, 0)
        lat = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
        be = vte.vte_vstream_create(ctx, vte.VTE_CLASS_BEST_EFFORT)
        vte.vte_vstream_set_tpot(lat, 0.8 * t_real32, per_token)      # the leaf cannot really meet this
        vte.vte_device_sync(ctx)
        vte.vte_stats_reset(ctx)
        ch.set_tokens(tok0)
        gq, toks, seen_standing, seen_escalated = [], [], set(), set()
        for s in range(steps):
            while len(gq) < 2:
                gq.append(vte.vte_submit(be, g))
            if vte.vte_token_query(ctx, gq[0]):
                gq.pop(0)
            toks.append(ch.submit_step(lat))
            if s >= 2:
                vte.vte_token_wait(ctx, toks[s - 2])
            info = vte.vte_vstream_tpot_info(lat)
            if info.standing_pctx >= 0:
                seen_standing.add(vte.vte_pool_info(ctx, info.standing_pctx).width)
            if info.escalated_pctx >= 0:
                seen_escalated.add(vte.vte_pool_info(ctx, info.escalated_pctx).width)
        vte.vte_vstream_sync(lat)
        got = ch.tok.cpu().numpy().copy()
        info = vte.vte_vstream_tpot_info(lat)
        st = vte.vte_stats(ctx)
        recs = vte.vte_stats_read(ctx)
        dec_widths = sorted({r.width for r in recs if r.klass == vte.VTE_CLASS_LATENCY})
        print("token on 32 CUs alone %.1f us; standing %s, escalated to %s, decode ran on %s; escalations %d, deadline misses %d of %d tokens, "
              "gates closed %d, reservations %d" % (t_real32 * 1e6, sorted(seen_standing), sorted(seen_escalated), dec_widths,
                                                    info.escalations, info.deadline_misses, info.tokens_done, st.gates_closed, st.reservations))
        for t in gq:
            vte.vte_token_wait(ctx, t)
        assert np.array_equal(got, ref)                         # the bits do not know where they ran
        assert seen_standing == {32}                            # sized from the (optimistic) profiles
        assert info.escalations > 0 and seen_escalated and min(seen_escalated) > 32   # Prepare reserved a wider pCtx
        assert st.gates_closed > 0                              # overlapping best-effort leases were drained
        assert st.reservations >= 1 + info.escalations
        assert max(dec_widths) > 32                             # and decode launches were really bound to it
        assert info.tokens_done == steps
        vte.vte_vstream_set_tpot(lat, 0.0, 0)
        vte.vte_vstream_destroy(lat)
        vte.vte_vstream_destroy(be)
    finally:
        vte.vte_shutdown(ctx)
