"""GPU: the dispatcher on real CU-masked streams — strict vs pipelined binding,
policy-driven late binding and co-tenancy give the same bits as explicit runs."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2603_15042_amd import inputs, vte

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    from paper_2603_15042_amd import harness
    return harness


@pytest.fixture(scope="module")
def setup(H):
    shp = inputs.DecodeShapes(D=1024, Nqkv=1536, F=3584, V=8200)
    w = inputs.decode_weights(5, shp)
    for k in ("Wqkv", "Wo", "Wgu", "Wd"):
        w[k] = inputs.normal_bf16(5, 100 + len(k), w[k].shape, 0.0, 1.5 * w[k].shape[1] ** -0.5)
    return shp, w


def free_run(H, ctx, shp, wd, B, steps, vs_setup=None, cotenant=None):
    ch = H.DecodeChain(ctx, wd, shp, B, feedback=True)
    ch.set_tokens(inputs.tokens(5, inputs.T_TOK0, B, shp.V))
    vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
    if vs_setup:
        vs_setup(vs)
    toks = []
    for s in range(steps):
        if cotenant:
            cotenant()
        ch.submit_step(vs)
        vte.vte_vstream_sync(vs)
        toks.append(ch.tok.cpu().numpy().copy())
    for i in range(vte.vte_pool_count(ctx)):              # reservations a setup hook made for this stream
        if vte.vte_pool_info(ctx, i).reserved_for == vte.vte_vstream_id(vs):
            vte.vte_pctx_unreserve(ctx, i)
    vte.vte_vstream_destroy(vs)
    ch.close()
    return np.stack(toks)


def test_strict_pipelined_and_pinned_runs_agree_bitwise(H, setup):
    shp, w = setup
    B, steps = 8, 24
    out = {}
    for name, mode in (("strict", vte.VTE_MODE_STRICT), ("pipelined", vte.VTE_MODE_PIPELINED)):
        ctx = H.make_ctx(mode)
        wd = H.upload_weights(w)
        out[name] = free_run(H, ctx, shp, wd, B, steps)
        if name == "pipelined":
            for wdt in (32, 64, 128):
                p = H.pctx_of_width(ctx, wdt)
                out["pinned%d" % wdt] = free_run(H, ctx, shp, wd, B, steps, lambda vs: vte.vte_vstream_pin(vs, p))
            recs = vte.vte_stats_read(ctx)
            assert all(r.t_submit <= r.t_bound <= r.t_done for r in recs)
        st = vte.vte_stats(ctx)
        assert st.completed == st.submitted and st.submit_failures == 0
        vte.vte_shutdown(ctx)
    base = out["strict"]
    assert len(np.unique(base)) > steps                  # the chain really moves through the vocabulary
    for k, v in out.items():
        assert np.array_equal(base, v), k


def test_cotenant_gemm_does_not_change_decode_bits(H, setup):
    """Decode steps with a best-effort GEMM tenant kept queued beside them: same tokens as alone, the
    GEMM's own bits unchanged -- and the two really ran side by side: by the device clock of the
    timed launches, GEMM launches on fewer than all CUs overlap decode steps on another pCtx."""
    from paper_2603_15042_amd import experiments as E
    shp, w = setup
    B, steps = 8, 24
    cfg = vte.vte_pool_cfg_default()
    cfg.mode = vte.VTE_MODE_PIPELINED
    cfg.lookahead = 32
    cfg.device_timing_mask = (1 << vte.VTE_K_GATHER) | (1 << vte.VTE_K_ARGMAX_FINISH) | (1 << vte.VTE_K_GEMM)
    torch.zeros(1, device="cuda")
    ctx = vte.vte_init(0, cfg)
    wd = H.upload_weights(w)
    solo = free_run(H, ctx, shp, wd, B, steps)
    M = 4096
    A = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_A, (M, M)))
    Bm = H.to_dev(inputs.normal_bf16(0, inputs.T_GEMM_B, (M, M)))
    Cm = H.dev_empty((M, M))
    g = vte.vte_desc_gemm(ctx, A, Bm, Cm, M, M, M)
    H.run_on(ctx, g, H.pctx_of_width(ctx, 256))
    c_solo = H.to_bits(Cm).copy()
    be = vte.vte_vstream_create(ctx, vte.VTE_CLASS_BEST_EFFORT)
    vte.vte_set_builtin_policy(ctx, vte.VTE_POLICY_QUEUE_STATE, 0.25, 64)
    vte.vte_device_sync(ctx)
    vte.vte_stats_reset(ctx)
    # a quarter of the device is reserved for the decode stream (Sec. 4.3, policy-directed reservation):
    # without it the GEMM, submitted while no decode launch is ready, takes all 256 CUs and the tenants
    # merely alternate in time
    reserve = lambda vs: vte.vte_hint_submit(ctx, vte.vte_hint(vte.vte_vstream_id(vs), 64, 0.0, 0.0))
    shared = free_run(H, ctx, shp, wd, B, steps, vs_setup=reserve, cotenant=lambda: [vte.vte_submit(be, g) for _ in range(2)])
    vte.vte_vstream_sync(be)
    assert np.array_equal(solo, shared)                  # same tokens with a co-tenant on other CUs
    assert np.array_equal(c_solo, H.to_bits(Cm))         # and the co-tenant's own bits are unchanged
    recs = vte.vte_stats_read(ctx)
    ov = E.overlap_of_tenants(recs, vte.VTE_K_GATHER, vte.VTE_K_ARGMAX_FINISH)
    widths = {r.width for r in recs if r.klass == vte.VTE_CLASS_BEST_EFFORT}
    print("co-tenant GEMM ran at widths", sorted(widths), ov)
    assert ov["decode_steps"] == steps
    assert ov["decode_steps_beside_a_best_effort_launch"] >= 4               # overlap in time, on another pCtx (12 of 24 when measured)
    assert ov["their_widths"] and max(ov["their_widths"]) < 256              # i.e. on a share of the CUs
    vte.vte_vstream_destroy(be)
    vte.vte_shutdown(ctx)


def test_hbm_bound_gemm_is_exact_beside_a_stream_that_saturates_hbm(H):
    """The GEMM's LDS fills really have to be waited for when its operands stream from HBM and a
    neighbour takes most of the bandwidth: a skinny GEMM on one half of the device, a 1 GB GEMV
    launched back to back on the other.  Small-integer inputs: every output bit must equal the
    exact product, launch after launch."""
    ctx = H.make_ctx(vte.VTE_MODE_PIPELINED)
    M, N, K = 32768, 256, 8192
    A = H.to_dev(inputs.int_bf16(71, inputs.T_GEMM_A, (M, K), -8, 8))
    Bm = H.to_dev(inputs.int_bf16(71, inputs.T_GEMM_B, (N, K), -8, 8, -2))
    C = H.dev_empty((M, N))
    g = vte.vte_desc_gemm(ctx, A, Bm, C, M, N, K)
    Bf = Bm.view(torch.bfloat16).float().t().contiguous()
    ref = torch.cat([torch.matmul(A[r0:r0 + 4096].view(torch.bfloat16).float(), Bf).to(torch.bfloat16).view(torch.int16)
                     for r0 in range(0, M, 4096)])
    Nw, Kw, B = 65536, 8192, 8
    W = H.to_dev(inputs.normal_bf16(71, inputs.T_W, (Nw, Kw), 0.0, Kw ** -0.5))
    X = H.to_dev(inputs.normal_bf16(71, inputs.T_XB, (B, Kw)))
    Y = H.dev_empty((B, Nw))
    hog = vte.vte_desc_gemv(ctx, W, X, Y, B, Nw, Kw)
    half0 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 0)
    half1 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 1)
    vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_BEST_EFFORT)
    vte.vte_vstream_pin(vs, half0)
    H.run_on(ctx, hog, half0)
    y_ref = H.to_bits(Y).copy()
    shared = 0
    for rep in range(6):
        C.fill_(0x7FC1)
        torch.cuda.synchronize()
        tail = [vte.vte_submit(vs, hog) for _ in range(24)][-1]      # several milliseconds of streaming next door
        H.run_on(ctx, g, half1)
        busy = not vte.vte_token_query(ctx, tail)
        assert int((C != ref).sum()) == 0, rep
        vte.vte_token_wait(ctx, tail)
        shared += int(busy)
    assert shared >= 3, "the neighbour had mostly finished before the GEMM did: little was shared"
    assert np.array_equal(H.to_bits(Y), y_ref)
    vte.vte_vstream_destroy(vs)
    vte.vte_shutdown(ctx)
