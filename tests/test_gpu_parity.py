"""GPU parity: every kernel through the C ABI against the CPU oracle, and the
invariant itself (bitwise equality across CU widths).  Needs an MI355X."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2603_15042_amd import inputs, vte
from gpu_common import bf16_close, f64

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    from paper_2603_15042_amd import harness
    return harness


@pytest.fixture(scope="module")
def ctx(H):
    c = H.make_ctx(vte.VTE_MODE_STRICT)
    yield c
    vte.vte_shutdown(c)


def all_pctx(ctx):
    return list(range(vte.vte_pool_count(ctx)))


def widths_of(ctx):
    return {i: vte.vte_pool_info(ctx, i).width for i in all_pctx(ctx)}


def run_everywhere(H, ctx, desc, out_tensor, pctxs=None):
    """Runs desc on each pCtx, returns {pctx: output bits}; output is poisoned between runs."""
    res = {}
    for p in (pctxs or all_pctx(ctx)):
        out_tensor.fill_(0x7FC1 if out_tensor.dtype == torch.int16 else -1)
        torch.cuda.synchronize()
        H.run_on(ctx, desc, p)
        torch.cuda.synchronize()
        res[p] = out_tensor.cpu().numpy().copy()
    return res


def assert_all_equal(res):
    vals = list(res.values())
    for v in vals[1:]:
        assert np.array_equal(vals[0].view(np.uint8), v.view(np.uint8))
    return vals[0]


# ---------- pool on the device --------------------------------------------------------------
def test_pool_is_precreated_with_every_width(ctx):
    w = sorted(set(widths_of(ctx).values()))
    assert w == [32, 64, 128, 192, 224, 256]
    assert vte.vte_pool_count(ctx) == 17          # full tree + one remainder per level: stays under the queue limit
    assert all(vte.vte_pctx_native_stream(ctx, i) for i in all_pctx(ctx))


# ---------- RMSNorm / LayerNorm ---------------------------------------------------------------
@pytest.mark.parametrize("rows,cols", [(8, 1024), (1, 8), (5, 1000), (3, 4096), (2, 16384), (300, 2048),
                                       (1000, 4096), (515, 520), (777, 1536), (512, 8), (600, 4104)])   # from 512 rows: one wave per row
def test_rmsnorm_parity_and_width_invariance(H, ctx, rows, cols):
    x, g = inputs.rmsnorm_case(seed=0, rows=rows, cols=cols)
    dx, dg, dy = H.to_dev(x), H.to_dev(g), H.dev_empty((rows, cols))
    d = vte.vte_desc_rmsnorm(ctx, dx, dg, dy, rows, cols, 1e-6)
    res = run_everywhere(H, ctx, d, dy)
    y = assert_all_equal(res).view(np.uint16)           # 0 mismatched bits on every pCtx of the pool
    bf16_close(y, oracle.rmsnorm(x, g, 1e-6), "rmsnorm %dx%d" % (rows, cols))
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("rows,cols", [(8, 1024), (5, 1000), (3, 4096), (2, 16384), (300, 2048), (1000, 4096), (515, 520), (777, 1536)])
def test_rmsnorm_bits_equal_the_documented_tree(H, ctx, rows, cols):
    """The kernel's output is the bits of the tree its header documents, emulated in float32 on the CPU."""
    import tree_emulator
    x, g = inputs.rmsnorm_case(seed=5, rows=rows, cols=cols)
    dx, dg, dy = H.to_dev(x), H.to_dev(g), H.dev_empty((rows, cols))
    d = vte.vte_desc_rmsnorm(ctx, dx, dg, dy, rows, cols, 1e-6)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 64))
    assert H.mismatched_bits(H.to_bits(dy), tree_emulator.rmsnorm_bits(x, g, 1e-6)) == (0, 0)
    vte.vte_desc_destroy(d)
    if rows < 512:
        # a regrouped sum (the reshaped baseline's thread count) is another tree: the emulator follows it too
        for cus in (32, 256):
            t = 64 * (cus // 32)
            if cols > 64 * t:
                continue
            d = vte.vte_desc_rmsnorm_reshaped(ctx, dx, dg, dy, rows, cols, 1e-6, cus)
            H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
            assert H.mismatched_bits(H.to_bits(dy), tree_emulator.rmsnorm_bits(x, g, 1e-6, threads=t)) == (0, 0)
            vte.vte_desc_destroy(d)


def test_rmsnorm_closed_forms_on_gpu(H, ctx):
    n = 1024
    sign = np.where(np.arange(n) % 3 == 0, -1.0, 1.0).astype(np.float32)
    x = np.stack([sign, np.zeros(n, np.float32), 4 * sign, np.eye(n, dtype=np.float32)[17] * 3])
    xb, gb = inputs.bf16_bits(x), inputs.bf16_bits(np.ones(n, np.float32))
    dx, dg, dy = H.to_dev(xb), H.to_dev(gb), H.dev_empty((4, n))
    d = vte.vte_desc_rmsnorm(ctx, dx, dg, dy, 4, n, 1e-6)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
    y = f64(H.to_bits(dy))
    assert np.array_equal(y[0], sign)                   # unit-RMS row -> exactly +-1
    assert np.all(y[1] == 0)                            # zero row stays zero (eps keeps it finite)
    assert np.array_equal(y[2], sign)                   # scale invariance at bf16 precision
    assert y[3, 17] == 32.0 and np.count_nonzero(y[3]) == 1   # one-hot -> sqrt(n)
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("rows,cols", [(8, 1024), (4, 96), (2, 4096), (3, 8192), (1001, 4096), (530, 1000)])
def test_layernorm_parity_and_width_invariance(H, ctx, rows, cols):
    x, g, b = inputs.layernorm_case(seed=1, rows=rows, cols=cols)
    dx, dg, db, dy = H.to_dev(x), H.to_dev(g), H.to_dev(b), H.dev_empty((rows, cols))
    d = vte.vte_desc_layernorm(ctx, dx, dg, db, dy, rows, cols, 1e-6)
    res = run_everywhere(H, ctx, d, dy)
    y = assert_all_equal(res).view(np.uint16)
    bf16_close(y, oracle.layernorm(x, g, b, 1e-6), "layernorm")
    # constant row -> beta exactly
    xc = inputs.bf16_bits(np.full((rows, cols), 2.5, np.float32))
    dx.copy_(H.to_dev(xc))
    H.run_on(ctx, d, 0)
    assert H.mismatched_bits(H.to_bits(dy), np.ascontiguousarray(np.broadcast_to(b, (rows, cols)))) == (0, 0)
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("layer,rows,cols", [(False, 524357, 4096), (True, 270001, 8192)])
def test_norms_beyond_2_to_the_31_elements(H, ctx, layer, rows, cols):
    """Maximum sizes: more than 2^31 elements (4.3 GB in, 4.3 GB out), one wave per row (cols <= 4096) and one
    workgroup per row.  Sampled rows (both ends, both sides of the row where element offsets pass 2^31 and
    byte offsets 2^32, random ones) against the oracle; every row against a float32 evaluation on the GPU."""
    x = inputs.normal_bf16(21, inputs.T_X, (rows, cols))
    g = inputs.uniform_bf16(21, inputs.T_GAMMA, (cols,), 0.5, 1.5)
    b = inputs.normal_bf16(21, inputs.T_BETA, (cols,), 0.0, 0.5)
    edge = (1 << 31) // cols
    pick = np.unique(np.concatenate([np.arange(40), np.arange(edge - 20, edge + 20), np.arange(rows - 40, rows),
                                     np.random.default_rng(6).integers(0, rows, 100)]))
    assert 0 <= pick.min() and pick.max() < rows and edge + 20 <= rows
    xs = np.ascontiguousarray(x[pick])
    dx, dg, db, dy = H.to_dev(x), H.to_dev(g), H.to_dev(b), H.dev_empty((rows, cols))
    d = (vte.vte_desc_layernorm(ctx, dx, dg, db, dy, rows, cols, 1e-6) if layer
         else vte.vte_desc_rmsnorm(ctx, dx, dg, dy, rows, cols, 1e-6))
    H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
    got = dy[torch.from_numpy(pick).cuda()].cpu().numpy().view(np.uint16)
    bf16_close(got, oracle.layernorm(xs, g, b, 1e-6) if layer else oracle.rmsnorm(xs, g, 1e-6), "norm rows")
    gf = dg.view(torch.bfloat16).float()
    step = 1 << 15
    for r0 in range(0, rows, step):                        # float32 on the GPU, a slab at a time
        xf = dx[r0:r0 + step].view(torch.bfloat16).float()
        if layer:
            mu = xf.mean(1, keepdim=True)
            ref = (xf - mu) * torch.rsqrt(((xf - mu) ** 2).mean(1, keepdim=True) + 1e-6) * gf + db.view(torch.bfloat16).float()
        else:
            ref = xf * torch.rsqrt((xf * xf).mean(1, keepdim=True) + 1e-6) * gf
        yf = dy[r0:r0 + step].view(torch.bfloat16).float()
        assert bool(((yf - ref).abs() <= 2.0 ** -7 * ref.abs() + 1e-3).all()), r0
    vte.vte_desc_destroy(d)
    del dx, dy
    torch.cuda.empty_cache()


def test_rmsnorm_reshaped_drifts_on_random_and_not_on_exact_inputs(H, ctx):
    rows, cols = 64, 4096
    x, g = inputs.rmsnorm_case(seed=3, rows=rows, cols=cols)
    dx, dg, dy = H.to_dev(x), H.to_dev(g), H.dev_empty((rows, cols))
    outs = {}
    for w in (32, 64, 128, 256):
        d = vte.vte_desc_rmsnorm_reshaped(ctx, dx, dg, dy, rows, cols, 1e-6, w)
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        outs[w] = H.to_bits(dy).copy()
        bf16_close(outs[w], oracle.rmsnorm(x, g, 1e-6), "reshaped rmsnorm")   # still correct, just not bit-stable
        vte.vte_desc_destroy(d)
    drift = [H.mismatched_bits(outs[256], outs[w])[1] for w in (32, 64, 128)]
    assert sum(drift) > 0, "regrouping the sum of squares should move some bits on random data"
    # exact inputs: every partial sum is exact in fp32, so every grouping gives the same bits
    xi = inputs.int_bf16(3, inputs.T_X, (rows, cols), -4, 4)
    dx.copy_(H.to_dev(xi))
    outs = {}
    for w in (32, 256):
        d = vte.vte_desc_rmsnorm_reshaped(ctx, dx, dg, dy, rows, cols, 1e-6, w)
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        outs[w] = H.to_bits(dy).copy()
        vte.vte_desc_destroy(d)
    assert H.mismatched_bits(outs[32], outs[256]) == (0, 0)


# ---------- GEMV -------------------------------------------------------------------------------
@pytest.mark.parametrize("B,N,K", [(1, 4096, 4096), (4, 4096, 4096), (8, 4096, 4096), (3, 37, 520), (5, 1, 8),
                                   (16, 1000, 1024), (2, 260, 14336), (8, 513, 2048)])
def test_gemv_parity_and_width_invariance(H, ctx, B, N, K):
    W, X = inputs.gemv_case(seed=0, B=B, N=N, K=K)
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, N))
    d = vte.vte_desc_gemv(ctx, dW, dX, dY, B, N, K)
    pct = [H.pctx_of_width(ctx, w) for w in (32, 64, 128, 192, 224, 256)] + [H.pctx_of_width(ctx, 32, 7)]
    res = run_everywhere(H, ctx, d, dY, pct)
    y = assert_all_equal(res).view(np.uint16)
    err, ulps = bf16_close(y, oracle.gemv(W, X), "gemv B%d %dx%d" % (B, N, K))
    assert err <= 2e-2                                   # |y| < 8 here: the literal tolerance holds
    vte.vte_desc_destroy(d)


def test_gemv_weights_beyond_4_gib_are_addressed_with_64_bits(H, ctx):
    """Maximum sizes: W = 278531 x 8192 bf16 is 4.56 GB and 2.28e9 elements, so byte offsets pass 2^32 and
    element offsets 2^31 at row 262144, and the last tile is ragged.  Small-integer inputs make every
    partial sum exact in fp32, so each kernel family (dot products at batch 4, K-split matrix-core tiles
    at batch 8, row-split ones at batch 40) must equal the oracle bit for bit on the sampled rows
    (both ends, both sides of the boundary, random ones) and the exact fp32 product everywhere."""
    N, K = 278531, 8192
    W = inputs.int_bf16(11, inputs.T_W, (N, K), -8, 8)
    rows = np.unique(np.concatenate([np.arange(64), np.arange(262144 - 64, 262144 + 64), np.arange(N - 300, N),
                                     np.random.default_rng(5).integers(0, N, 256)]))
    dW = H.to_dev(W)
    Wf = dW.view(torch.bfloat16).float()
    for B in (4, 8, 40):
        X = inputs.int_bf16(11 + B, inputs.T_XB, (B, K), -8, 8, -2)
        dX, dY = H.to_dev(X), H.dev_empty((B, N))
        d = vte.vte_desc_gemv(ctx, dW, dX, dY, B, N, K)
        H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
        y = H.to_bits(dY)
        assert np.array_equal(y[:, rows], oracle.f64_to_bf16(oracle.gemv(W[rows], X))), B
        whole = torch.matmul(dX.view(torch.bfloat16).float(), Wf.t()).to(torch.bfloat16).view(torch.int16)
        assert torch.equal(whole, dY), B
        vte.vte_desc_destroy(d)
        del whole, dX, dY
    del dW, Wf
    torch.cuda.empty_cache()


def test_gemv_identity_permutation_and_exact_inputs(H, ctx):
    K = 1024
    X = inputs.normal_bf16(7, inputs.T_XB, (4, K))
    perm = np.random.default_rng(0).permutation(K)
    P = np.zeros((K, K), np.float32)
    P[np.arange(K), perm] = 1.0
    dW, dX, dY = H.to_dev(inputs.bf16_bits(P)), H.to_dev(X), H.dev_empty((4, K))
    d = vte.vte_desc_gemv(ctx, dW, dX, dY, 4, K, K)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 64))
    assert np.array_equal(H.to_bits(dY), X[:, perm])     # bit-exact: all other products are zero
    vte.vte_desc_destroy(d)
    # small integers: every fp32 partial sum is exact -> GPU == oracle bitwise, whatever the tree
    W = inputs.int_bf16(3, inputs.T_W, (300, 4096), -8, 8)
    Xi = inputs.int_bf16(3, inputs.T_XB, (8, 4096), -8, 8, -2)
    dW, dX, dY = H.to_dev(W), H.to_dev(Xi), H.dev_empty((8, 300))
    d = vte.vte_desc_gemv(ctx, dW, dX, dY, 8, 300, 4096)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 128))
    assert np.array_equal(H.to_bits(dY), oracle.f64_to_bf16(oracle.gemv(W, Xi)))
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B", [1, 8])
def test_gemv_splitk_reshaping_drifts_and_fixed_does_not(H, ctx, B):
    N = K = 4096
    W, X = inputs.gemv_case(seed=0, B=B, N=N, K=K)
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, N))
    fixed = vte.vte_desc_gemv(ctx, dW, dX, dY, B, N, K)
    H.run_on(ctx, fixed, H.pctx_of_width(ctx, 256))
    y_fixed = H.to_bits(dY).copy()
    ref = oracle.gemv(W, X)
    drift = {}
    for w in (32, 64, 128, 256):
        S = w // 32
        ws = H.dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S))
        d = vte.vte_desc_gemv_splitk(ctx, dW, dX, dY, ws, B, N, K, 0, S)
        for rep in range(2):                             # second launch checks the tickets were reset
            dY.fill_(0)
            H.run_on(ctx, d, H.pctx_of_width(ctx, w))
            y = H.to_bits(dY).copy()
            bf16_close(y, ref, "split-K S=%d" % S)
            if rep == 0:
                first = y
            assert np.array_equal(first, y)
        drift[w] = H.mismatched_bits(y_fixed, y)
        vte.vte_desc_destroy(d)
    assert drift[32] == (0, 0)                           # S = 1 is the fixed structure
    print("split-K drift of bf16 outputs (elements, bits) vs fixed, B=%d:" % B, drift)
    # bf16 rounding hides most fp32-level regrouping (a flip needs the sum to sit within ~1e-7 of
    # a rounding boundary), so the unrounded fp32 sums are compared as well: same W and X through
    # the LM-head form of the kernel, which stores its fp32 accumulators
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    lg = torch.zeros((B, N), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, N, K))
    d = vte.vte_desc_lmhead_argmax(ctx, dW, dX, tok, lg, ws, B, N, K)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
    lg_fixed, tok_fixed = lg.cpu().numpy().copy(), tok.cpu().numpy().copy()
    vte.vte_desc_destroy(d)
    assert np.abs(lg_fixed - ref).max() < 1e-4
    drift32 = {}
    for w in (32, 64, 128, 256):
        S = w // 32
        part = H.dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S))
        d = vte.vte_desc_lmhead_argmax_splitk(ctx, dW, dX, tok, lg, ws, part, B, N, K, S)
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        drift32[w] = H.mismatched_bits(lg_fixed, lg.cpu().numpy())
        assert np.abs(lg.cpu().numpy() - ref).max() < 1e-4
        vte.vte_desc_destroy(d)
    print("split-K drift of fp32 sums (elements, bits) vs fixed, B=%d:" % B, drift32)
    assert drift32[32] == (0, 0)
    # An S coincides with the fixed tree exactly when K/S equals the fixed kernel's own K-slice
    # (adding one-slice chunks in order IS the fixed order): S = 2 at batch 8 (2048-wide slices),
    # S = 4 at batch 1 (1024-wide slices).  Every other S regroups the sum.
    assert sum(1 for w in (64, 128, 256) if drift32[w][1] > 0) >= 2   # regrouping moves bits on random data
    # negative control: exact inputs -> no drift for any S
    Wi = inputs.int_bf16(5, inputs.T_W, (N, K), -8, 8)
    Xi = inputs.int_bf16(5, inputs.T_XB, (B, K), -8, 8, -2)
    dW.copy_(H.to_dev(Wi))
    dX.copy_(H.to_dev(Xi))
    H.run_on(ctx, fixed, H.pctx_of_width(ctx, 256))
    y_fixed = H.to_bits(dY).copy()
    for S in (2, 8):
        ws = H.dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S))
        d = vte.vte_desc_gemv_splitk(ctx, dW, dX, dY, ws, B, N, K, 0, S)
        H.run_on(ctx, d, H.pctx_of_width(ctx, 32 * S))
        assert H.mismatched_bits(y_fixed, H.to_bits(dY)) == (0, 0)
        vte.vte_desc_destroy(d)
    vte.vte_desc_destroy(fixed)


@pytest.mark.parametrize("B,N,K", [(17, 4096, 4096), (32, 4096, 4096), (24, 513, 2048), (32, 37, 520), (20, 16, 8), (32, 260, 14336)])
def test_gemv_batch_17_to_32_parity_and_width_invariance(H, ctx, B, N, K):
    """Two column tiles per weight tile: same parity bar, same bits on every pCtx, and a row's result
    is the one it has in a batch of 16 (the column tiles run the same chain)."""
    W, X = inputs.gemv_case(seed=2, B=B, N=N, K=K)
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, N))
    d = vte.vte_desc_gemv(ctx, dW, dX, dY, B, N, K)
    res = run_everywhere(H, ctx, d, dY, [H.pctx_of_width(ctx, w) for w in (32, 64, 128, 224, 256)])
    y = assert_all_equal(res).view(np.uint16)
    bf16_close(y, oracle.gemv(W, X), "gemv B=%d" % B)
    vte.vte_desc_destroy(d)
    if N >= 16:
        # rows 1..16 as a batch of 16 through the one-tile kernel with the same K chunking and wave count
        p32 = vte.vte_gemv_default_plan(B, N, K, 0, 1)
        plan = vte.vte_gemv_default_plan(16, N, K, 0, 1)
        if plan.kind == vte.VTE_GEMV_MFMA and plan.ksteps == p32.ksteps:
            dX16, dY16 = H.to_dev(np.ascontiguousarray(X[1:17])), H.dev_empty((16, N))
            plan.max_waves, plan.rows, plan.prefetch, plan.groups = p32.max_waves, p32.rows, p32.prefetch, p32.groups
            try:
                d16 = vte.vte_desc_gemv_planned(ctx, dW, dX16, dY16, 16, N, K, 0, plan)
            except vte.VteError:
                d16 = None                         # this combination is not built for one tile
            if d16 is not None:
                H.run_on(ctx, d16, H.pctx_of_width(ctx, 256))
                assert np.array_equal(H.to_bits(dY16), y[1:17])
                vte.vte_desc_destroy(d16)


@pytest.mark.parametrize("B,F,K", [(32, 1000, 1024), (20, 14336, 4096)])
def test_gate_up_silu_batch_17_to_32(H, ctx, B, F, K):
    W = inputs.normal_bf16(4, inputs.T_WGU, (2 * F, K), 0.0, 2.0 * K ** -0.5)
    X = inputs.normal_bf16(4, inputs.T_XB, (B, K))
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, F))
    d = vte.vte_desc_gemv(ctx, dW, dX, dY, B, 2 * F, K, vte.VTE_EPI_SILU_MUL)
    res = run_everywhere(H, ctx, d, dY, [H.pctx_of_width(ctx, w) for w in (32, 256)])
    y = assert_all_equal(res).view(np.uint16)
    bf16_close(y, oracle.gemv_silu_mul(W, X), "silu B=%d" % B)
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B,V,K", [(32, 4099, 512), (19, 32064, 4096)])
def test_lmhead_batch_17_to_32_tokens_and_logits(H, ctx, B, V, K):
    W = inputs.normal_bf16(8, inputs.T_WLM, (V, K), 0.0, 0.02)
    X = inputs.normal_bf16(8, inputs.T_XB, (B, K))
    dW, dX = H.to_dev(W), H.to_dev(X)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    lg = torch.zeros((B, V), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    d = vte.vte_desc_lmhead_argmax(ctx, dW, dX, tok, lg, ws, B, V, K)
    fin = vte.vte_desc_argmax_finish(ctx, d)
    outs = []
    for w in (256, 32):
        tok.zero_()
        torch.cuda.synchronize()
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        H.run_on(ctx, fin, H.pctx_of_width(ctx, w))
        outs.append((lg.cpu().numpy().copy(), tok.cpu().numpy().copy()))
    assert np.array_equal(outs[0][0].view(np.uint32), outs[1][0].view(np.uint32)) and np.array_equal(outs[0][1], outs[1][1])
    ref, t_ref, margin = oracle.lmhead_argmax(W, X)
    eps_l = np.abs(outs[0][0] - ref).max()
    assert eps_l < 1e-3
    assert np.array_equal(outs[0][1], np.argmax(outs[0][0], axis=1))          # the token is the argmax of the GPU's own logits
    assert all(outs[0][1][b] == t_ref[b] or margin[b] <= 2 * eps_l for b in range(B))
    vte.vte_desc_destroy(fin)
    vte.vte_desc_destroy(d)


def rows_plan(g=2, ka=2, wr=8, rounds=1, bt=64):
    p = vte.vte_gemv_plan()
    p.batch_tile, p.rows, p.ksteps, p.prefetch, p.max_waves, p.groups, p.kind = bt, 16 * g, 1, ka, wr, rounds, vte.VTE_GEMV_MFMA_ROWS
    return p


@pytest.mark.parametrize("plan", [(2, 2, 4, 1), (2, 2, 8, 2), (4, 1, 4, 1), (4, 1, 8, 3), (4, 2, 4, 1), (4, 2, 8, 2)])
def test_row_split_kind_with_two_column_tiles(H, ctx, plan):
    """Batch 17 to 32 through the row-split kind (the default for the LM head there): plain, SiLU-mul
    and LM head on ragged shapes, every built combination; same bits on 32 and 256 CUs, and for the
    plain GEMV the same bits from every plan (an output is one chain along K)."""
    g, ka, wr, rounds = plan
    B, N, K = 29, 1000, 1160
    W, X = inputs.gemv_case(seed=9, B=B, N=N, K=K)
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, N))
    d = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, N, K, 0, rows_plan(g, ka, wr, rounds, 32))
    y = assert_all_equal(run_everywhere(H, ctx, d, dY, [H.pctx_of_width(ctx, w) for w in (32, 256)])).view(np.uint16)
    bf16_close(y, oracle.gemv(W, X), "gemv rows plan %s" % (plan,))
    vte.vte_desc_destroy(d)
    d0 = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, N, K, 0, rows_plan(2, 2, 8, 1, 32))
    dY.fill_(0x7FC1)
    H.run_on(ctx, d0, H.pctx_of_width(ctx, 256))
    assert np.array_equal(H.to_bits(dY), y)
    vte.vte_desc_destroy(d0)
    # the four-column-tile kernel runs the same chain: the same rows in a batch of 64 slots give the same bits
    d4 = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, N, K, 0, rows_plan(2, 2, 8, 1, 64))
    dY.fill_(0x7FC1)
    H.run_on(ctx, d4, H.pctx_of_width(ctx, 64))
    assert np.array_equal(H.to_bits(dY), y)
    vte.vte_desc_destroy(d4)
    # SiLU-mul
    F = 500
    Wg = inputs.normal_bf16(4, inputs.T_WGU, (2 * F, K), 0.0, 2.0 * K ** -0.5)
    dWg, dYs = H.to_dev(Wg), H.dev_empty((B, F))
    d = vte.vte_desc_gemv_planned(ctx, dWg, dX, dYs, B, 2 * F, K, vte.VTE_EPI_SILU_MUL, rows_plan(g, ka, wr, rounds, 32))
    ys = assert_all_equal(run_everywhere(H, ctx, d, dYs, [H.pctx_of_width(ctx, w) for w in (32, 256)])).view(np.uint16)
    bf16_close(ys, oracle.gemv_silu_mul(Wg, X), "silu rows plan %s" % (plan,))
    vte.vte_desc_destroy(d)
    # LM head
    V = 4099
    Wl = inputs.normal_bf16(8, inputs.T_WLM, (V, K), 0.0, 0.02)
    dWl = H.to_dev(Wl)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    lg = torch.zeros((B, V), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    d = vte.vte_desc_lmhead_argmax_planned(ctx, dWl, dX, tok, lg, ws, B, V, K, rows_plan(g, ka, wr, rounds, 32))
    fin = vte.vte_desc_argmax_finish(ctx, d)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 128))
    H.run_on(ctx, fin, H.pctx_of_width(ctx, 32))
    ref, t_ref, margin = oracle.lmhead_argmax(Wl, X)
    l, t = lg.cpu().numpy(), tok.cpu().numpy()
    eps_l = np.abs(l - ref).max()
    assert eps_l < 1e-3
    assert np.array_equal(t, np.argmax(l, axis=1))
    assert all(t[b] == t_ref[b] or margin[b] <= 2 * eps_l for b in range(B))
    vte.vte_desc_destroy(fin)
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("kind", ["default", "rows", "chunks"])
@pytest.mark.parametrize("B,N,K", [(33, 4096, 4096), (64, 4096, 4096), (48, 513, 2048), (64, 37, 520), (40, 16, 8),
                                   (64, 260, 14336), (50, 6144, 1000), (64, 33000, 256)])
def test_gemv_batch_33_to_64_parity_width_and_position_invariance(H, ctx, B, N, K, kind):
    """Batch 33 to 64 in one launch, four column tiles per weight tile.  Wide outputs: the waves split
    the rows and share X through LDS; narrow outputs: the K-split kernel with 256-element chunks;
    on request: two chunks of 32 rows through the two-column-tile kernel.  All: the parity bar of the
    other kinds, the same bits on every pCtx, and a row's result does not depend on where in the batch
    it stands or on the rows beside it."""
    W, X = inputs.gemv_case(seed=2, B=B, N=N, K=K)
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, N))

    def make(x, y, b):
        if kind == "rows":
            return vte.vte_desc_gemv_planned(ctx, dW, x, y, b, N, K, 0, rows_plan())
        if kind == "chunks":
            p32 = vte.vte_gemv_default_plan(32, N, K, 0, 1)
            if p32.kind == vte.VTE_GEMV_MFMA_ROWS:
                p32 = vte.vte_gemv_default_plan(32, 4096, K, 0, 1)
            return vte.vte_desc_gemv_planned(ctx, dW, x, y, b, N, K, 0, p32)
        return vte.vte_desc_gemv(ctx, dW, x, y, b, N, K)

    want = vte.VTE_GEMV_MFMA_ROWS if N >= 16384 else vte.VTE_GEMV_MFMA
    assert vte.vte_gemv_default_plan(B, N, K, 0, 1).kind == want
    d = make(dX, dY, B)
    res = run_everywhere(H, ctx, d, dY, [H.pctx_of_width(ctx, w) for w in (32, 64, 128, 224, 256)])
    y = assert_all_equal(res).view(np.uint16)
    bf16_close(y, oracle.gemv(W, X), "gemv B=%d" % B)
    vte.vte_desc_destroy(d)
    # the batch reversed, and a smaller batch made of its odd rows: every row keeps its bits
    dXr = H.to_dev(np.ascontiguousarray(X[::-1]))
    d = make(dXr, dY, B)
    dY.fill_(0x7FC1)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
    assert np.array_equal(H.to_bits(dY)[::-1], y)
    vte.vte_desc_destroy(d)
    odd = np.arange(1, B, 2)
    if len(odd) > 32 or kind != "default":
        dXo, dYo = H.to_dev(np.ascontiguousarray(X[odd])), H.dev_empty((len(odd), N))
        d = make(dXo, dYo, len(odd))
        H.run_on(ctx, d, H.pctx_of_width(ctx, 128))
        assert np.array_equal(H.to_bits(dYo), y[odd])
        vte.vte_desc_destroy(d)


@pytest.mark.parametrize("plan", [(1, 2, 4, 1), (1, 2, 8, 2), (2, 2, 4, 2), (2, 2, 8, 3), (2, 1, 8, 1), (4, 1, 4, 2), (4, 1, 8, 1)])
def test_gemv_batch_64_every_built_row_split_plan(H, ctx, plan):
    """Every built combination (tiles per wave, K steps ahead, waves, rounds) on a ragged shape: the
    plan changes who computes a row, not the chain of an output along K, so all give the same bits."""
    g, ka, wr, rounds = plan
    B, N, K = 57, 1000, 1160
    W, X = inputs.gemv_case(seed=9, B=B, N=N, K=K)
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, N))
    d = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, N, K, 0, rows_plan(g, ka, wr, rounds))
    res = run_everywhere(H, ctx, d, dY, [H.pctx_of_width(ctx, w) for w in (32, 256)])
    y = assert_all_equal(res).view(np.uint16)
    bf16_close(y, oracle.gemv(W, X), "gemv rows plan %s" % (plan,))
    vte.vte_desc_destroy(d)
    d0 = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, N, K, 0, rows_plan())
    dY.fill_(0x7FC1)
    H.run_on(ctx, d0, H.pctx_of_width(ctx, 256))
    assert np.array_equal(H.to_bits(dY), y)
    vte.vte_desc_destroy(d0)


@pytest.mark.parametrize("kind", ["default", "rows"])
@pytest.mark.parametrize("B,F,K", [(64, 1000, 1024), (40, 14336, 4096), (33, 8, 264)])
def test_gate_up_silu_batch_33_to_64(H, ctx, B, F, K, kind):
    W = inputs.normal_bf16(4, inputs.T_WGU, (2 * F, K), 0.0, 2.0 * K ** -0.5)
    X = inputs.normal_bf16(4, inputs.T_XB, (B, K))
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, F))
    if kind == "rows":
        d = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, 2 * F, K, vte.VTE_EPI_SILU_MUL, rows_plan(4, 1, 4, 2))
    else:
        d = vte.vte_desc_gemv(ctx, dW, dX, dY, B, 2 * F, K, vte.VTE_EPI_SILU_MUL)
    res = run_everywhere(H, ctx, d, dY, [H.pctx_of_width(ctx, w) for w in (32, 256)])
    y = assert_all_equal(res).view(np.uint16)
    bf16_close(y, oracle.gemv_silu_mul(W, X), "silu B=%d" % B)
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("kind", ["default", "rows"])
@pytest.mark.parametrize("B,V,K", [(64, 4099, 512), (37, 32064, 4096), (64, 16, 128)])
def test_lmhead_batch_33_to_64_tokens_and_logits(H, ctx, B, V, K, kind):
    W = inputs.normal_bf16(8, inputs.T_WLM, (V, K), 0.0, 0.02)
    X = inputs.normal_bf16(8, inputs.T_XB, (B, K))
    dW, dX = H.to_dev(W), H.to_dev(X)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    lg = torch.zeros((B, V), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    if kind == "rows":
        d = vte.vte_desc_lmhead_argmax_planned(ctx, dW, dX, tok, lg, ws, B, V, K, rows_plan(2, 2, 8, 2))
    else:
        d = vte.vte_desc_lmhead_argmax(ctx, dW, dX, tok, lg, ws, B, V, K)
    fin = vte.vte_desc_argmax_finish(ctx, d)
    outs = []
    for w in (256, 32):
        tok.zero_()
        torch.cuda.synchronize()
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        H.run_on(ctx, fin, H.pctx_of_width(ctx, w))
        outs.append((lg.cpu().numpy().copy(), tok.cpu().numpy().copy()))
    assert np.array_equal(outs[0][0].view(np.uint32), outs[1][0].view(np.uint32)) and np.array_equal(outs[0][1], outs[1][1])
    ref, t_ref, margin = oracle.lmhead_argmax(W, X)
    eps_l = np.abs(outs[0][0] - ref).max()
    assert eps_l < 1e-3
    assert np.array_equal(outs[0][1], np.argmax(outs[0][0], axis=1))          # the token is the argmax of the GPU's own logits
    assert all(outs[0][1][b] == t_ref[b] or margin[b] <= 2 * eps_l for b in range(B))
    vte.vte_desc_destroy(fin)
    vte.vte_desc_destroy(d)


# ---------- the matrix-core trees, emulated on the CPU ------------------------------------------------
@pytest.mark.parametrize("B,N,K,S,epi", [(64, 4096, 4096, 4, 0), (40, 528, 2048, 2, 0), (64, 4096, 14336, 14, 0), (33, 6144, 4096, 4, 0),
                                         (64, 1000, 2048, 2, 1), (16, 272, 1024, 2, 0)])
def test_gemv_shape_derived_split_and_finish(H, ctx, B, N, K, S, epi):
    """The two-launch GEMV for narrow outputs at a large batch: a K split whose factor comes from the
    shape, partial sums in a workspace, a finish launch that adds them in order.  Against the oracle,
    bit-equal on every width, and a row's bits do not depend on the rows beside it."""
    W = inputs.normal_bf16(41, inputs.T_W, (N, K), 0.0, K ** -0.5)
    X = inputs.normal_bf16(41, inputs.T_XB, (B, K))
    dW, dX = H.to_dev(W), H.to_dev(X)
    n_out = N // 2 if epi else N
    dY = H.dev_empty((B, n_out))
    ws = H.dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S))
    d1 = vte.vte_desc_gemv_split(ctx, dW, dX, 0, ws, B, N, K, epi, S)
    d2 = vte.vte_desc_gemv_split_finish(ctx, d1, dY)
    v1, v2 = vte.vte_desc_info(d1), vte.vte_desc_info(d2)
    assert v1.kernel == vte.VTE_K_GEMV_SPLIT and v1.grid[1] == S and v2.kernel == vte.VTE_K_GEMV_SPLIT_FINISH
    res = {}
    for p in (H.pctx_of_width(ctx, 256), H.pctx_of_width(ctx, 32), H.pctx_of_width(ctx, 192)):
        dY.fill_(0x7FC1)
        ws.fill_(-1)                                    # stale partials of an earlier launch must not matter
        torch.cuda.synchronize()
        H.run_on(ctx, d1, p)
        H.run_on(ctx, d2, H.pctx_of_width(ctx, 64))     # the finish launch may be bound elsewhere
        res[p] = H.to_bits(dY).copy()
    y = assert_all_equal(res)
    ref = oracle.gemv_silu_mul(W, X) if epi else oracle.gemv(W, X)
    bf16_close(y, ref, "split GEMV %dx%d batch %d S %d" % (N, K, B, S))
    if B > 8:                                           # every second row alone: same bits
        Xh = np.ascontiguousarray(X[::2])
        Bh = Xh.shape[0]
        dXh, dYh = H.to_dev(Xh), H.dev_empty((Bh, n_out))
        wsh = H.dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S))
        plan = None
        if (Bh > 32) != (B > 32) or (Bh > 16) != (B > 16):   # keep the batch tile of the full batch: the tree depends on the plan
            plan = vte.vte_gemv_plan()
            plan.kind, plan.batch_tile = vte.VTE_GEMV_MFMA, (64 if B > 32 else 32)
            plan.ksteps, plan.prefetch, plan.max_waves = (2 if B > 32 else 4), (2 if B > 32 else 4), 4
            plan.rows, plan.groups = (32 if B > 32 else 16), (2 if (n_out + (7 if epi else 15)) // (8 if epi else 16) >= 512 else 1)
        e1 = vte.vte_desc_gemv_split(ctx, dW, dXh, 0, wsh, Bh, N, K, epi, S, plan)
        e2 = vte.vte_desc_gemv_split_finish(ctx, e1, dYh)
        H.run_on(ctx, e1, H.pctx_of_width(ctx, 128))
        H.run_on(ctx, e2, H.pctx_of_width(ctx, 128))
        assert np.array_equal(H.to_bits(dYh), y[::2])
        vte.vte_desc_destroy(e2); vte.vte_desc_destroy(e1)
    vte.vte_desc_destroy(d2); vte.vte_desc_destroy(d1)


@pytest.mark.parametrize("B,N,K,S,binades", [(64, 48, 4096, 4, 0), (40, 32, 2048, 2, 6), (64, 16, 14336, 14, 0)])
def test_shape_derived_split_equals_its_emulated_tree_bit_for_bit(H, ctx, B, N, K, S, binades):
    """Partial sums and finished outputs of the two-launch GEMV against the CPU emulation of its tree:
    per part the K-split matrix-core tree (256-element chunks, one per wave), then p[0] + p[1] + ..."""
    import tree_emulator
    W = inputs.normal_bf16(43, inputs.T_W, (N, K), 0.0, K ** -0.5)
    if binades:
        W = _spread(W, 43, binades)
    X = inputs.normal_bf16(43, inputs.T_XB, (B, K))
    parts, total = tree_emulator.gemv_fixed_split_sums(W, X, S, 2, 4)
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, N))
    nbytes = vte.vte_splitk_workspace_bytes(B, N, S)
    ws = H.dev_zeros_bytes(nbytes)
    d1 = vte.vte_desc_gemv_split(ctx, dW, dX, 0, ws, B, N, K, 0, S)
    d2 = vte.vte_desc_gemv_split_finish(ctx, d1, dY)
    for wdt in (256, 64):
        ws.fill_(-1)
        H.run_on(ctx, d1, H.pctx_of_width(ctx, wdt))
        H.run_on(ctx, d2, H.pctx_of_width(ctx, wdt))
        raw = ws.cpu().numpy().view(np.float32)
        head = (nbytes - S * 64 * N * 4) // 4               # ticket words in front of the partials [S][64][N]
        got = raw[head:head + S * 64 * N].reshape(S, 64, N)[:, :B, :]
        assert np.array_equal(got.view(np.uint32), parts.view(np.uint32)), wdt
        assert np.array_equal(H.to_bits(dY), tree_emulator._f32_to_bf16(total)), wdt
    vte.vte_desc_destroy(d2); vte.vte_desc_destroy(d1)


def _spread(Wbits, seed, binades):
    """bf16 weights times seeded powers of two: makes the alignment inside the instruction visible."""
    rng = np.random.default_rng(seed)
    f = inputs.bf16_to_f32(Wbits) * np.exp2(rng.integers(-binades, binades + 1, size=Wbits.shape)).astype(np.float32)
    return inputs.bf16_bits(f)


@pytest.mark.parametrize("B,N,K,binades", [(40, 48, 520, 0), (64, 100, 1160, 0), (33, 37, 264, 6), (57, 64, 128, 20), (17, 32, 4096, 0),
                                           (40, 1300, 1160, 0), (64, 2100, 2048, 3), (33, 600, 1024, 4)])
def test_row_split_kernel_equals_its_emulated_tree_bit_for_bit(H, ctx, B, N, K, binades):
    """The fp32 sums (LM-head logits) of the row-split kernel against the CPU emulation of its tree
    (tests/tree_emulator.py: one chain of 8-product groups along K, walked from the start that the
    output's block of 512 fixes, the instruction's alignment and rounding reproduced): every bit, on a
    narrow and on the full-width pCtx, with two plans whose workgroups cover 128 and 512 outputs; and the
    bf16 outputs of the plain GEMV are those sums rounded once."""
    import tree_emulator
    W = inputs.normal_bf16(31, inputs.T_W, (N, K), 0.0, K ** -0.5)
    if binades:
        W = _spread(W, 31, binades)
    X = inputs.normal_bf16(31, inputs.T_XB, (B, K))
    want = tree_emulator.gemv_rows_kernel_sums(W, X)
    bt = 64 if B > 32 else 32
    dW, dX = H.to_dev(W), H.to_dev(X)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    lg = torch.zeros((B, N), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, N, K))
    d = vte.vte_desc_lmhead_argmax_planned(ctx, dW, dX, tok, lg, ws, B, N, K, rows_plan(2, 2, 8, 1, bt))
    for w in (32, 256):
        lg.fill_(-1.0)
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        assert np.array_equal(lg.cpu().numpy().view(np.uint32), want.view(np.uint32)), w
    vte.vte_desc_destroy(d)
    dY = H.dev_empty((B, N))
    d = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, N, K, 0, rows_plan(4, 1, 4, 2, bt))
    H.run_on(ctx, d, H.pctx_of_width(ctx, 128))
    assert np.array_equal(H.to_bits(dY), tree_emulator._f32_to_bf16(want))
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B,N,K,nbk,g,mw,binades", [(8, 64, 4096, 8, 2, 4, 0), (8, 48, 2088, 4, 1, 8, 0), (16, 40, 4096, 4, 2, 4, 0),
                                                    (5, 32, 14336, 4, 1, 8, 0), (13, 64, 1160, 8, 1, 4, 5), (32, 48, 4096, 4, 2, 8, 0),
                                                    (64, 32, 1032, 2, 1, 4, 0)])
def test_k_split_kernel_equals_its_emulated_tree_bit_for_bit(H, ctx, B, N, K, nbk, g, mw, binades):
    """The K-split matrix-core kernel (the benchmark's LM head is its 1024-element-chunk, four-wave
    plan): wave w chains its chunks w, w + nw, ... in ascending K, the waves' sums are added in wave
    order — emulated on the CPU and equal to the GPU's fp32 sums in every bit."""
    import tree_emulator
    W = inputs.normal_bf16(32, inputs.T_W, (N, K), 0.0, K ** -0.5)
    if binades:
        W = _spread(W, 32, binades)
    X = inputs.normal_bf16(32, inputs.T_XB, (B, K))
    want = tree_emulator.gemv_ksplit_sums(W, X, nbk, mw)
    bt = 16 if B <= 16 else (32 if B <= 32 else 64)
    plan = vte.vte_gemv_plan()
    plan.batch_tile, plan.rows, plan.ksteps, plan.prefetch, plan.max_waves, plan.groups, plan.kind = bt, 16 * g, nbk, 2, mw, 2, vte.VTE_GEMV_MFMA
    dW, dX = H.to_dev(W), H.to_dev(X)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    lg = torch.zeros((B, N), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, N, K))
    d = vte.vte_desc_lmhead_argmax_planned(ctx, dW, dX, tok, lg, ws, B, N, K, plan)
    for w in (64, 256):
        lg.fill_(-1.0)
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        assert np.array_equal(lg.cpu().numpy().view(np.uint32), want.view(np.uint32)), w
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B,N,K,binades", [(1, 64, 4096, 0), (4, 48, 1000, 0), (2, 32, 14336, 0), (3, 40, 520, 8), (1, 16, 8, 20),
                                           (4, 24, 2048, 3)])
def test_dot_product_kernels_equal_their_emulated_tree_bit_for_bit(H, ctx, B, N, K, binades):
    """Batch <= 4: v_dot2c_f32_bf16 accumulates by the same rule as the matrix cores (groups of 2), so the
    whole tree — pairs in a lane, k-steps of a wave, the 64-lane butterfly, the waves in order — is
    emulated on the CPU and must equal the GPU's fp32 sums in every bit, at every width."""
    import tree_emulator
    W = inputs.normal_bf16(33, inputs.T_W, (N, K), 0.0, K ** -0.5)
    if binades:
        W = _spread(W, 33, binades)
    X = inputs.normal_bf16(33, inputs.T_XB, (B, K))
    plan = vte.vte_gemv_default_plan(B, N, K, 0, 1)
    if B > 2:                         # from batch 3 the default is the matrix-core kind: ask for the four-row dot-product tile
        plan = vte.vte_gemv_plan(4, 8, 2, 1, 8, 1, vte.VTE_GEMV_DOT2)
    assert plan.kind == vte.VTE_GEMV_DOT2
    want = tree_emulator.gemv_dot2_sums(W, X, plan.ksteps)
    dW, dX = H.to_dev(W), H.to_dev(X)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    lg = torch.zeros((B, N), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, N, K))
    d = vte.vte_desc_lmhead_argmax_planned(ctx, dW, dX, tok, lg, ws, B, N, K, plan)
    for w in (32, 128, 256):
        lg.fill_(-1.0)
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        assert np.array_equal(lg.cpu().numpy().view(np.uint32), want.view(np.uint32)), w
    vte.vte_desc_destroy(d)
    dY = H.dev_empty((B, N))
    d = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, N, K, vte.VTE_EPI_NONE, plan)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 64))
    assert np.array_equal(H.to_bits(dY), tree_emulator._f32_to_bf16(want))
    vte.vte_desc_destroy(d)


def test_k_tail_pieces_are_not_fetched_behind_the_last_row(H, ctx):
    """Down-projection shape split 8 ways: K / S = 1792 is no multiple of the 512-element chunk of the
    matrix-core kernel, and the weight tensor (56 x 2 MiB exactly) ends where its allocation ends.  The
    pieces of the last chunk that lie past the end of a split must not be loaded: behind the last row
    they are outside the tensor."""
    B, N, K, S = 8, 4096, 14336, 8
    W = inputs.normal_bf16(6, inputs.T_WD, (N, K), 0.0, K ** -0.5)
    X = inputs.normal_bf16(6, inputs.T_XB, (B, K))
    torch.cuda.empty_cache()
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, N))
    ws = H.dev_zeros_bytes(vte.vte_splitk_workspace_bytes(B, N, S))
    d = vte.vte_desc_gemv_splitk(ctx, dW, dX, dY, ws, B, N, K, 0, S)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
    rows = np.array([0, 1, 2047, 4094, 4095])
    ref = oracle.gemv(W[rows], X)
    bf16_close(H.to_bits(dY)[:, rows], ref, "split-K with a K tail")
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B,F,K", [(2, 50, 256), (8, 1000, 1024), (4, 14336, 4096)])
def test_gate_up_silu_epilogue(H, ctx, B, F, K):
    W = inputs.normal_bf16(4, inputs.T_WGU, (2 * F, K), 0.0, 2.0 * K ** -0.5)
    X = inputs.normal_bf16(4, inputs.T_XB, (B, K))
    dW, dX, dY = H.to_dev(W), H.to_dev(X), H.dev_empty((B, F))
    d = vte.vte_desc_gemv(ctx, dW, dX, dY, B, 2 * F, K, vte.VTE_EPI_SILU_MUL)
    res = run_everywhere(H, ctx, d, dY, [H.pctx_of_width(ctx, w) for w in (32, 128, 256)])
    y = assert_all_equal(res).view(np.uint16)
    bf16_close(y, oracle.gemv_silu_mul(W, X), "gate/up")
    vte.vte_desc_destroy(d)


def test_strided_gemv_reads_a_column_slice(H, ctx):
    B, N, K, ld = 4, 96, 512, 768
    W = inputs.normal_bf16(2, inputs.T_W, (N, K), 0.0, K ** -0.5)
    Xw = inputs.normal_bf16(2, inputs.T_XB, (B, ld))
    dW, dX, dY = H.to_dev(W), H.to_dev(Xw), H.dev_empty((B, N))
    d = vte.vte_desc_gemv_strided(ctx, dW, dX, ld, dY, N, B, N, K)
    H.run_on(ctx, d, 0)
    bf16_close(H.to_bits(dY), oracle.gemv(W, np.ascontiguousarray(Xw[:, :K])), "strided")
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B,N,K,ld,ldy", [(8, 6160, 264, 520, 6176), (24, 4112, 1032, 2048, 4128), (40, 16400, 264, 520, 16416),
                                          (64, 272, 520, 1024, 288), (20, 65552, 136, 256, 65552)])
def test_strided_gemv_in_every_kernel_family(H, ctx, B, N, K, ld, ldy):
    """X rows ld elements apart, Y rows ldy apart, through the default plan of each family: matrix-core
    K split with one, two and four column tiles, row split with two and four; the columns of Y between
    N and ldy keep their poison."""
    W = inputs.normal_bf16(2, inputs.T_W, (N, K), 0.0, K ** -0.5)
    Xw = inputs.normal_bf16(2, inputs.T_XB, (B, ld))
    dW, dX, dY = H.to_dev(W), H.to_dev(Xw), H.dev_empty((B, ldy))
    dY.fill_(0x7FC1)
    d = vte.vte_desc_gemv_strided(ctx, dW, dX, ld, dY, ldy, B, N, K)
    out = []
    for w in (256, 32):
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        out.append(H.to_bits(dY).copy())
    assert np.array_equal(out[0], out[1])
    bf16_close(out[0][:, :N], oracle.gemv(W, np.ascontiguousarray(Xw[:, :K])), "strided B=%d" % B)
    assert np.all(out[0][:, N:] == 0x7FC1)
    vte.vte_desc_destroy(d)


# ---------- matrix-core GEMV plans (batch 3-16) ---------------------------------------------------------
MFMA_PLANS = [(1, 2, 8, 1), (2, 4, 4, 3), (4, 2, 8, 2), (8, 2, 8, 1), (4, 4, 4, 1), (8, 4, 4, 2), (2, 2, 4, 2)]


@pytest.mark.parametrize("G,NB,MW,rounds", MFMA_PLANS)
@pytest.mark.parametrize("B,N,K", [(5, 530, 2088), (8, 48, 4096), (16, 2100, 512), (13, 32, 14336)])
def test_gemv_mfma_plans(H, ctx, G, NB, MW, rounds, B, N, K):
    """Every built matrix-core decomposition, on shapes with ragged row tiles, a ragged
    K tail and several chunks per wave: plain, SiLU-mul and LM-head epilogues against
    the oracle, bit-equal on a narrow and the full-width pCtx."""
    plan = vte.vte_gemv_plan(16, 16 * G, 4, NB, MW, rounds, vte.VTE_GEMV_MFMA)
    W = inputs.normal_bf16(11, inputs.T_W, (N, K), 0.0, K ** -0.5)
    X = inputs.normal_bf16(11, inputs.T_XB, (B, K))
    dW, dX = H.to_dev(W), H.to_dev(X)
    pct = [H.pctx_of_width(ctx, 32, 3), H.pctx_of_width(ctx, 256)]
    ref = oracle.gemv(W, X)
    dY = H.dev_empty((B, N))
    d = vte.vte_desc_gemv_planned(ctx, dW, dX, dY, B, N, K, vte.VTE_EPI_NONE, plan)
    y = assert_all_equal(run_everywhere(H, ctx, d, dY, pct)).view(np.uint16)
    bf16_close(y, ref, "mfma gemv")
    vte.vte_desc_destroy(d)
    dY2 = H.dev_empty((B, N // 2))
    d = vte.vte_desc_gemv_planned(ctx, dW, dX, dY2, B, N, K, vte.VTE_EPI_SILU_MUL, plan)
    y = assert_all_equal(run_everywhere(H, ctx, d, dY2, pct)).view(np.uint16)
    bf16_close(y, oracle.gemv_silu_mul(W, X), "mfma gate/up")
    vte.vte_desc_destroy(d)
    tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    logits = torch.zeros((B, N), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, N, K))
    d = vte.vte_desc_lmhead_argmax_planned(ctx, dW, dX, tok, logits, ws, B, N, K, plan)
    fin = vte.vte_desc_argmax_finish(ctx, d)
    got = []
    for p_ in pct:
        tok.fill_(-7)
        logits.zero_()
        H.run_on(ctx, d, p_)
        H.run_on(ctx, fin, p_)
        torch.cuda.synchronize()
        got.append((tok.cpu().numpy().copy(), logits.cpu().numpy().copy()))
    assert np.array_equal(got[0][0], got[1][0]) and np.array_equal(got[0][1].view(np.uint32), got[1][1].view(np.uint32))
    assert np.abs(got[0][1].astype(np.float64) - ref).max() < 1e-4 * max(1.0, np.abs(ref).max())
    assert np.array_equal(got[0][0], oracle.argmax(got[0][1].astype(np.float64))[0])
    vte.vte_desc_destroy(d)
    vte.vte_desc_destroy(fin)


def test_gemv_mfma_plan_is_the_default_from_batch_3_and_rejects_what_is_not_built(H, ctx):
    assert vte.vte_gemv_default_plan(2, 4096, 4096).kind == vte.VTE_GEMV_DOT2
    p = vte.vte_gemv_default_plan(3, 4096, 4096)
    assert p.kind == vte.VTE_GEMV_MFMA and p.batch_tile == 16 and p.rows % 16 == 0
    assert vte.vte_gemv_default_plan(8, 8, 4096).kind == vte.VTE_GEMV_DOT2        # less than one tile of outputs
    W, X, Y = H.dev_empty((64, 512)), H.dev_empty((8, 512)), H.dev_empty((8, 64))
    for bad in (vte.vte_gemv_plan(16, 48, 4, 2, 8, 1, vte.VTE_GEMV_MFMA),       # 3 tiles at once: not built
                vte.vte_gemv_plan(8, 16, 4, 2, 8, 1, vte.VTE_GEMV_MFMA),        # batch tile is 16
                vte.vte_gemv_plan(16, 16, 4, 2, 8, 1, 7)):                      # unknown kind
        with pytest.raises(vte.VteError):
            vte.vte_desc_gemv_planned(ctx, W, X, Y, 8, 64, 512, vte.VTE_EPI_NONE, bad)


# ---------- LM head + argmax -----------------------------------------------------------------------
@pytest.mark.parametrize("B,V,K", [(1, 1, 64), (2, 7, 64), (4, 1000, 256), (8, 4097, 1024), (16, 2049, 512)])
def test_lmhead_logits_and_token(H, ctx, B, V, K):
    W = inputs.normal_bf16(6, inputs.T_WLM, (V, K), 0.0, 0.02)
    Hh = inputs.normal_bf16(6, inputs.T_XB, (B, K))
    plant = [0, V - 1, V // 2, min(V - 1, 63), min(V - 1, 64)]
    for b in range(min(B, len(plant))):                  # planted maxima at block boundaries
        W[plant[b]] = oracle.f64_to_bf16(0.25 * f64(Hh[b]))
    dW, dH = H.to_dev(W), H.to_dev(Hh)
    tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    logits = torch.zeros((B, V), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    d = vte.vte_desc_lmhead_argmax(ctx, dW, dH, tok, logits, ws, B, V, K)
    fin = vte.vte_desc_argmax_finish(ctx, d)
    ref_logits, ref_tok, margin = oracle.lmhead_argmax(W, Hh)
    got = {}
    for p in [H.pctx_of_width(ctx, w) for w in (32, 64, 128, 256)]:
        tok.fill_(-7)
        H.run_on(ctx, d, p)
        H.run_on(ctx, fin, p)
        torch.cuda.synchronize()
        got[p] = (tok.cpu().numpy().copy(), logits.cpu().numpy().copy())
    first = next(iter(got.values()))
    for t, l in got.values():
        assert np.array_equal(t, first[0]) and np.array_equal(l.view(np.uint32), first[1].view(np.uint32))
    eps_logit = np.abs(first[1].astype(np.float64) - ref_logits).max()
    assert eps_logit < 1e-4
    for b in range(B):
        assert first[0][b] == ref_tok[b] or margin[b] <= 2 * eps_logit
    # the token is the argmax of the GPU's own logits with ties to the lowest index
    assert np.array_equal(first[0], oracle.argmax(first[1].astype(np.float64))[0])
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B,V,K,g", [(8, 4099, 4096, 2), (13, 1000, 1160, 2), (16, 530, 8200, 1), (5, 2049, 1024, 2), (8, 300, 520, 1)])
def test_lmhead_with_1024_element_chunks(H, ctx, B, V, K, g):
    """The LM-head plan of the large vocabularies (1024-element K chunks, four waves, eight rounds) on
    small ragged shapes: K a multiple of the chunk, with a tail, shorter than one chunk and longer than
    the four chunks the waves hold at once; logits against the oracle, same bits at 32 and 256 CUs."""
    W = inputs.normal_bf16(6, inputs.T_WLM, (V, K), 0.0, 0.02)
    Hh = inputs.normal_bf16(6, inputs.T_XB, (B, K))
    dW, dH = H.to_dev(W), H.to_dev(Hh)
    tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    logits = torch.zeros((B, V), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    plan = vte.vte_gemv_plan()
    plan.batch_tile, plan.rows, plan.ksteps, plan.prefetch, plan.max_waves, plan.groups, plan.kind = 16, 16 * g, 8, 2, 4, 8, vte.VTE_GEMV_MFMA
    big = vte.vte_gemv_default_plan(8, 128256, 4096, 0, 1)
    assert (big.ksteps, big.rows, big.prefetch, big.max_waves, big.groups, big.kind) == (8, 32, 2, 4, 8, vte.VTE_GEMV_MFMA)
    d = vte.vte_desc_lmhead_argmax_planned(ctx, dW, dH, tok, logits, ws, B, V, K, plan)
    fin = vte.vte_desc_argmax_finish(ctx, d)
    ref_logits, ref_tok, margin = oracle.lmhead_argmax(W, Hh)
    got = []
    for w in (32, 256):
        tok.fill_(-7)
        logits.fill_(-1.0)
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        H.run_on(ctx, fin, H.pctx_of_width(ctx, w))
        got.append((tok.cpu().numpy().copy(), logits.cpu().numpy().copy()))
    assert np.array_equal(got[0][0], got[1][0]) and np.array_equal(got[0][1].view(np.uint32), got[1][1].view(np.uint32))
    eps_logit = np.abs(got[0][1].astype(np.float64) - ref_logits).max()
    assert eps_logit < 1e-4
    assert all(got[0][0][b] == ref_tok[b] or margin[b] <= 2 * eps_logit for b in range(B))
    assert np.array_equal(got[0][0], oracle.argmax(got[0][1].astype(np.float64))[0])
    vte.vte_desc_destroy(fin)
    vte.vte_desc_destroy(d)


def test_lmhead_ties_go_to_lowest_index(H, ctx):
    B, V, K = 2, 600, 128
    W = inputs.normal_bf16(8, inputs.T_WLM, (V, K), 0.0, 0.02)
    Hh = inputs.normal_bf16(8, inputs.T_XB, (B, K))
    row = oracle.f64_to_bf16(0.5 * f64(Hh[0]))
    for v in (599, 131, 300):                            # identical rows -> bitwise identical logits
        W[v] = row
    dW, dH = H.to_dev(W), H.to_dev(Hh)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    d = vte.vte_desc_lmhead_argmax(ctx, dW, dH, tok, None, ws, B, V, K)
    H.run_on(ctx, d, 3)
    H.run_on(ctx, vte.vte_desc_argmax_finish(ctx, d), 5)
    assert tok.cpu().numpy()[0] == 131
    assert tok.cpu().numpy()[0] == oracle.lmhead_argmax(W, Hh)[1][0]
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B", [1, 8, 32, 64])
def test_lmhead_full_vocabulary_exact_logits_and_planted_ties(H, ctx, B):
    """Small-integer weights and activations at the benchmark's LM-head shape: every logit is an exact
    fp32 number, so all B x 128256 logits must equal the exact product in every bit (each kernel family
    by batch); row 0's maximum is planted at three vocabulary entries, the last one included: the token
    must be the lowest of them, and equal the oracle's on the rows it computes."""
    V, K = 128256, 4096
    W = inputs.int_bf16(51, inputs.T_WLM, (V, K), -8, 8)
    X = inputs.int_bf16(51 + B, inputs.T_XB, (B, K), -2, 2)
    best = inputs.bf16_bits(8.0 * np.sign(inputs.bf16_to_f32(X[0])))   # the largest logit row 0 can have
    for v in (90001, 7, V - 1):
        W[v] = best
    dW, dX = H.to_dev(W), H.to_dev(X)
    tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    d = vte.vte_desc_lmhead_argmax(ctx, dW, dX, tok, logits, ws, B, V, K)
    fin = vte.vte_desc_argmax_finish(ctx, d)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
    H.run_on(ctx, fin, H.pctx_of_width(ctx, 32))
    exact = torch.matmul(dX.view(torch.bfloat16).float(), dW.view(torch.bfloat16).float().t())
    assert torch.equal(exact.view(torch.int32), logits.view(torch.int32))
    top = exact.max(1, keepdim=True).values
    ties = (exact == top).sum(1)
    first = torch.where(exact == top, torch.arange(V, device="cuda")[None, :], V).min(1).values
    assert torch.equal(first.to(torch.int32), tok)
    assert int(ties[0]) >= 3 and int(tok[0]) == 7        # the planted maximum is shared by three entries
    rows = list(range(min(B, 2)))
    assert np.array_equal(oracle.lmhead_argmax(W, X[rows])[1], tok.cpu().numpy()[rows])
    vte.vte_desc_destroy(fin)
    vte.vte_desc_destroy(d)
    del dW, exact, logits
    torch.cuda.empty_cache()


@pytest.mark.parametrize("B", [3, 8, 40])
def test_lmhead_nan_and_infinite_logits(H, ctx, B):
    """Degenerate logits in every kernel family: a NaN never wins, -inf never wins against a finite
    value, +inf wins and a tie at +inf goes to the lower index, a batch row whose logits are all NaN
    gives token 0 -- the oracle's rules."""
    V, K = 1000, 256
    W = inputs.normal_bf16(61, inputs.T_WLM, (V, K), 0.0, 0.02)
    X = inputs.normal_bf16(61, inputs.T_XB, (B, K))
    X &= 0x7FFF                                          # positive activations: an infinite weight row gives an infinite logit
    W[17] = 0x7FC0                                       # NaN
    W[800] = 0xFF80                                      # -inf
    W[300] = 0x7F80                                      # +inf, twice
    W[640] = 0x7F80
    X[2, 5] = 0x7FC0                                     # every logit of batch row 2 is NaN
    lg, t_ref, _ = oracle.lmhead_argmax(W, X)
    assert t_ref[0] == 300 and t_ref[2] == 0
    dW, dX = H.to_dev(W), H.to_dev(X)
    tok = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    logits = torch.empty((B, V), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    d = vte.vte_desc_lmhead_argmax(ctx, dW, dX, tok, logits, ws, B, V, K)
    fin = vte.vte_desc_argmax_finish(ctx, d)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 64))
    H.run_on(ctx, fin, H.pctx_of_width(ctx, 32))
    got = logits.cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(lg))
    fin_mask = np.isfinite(lg)
    assert np.array_equal(got[~fin_mask & ~np.isnan(lg)], lg[~fin_mask & ~np.isnan(lg)])   # the infinities, with their signs
    assert np.abs(got[fin_mask] - lg[fin_mask]).max() < 1e-4
    assert np.array_equal(tok.cpu().numpy(), t_ref)
    vte.vte_desc_destroy(fin)
    vte.vte_desc_destroy(d)


# ---------- gather ------------------------------------------------------------------------------------
def test_gather(H, ctx):
    V, K, B = 500, 4096, 16
    E = inputs.normal_bf16(1, inputs.T_EMB, (V, K))
    t = np.array([499, 0, 7, 7] + list(range(12)), np.int32)
    dE, dt, dH = H.to_dev(E), H.to_dev(t), H.dev_empty((B, K))
    d = vte.vte_desc_gather(ctx, dE, dt, dH, B, V, K)
    res = run_everywhere(H, ctx, d, dH, [0, 5, H.pctx_of_width(ctx, 256)])
    assert np.array_equal(assert_all_equal(res).view(np.uint16), oracle.gather(E, t))
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B,V", [(8, 128256), (3, 4099), (1, 1), (5, 1000), (16, 32064)])
def test_softmax_prob_parity_and_width_invariance(H, ctx, B, V):
    rng = np.random.default_rng(V)
    lg = (rng.standard_normal((B, V)) * 3).astype(np.float32)
    tok = rng.integers(0, V, size=B).astype(np.int32)
    tok[0] = int(np.argmax(lg[0]))                       # the greedy token of a row
    if B > 2:
        tok[2] = V + 5                                    # outside the vocabulary -> 0
        lg[1, : V // 2] = -np.inf                         # dead entries
    dl, dt = torch.from_numpy(lg).cuda(), torch.from_numpy(tok).cuda()
    dp = torch.zeros(B, dtype=torch.float32, device="cuda")
    d = vte.vte_desc_softmax_prob(ctx, dl, dt, dp, B, V)
    res = run_everywhere(H, ctx, d, dp, [H.pctx_of_width(ctx, w) for w in (32, 64, 128, 224, 256)])
    p = assert_all_equal(res).view(np.float32)            # same bits on every width
    ref = oracle.softmax_prob(lg, tok)
    assert np.all(np.abs(p - ref) <= 5e-5 * ref + 1e-30), (p, ref)
    if B > 2:
        assert p[2] == 0.0
    vte.vte_desc_destroy(d)


def test_memcpy_and_memset_launches(H, ctx):
    n = 3 * 16384 + 4096 + 16                                # several workgroups and a ragged last one
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (n // 4 + 8,), dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    d = vte.vte_desc_memcpy(ctx, dst, src, n)
    res = []
    for w in (256, 32):
        dst.zero_()
        torch.cuda.synchronize()
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        res.append(dst.cpu().numpy().copy())
    ref = src.cpu().numpy().copy()
    ref[n // 4:] = 0                                         # nothing past the byte count is written
    assert np.array_equal(res[0], ref) and np.array_equal(res[1], ref)
    m = vte.vte_desc_memset32(ctx, dst, 0x3f803f80, n)
    H.run_on(ctx, m, H.pctx_of_width(ctx, 64))
    got = dst.cpu().numpy().view(np.uint32)
    assert np.all(got[:n // 4] == 0x3f803f80) and np.all(got[n // 4:] == 0)
    # as operations of two virtual streams ordered by an event: fill, then copy the filled buffer
    a, b = vte.vte_vstream_create(ctx), vte.vte_vstream_create(ctx)
    out = torch.zeros_like(src)
    fill = vte.vte_desc_memset32(ctx, dst, 0x12345678, n)
    copy = vte.vte_desc_memcpy(ctx, out, dst, n)
    vte.vte_submit(a, fill)
    vte.vte_vstream_wait_event(b, vte.vte_event_record(a))
    vte.vte_token_wait(ctx, vte.vte_submit(b, copy))
    assert np.all(out.cpu().numpy().view(np.uint32)[:n // 4] == 0x12345678)
    for vs in (a, b):
        vte.vte_vstream_destroy(vs)
    for dd in (d, m, fill, copy):
        vte.vte_desc_destroy(dd)


# ---------- MFMA GEMM ---------------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (256, 512, 128), (512, 256, 192), (512, 512, 512), (1024, 768, 1024), (256, 256, 4160)])
def test_gemm_parity_and_width_invariance(H, ctx, M, N, K):
    A = inputs.normal_bf16(0, inputs.T_GEMM_A, (M, K))
    Bm = inputs.normal_bf16(0, inputs.T_GEMM_B, (N, K))
    dA, dB, dC = H.to_dev(A), H.to_dev(Bm), H.dev_empty((M, N))
    d = vte.vte_desc_gemm(ctx, dA, dB, dC, M, N, K)
    res = run_everywhere(H, ctx, d, dC, [H.pctx_of_width(ctx, w) for w in (32, 64, 128, 224, 256)])
    c = assert_all_equal(res).view(np.uint16)
    ref = oracle.gemm_rows(A, Bm, np.arange(M))
    err = np.abs(f64(c) - ref)
    assert np.all(err <= 2.0 ** -8 * np.abs(ref) * (1 + 1e-2) + 1e-2), err.max()
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("K,binades", [(192, 0), (1024, 0), (256, 6)])
def test_gemm_equals_its_emulated_tree_bit_for_bit(H, ctx, K, binades):
    """An output of the GEMM is one chain of matrix-core instructions along K (no split, four 16-wide
    instructions per 64-wide step): the emulated chain of 8-product groups, rounded to bf16 once, must be
    the GPU's bits on sampled rows of a 256 x 512 product."""
    import tree_emulator
    M, N = 256, 512
    A = inputs.normal_bf16(5, inputs.T_GEMM_A, (M, K))
    Bm = inputs.normal_bf16(5, inputs.T_GEMM_B, (N, K))
    if binades:
        Bm = _spread(Bm, 5, binades)
    dA, dB, dC = H.to_dev(A), H.to_dev(Bm), H.dev_empty((M, N))
    d = vte.vte_desc_gemm(ctx, dA, dB, dC, M, N, K)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 64))
    c = H.to_bits(dC)
    rows = np.array([0, 1, 31, 32, 63, 64, 100, 127, 128, 200, 255])
    want = tree_emulator._f32_to_bf16(tree_emulator.gemv_rows_sums(Bm, np.ascontiguousarray(A[rows])))   # [rows, N]
    assert np.array_equal(c[rows], want)
    vte.vte_desc_destroy(d)


@pytest.mark.parametrize("K", [512, 8192])
def test_gemm_full_grid_sampled_rows(H, ctx, K):
    """The co-tenant's own size (8192 x 8192 outputs: 1024 tiles in the XCD-aware order, L2 warm-up
    touches active), checked on sampled rows and columns the oracle computes one by one; bit-equal
    between a 32-CU and the 256-CU pCtx."""
    M = N = 8192
    A = inputs.normal_bf16(0, inputs.T_GEMM_A, (M, K))
    Bm = inputs.normal_bf16(0, inputs.T_GEMM_B, (N, K))
    dA, dB, dC = H.to_dev(A), H.to_dev(Bm), H.dev_empty((M, N))
    d = vte.vte_desc_gemm(ctx, dA, dB, dC, M, N, K)
    outs = []
    for w in ((256, 32) if K == 512 else (256,)):
        dC.fill_(0x7FC1)
        torch.cuda.synchronize()
        H.run_on(ctx, d, H.pctx_of_width(ctx, w))
        outs.append(H.to_bits(dC).copy())
    if len(outs) == 2:
        assert H.mismatched_bits(outs[0], outs[1]) == (0, 0)
    rows = np.array([0, 255, 256, 4095, 4101, 8191] if K == 512 else [3, 8191])
    ref = oracle.gemm_rows(A, Bm, rows)
    err = np.abs(f64(outs[0][rows]) - ref)
    assert np.all(err <= 2.0 ** -8 * np.abs(ref) * (1 + 1e-2) + 1e-2), err.max()
    cols = np.array([0, 257, 8191])                      # columns: rows of the transposed product
    refc = oracle.gemm_rows(Bm, A, cols)                 # [cols, M]
    errc = np.abs(f64(outs[0][:, cols]).T - refc)
    assert np.all(errc <= 2.0 ** -8 * np.abs(refc) * (1 + 1e-2) + 1e-2), errc.max()
    vte.vte_desc_destroy(d)
    del dA, dB, dC
    torch.cuda.empty_cache()


@pytest.mark.parametrize("M,N,K", [(32768, 256, 8192), (8192, 2048, 4096), (2048, 256, 65536)])
def test_gemm_every_output_is_exact_on_small_integers(H, ctx, M, N, K):
    """Small-integer inputs: every partial sum is exact in fp32, so each output must equal the exact
    product rounded once, in every bit, at every width -- also when the operands stream from HBM
    (N = 256) and the kernel waits for its LDS fills, the regime a tolerance test on N(0,1) inputs
    at a compute-bound shape never reaches."""
    A = inputs.int_bf16(41, inputs.T_GEMM_A, (M, K), -8, 8)
    Bm = inputs.int_bf16(41, inputs.T_GEMM_B, (N, K), -8, 8, -2)
    rows = np.array([0, 33, 160, 255, M - 200, M - 1])
    ref_rows = oracle.f64_to_bf16(oracle.gemm_rows(A, Bm, rows))
    dA, dB, dC = H.to_dev(A), H.to_dev(Bm), H.dev_empty((M, N))
    d = vte.vte_desc_gemm(ctx, dA, dB, dC, M, N, K)
    Bf = dB.view(torch.bfloat16).float().t().contiguous()
    ref = torch.cat([torch.matmul(dA[r0:r0 + 4096].view(torch.bfloat16).float(), Bf).to(torch.bfloat16).view(torch.int16)
                     for r0 in range(0, M, 4096)])
    assert np.array_equal(ref[torch.from_numpy(rows).cuda()].cpu().numpy().view(np.uint16), ref_rows)   # the oracle agrees with the exact product
    for w in (256, 224, 128, 32):
        for rep in range(2):
            dC.fill_(0x7FC1)
            torch.cuda.synchronize()
            H.run_on(ctx, d, H.pctx_of_width(ctx, w))
            assert int((dC != ref).sum()) == 0, (w, rep)
    vte.vte_desc_destroy(d)
    del dA, dB, dC, ref
    torch.cuda.empty_cache()


def test_gemm_operand_beyond_2_to_the_31_elements(H, ctx):
    """Maximum sizes: A = 65536 x 32832 bf16 (2.15e9 elements, 4.3 GB; element offsets pass 2^31 at row
    65408).  Small-integer inputs keep every partial sum exact, so the sampled rows (both ends, both sides
    of that row) equal the oracle bit for bit and every output equals the exact float32 product."""
    M, N, K = 65536, 256, 32832
    A = inputs.int_bf16(31, inputs.T_GEMM_A, (M, K), -8, 8)
    Bm = inputs.int_bf16(31, inputs.T_GEMM_B, (N, K), -8, 8, -2)
    edge = (1 << 31) // K
    rows = np.unique(np.concatenate([np.arange(4), np.arange(edge - 3, edge + 3), np.arange(M - 4, M)]))
    assert rows.max() < M and edge + 3 <= M
    ref = oracle.f64_to_bf16(oracle.gemm_rows(A, Bm, rows))
    dA, dB, dC = H.to_dev(A), H.to_dev(Bm), H.dev_empty((M, N))
    d = vte.vte_desc_gemm(ctx, dA, dB, dC, M, N, K)
    H.run_on(ctx, d, H.pctx_of_width(ctx, 256))
    assert np.array_equal(dC[torch.from_numpy(rows).cuda()].cpu().numpy().view(np.uint16), ref)
    Bf = dB.view(torch.bfloat16).float().t().contiguous()
    for r0 in range(0, M, 8192):                           # the exact float32 product, a slab at a time
        whole = torch.matmul(dA[r0:r0 + 8192].view(torch.bfloat16).float(), Bf).to(torch.bfloat16).view(torch.int16)
        assert torch.equal(whole, dC[r0:r0 + 8192]), r0
    vte.vte_desc_destroy(d)
    del dA, dB, dC
    torch.cuda.empty_cache()


# ---------- the decode chain --------------------------------------------------------------------------
@pytest.fixture(scope="module")
def small_chain(H, ctx):
    shp = inputs.DecodeShapes(D=512, Nqkv=768, F=1792, V=4099)
    w = inputs.decode_weights(11, shp)
    for k in ("Wqkv", "Wo", "Wgu", "Wd"):                # keep activations O(1) through the short chain
        w[k] = inputs.normal_bf16(11, 100 + len(k), w[k].shape, 0.0, 1.5 * w[k].shape[1] ** -0.5)
    return shp, w, H.upload_weights(w)


@pytest.mark.parametrize("B", [1, 3, 8, 16])
def test_chain_teacher_forced_per_operator(H, ctx, small_chain, B):
    shp, w, wd = small_chain
    ch = H.DecodeChain(ctx, wd, shp, B, want_logits=True)
    tok = inputs.tokens(11, inputs.T_TOK0, B, shp.V)
    p256 = H.pctx_of_width(ctx, 256)
    near = 0
    for step in range(6):
        ch.set_tokens(tok)
        ch.run_step_on(p256)
        s = ch.snapshot()
        o = oracle.decode_step(w, tok, shp, want_logits=True)
        assert np.array_equal(s["h0"], o["h0"])
        # each operator is checked on the GPU's own inputs, so errors do not compound
        bf16_close(s["n"], oracle.rmsnorm(s["h0"], w["gamma"]), "n")
        bf16_close(s["qkv"], oracle.gemv(w["Wqkv"], s["n"]), "qkv")
        bf16_close(s["o"], oracle.gemv(w["Wo"], np.ascontiguousarray(s["qkv"][:, :shp.D])), "o")
        bf16_close(s["act"], oracle.gemv_silu_mul(w["Wgu"], s["o"]), "act")
        bf16_close(s["d"], oracle.gemv(w["Wd"], s["act"]), "d")
        lg, t_ref, margin = oracle.lmhead_argmax(w["Wlm"], s["d"])
        eps_logit = np.abs(s["logits"].astype(np.float64) - lg).max()
        assert eps_logit < 1e-3
        for b in range(B):
            if s["next"][b] != t_ref[b]:
                assert margin[b] <= 2 * eps_logit
                near += 1
        tok = o["next"]                                   # teacher forcing with the oracle's stream
    assert near <= 1
    ch.close()


def test_full_size_chain_in_the_benchmark_configuration(H, ctx):
    """Llama-8B shapes (V = 128256), batch 8, 32 and 64, the launch configuration bench.py times
    (step boundary fused, pipelined virtual stream): every operator of a step against the oracle on
    the GPU's own inputs, the greedy tokens of three free-running steps, and the same tokens and bits
    from the unfused chain launched explicitly on a 64-CU pCtx."""
    shp = inputs.DecodeShapes()
    w = inputs.decode_weights(0, shp)
    wd = H.upload_weights(w)
    p64 = H.pctx_of_width(ctx, 64)
    for B in (8, 32, 64):
        tok0 = inputs.tokens(0, inputs.T_TOK0, B, shp.V)
        plain = H.DecodeChain(ctx, wd, shp, B, want_logits=True)
        plain.set_tokens(tok0)
        plain.run_step_on(p64)
        s = plain.snapshot()
        assert np.array_equal(s["h0"], w["E"][tok0])
        bf16_close(s["n"], oracle.rmsnorm(s["h0"], w["gamma"]), "n")
        bf16_close(s["qkv"], oracle.gemv(w["Wqkv"], s["n"]), "qkv")
        bf16_close(s["o"], oracle.gemv(w["Wo"], np.ascontiguousarray(s["qkv"][:, :shp.D])), "o")
        bf16_close(s["act"], oracle.gemv_silu_mul(w["Wgu"], s["o"]), "act")
        bf16_close(s["d"], oracle.gemv(w["Wd"], s["act"]), "d")
        lg, t_ref, margin = oracle.lmhead_argmax(w["Wlm"], s["d"])
        eps_logit = np.abs(s["logits"].astype(np.float64) - lg).max()
        assert eps_logit < 1e-3
        assert all(s["next"][b] == t_ref[b] or margin[b] <= 2 * eps_logit for b in range(B))
        # three free-running steps: unfused, explicit launches vs the benchmark's fused, policy-bound form
        toks_plain = []
        t = tok0
        for _ in range(3):
            plain.set_tokens(t)
            plain.run_step_on(p64)
            t = plain.snapshot()["next"]
            toks_plain.append(t.copy())
        fused = H.DecodeChain(ctx, wd, shp, B, feedback=True, fused_gather=True, fused_argmax=True)
        fused.set_tokens(tok0)
        vs = vte.vte_vstream_create(ctx)
        vte.vte_token_wait(ctx, fused.submit_burst(vs, 3))
        assert np.array_equal(fused.tok.cpu().numpy(), toks_plain[-1])
        assert np.array_equal(H.to_bits(fused.d), plain.snapshot()["d"])          # same bits in the last step's activations
        vte.vte_vstream_destroy(vs)
        plain.close()
        fused.close()
    del wd
    torch.cuda.empty_cache()


def test_fused_gather_norm_equals_two_launches(H, ctx, small_chain):
    shp, w, wd = small_chain
    B = 5
    tok = inputs.tokens(9, inputs.T_TOK0, B, shp.V)
    snaps = []
    for fused in (False, True):
        ch = H.DecodeChain(ctx, wd, shp, B, want_logits=True, fused_gather=fused)
        assert len(ch.order) == (7 if fused else 8)
        ch.set_tokens(tok)
        ch.run_step_on(H.pctx_of_width(ctx, 64 if fused else 256))
        snaps.append(ch.snapshot())
        ch.close()
    for k in ("h0", "n", "qkv", "o", "act", "d", "next"):
        assert np.array_equal(snaps[0][k], snaps[1][k]), k
    assert np.array_equal(snaps[0]["logits"].view(np.uint32), snaps[1]["logits"].view(np.uint32))
    assert np.array_equal(snaps[0]["h0"], w["E"][tok])


@pytest.mark.parametrize("B", [3, 8, 16])
def test_fused_step_boundary_equals_finish_then_gather_norm(H, ctx, small_chain, B):
    """A burst whose step boundary is one launch (finish the token, gather, normalise) leaves the
    same tokens and the same activations as the chain with a separate finish and gather+norm."""
    shp, w, wd = small_chain
    tok = inputs.tokens(13, inputs.T_TOK0, B, shp.V)
    steps = 6
    snaps, toks = [], []
    for fused in (False, True):
        ch = H.DecodeChain(ctx, wd, shp, B, want_logits=True, feedback=True, fused_gather=True, fused_argmax=fused)
        if fused:
            assert len(ch.order_next) == 6 and ch.order_next[0] == "boundary"
        ch.set_tokens(tok)
        vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
        vte.vte_vstream_pin(vs, H.pctx_of_width(ctx, 64 if fused else 256))
        ch.submit_burst(vs, steps)
        vte.vte_vstream_sync(vs)
        snaps.append(ch.snapshot())
        toks.append(ch.tok.cpu().numpy().copy())
        vte.vte_vstream_destroy(vs)
        ch.close()
    assert np.array_equal(toks[0], toks[1])
    for k in ("h0", "n", "qkv", "o", "act", "d"):
        assert np.array_equal(snaps[0][k], snaps[1][k]), k
    assert np.array_equal(snaps[0]["logits"].view(np.uint32), snaps[1]["logits"].view(np.uint32))
    # the tokens really moved: six steps from random start tokens do not stand still
    assert not np.array_equal(toks[0], tok)


def test_fused_step_boundary_rejects_a_non_lmhead_descriptor(H, ctx, small_chain):
    shp, w, wd = small_chain
    ch = H.DecodeChain(ctx, wd, shp, 2, fused_gather=True)
    with pytest.raises(vte.VteError):
        vte.vte_desc_rmsnorm_gather_argmax(ctx, wd["E"], ch.desc["qkv"], None, wd["gamma"], ch.n, None, shp.V, shp.D, 1e-6)
    ch.close()


@pytest.fixture(scope="module")
def chain_4096(H, ctx):
    """Hidden size 4096 (what the fused QKV launch is built for), everything else small."""
    shp = inputs.DecodeShapes(D=4096, Nqkv=6144, F=1024, V=4099)
    w = inputs.decode_weights(12, shp)
    for k in ("Wqkv", "Wo", "Wgu", "Wd"):
        w[k] = inputs.normal_bf16(12, 100 + len(k), w[k].shape, 0.0, 1.5 * w[k].shape[1] ** -0.5)
    return shp, w, H.upload_weights(w)


@pytest.mark.parametrize("B,N", [(8, 6144), (1, 6144), (16, 6144), (11, 4096), (3, 1000), (16, 16)])
def test_gemv_with_the_step_boundary_in_its_prologue(H, ctx, chain_4096, B, N):
    """vte_desc_gemv_rmsnorm_gather: tokens -> embedding rows -> RMSNorm -> GEMV in one launch.  Against the
    oracle; against the two launches it replaces (gather+norm, then the GEMV with the same plan): every
    bit of the gathered rows, the normalised rows and the output; and on every pCtx."""
    shp, w, wd = chain_4096
    K, V = shp.D, shp.V
    tok = inputs.tokens(21 + B, inputs.T_TOK0, B, V)
    tok[0] = V - 1                                                # the last row of the table
    W = np.ascontiguousarray(w["Wqkv"][:N])
    dW, dtok = H.to_dev(W), torch.from_numpy(tok.astype(np.int32)).cuda()
    Y, h, n = H.dev_empty((B, N)), H.dev_empty((B, K)), H.dev_empty((B, K))
    fused = vte.vte_desc_gemv_rmsnorm_gather(ctx, dW, wd["E"], dtok, wd["gamma"], Y, h, n, B, V, N, K, 1e-6)
    info = vte.vte_desc_info(fused)
    assert info.kernel == vte.VTE_K_GEMV_NORM and list(info.block) == [256, 1, 1]
    res = run_everywhere(H, ctx, fused, Y)
    y_f = assert_all_equal(res).view(np.uint16)
    h_f, n_f = H.to_bits(h), H.to_bits(n)
    # the two launches it replaces
    Y2, h2, n2 = H.dev_empty((B, N)), H.dev_empty((B, K)), H.dev_empty((B, K))
    d1 = vte.vte_desc_rmsnorm_gather(ctx, wd["E"], dtok, wd["gamma"], n2, h2, B, V, K, 1e-6)
    pl = vte.vte_gemv_plan()
    pl.kind, pl.batch_tile, pl.ksteps, pl.prefetch, pl.max_waves, pl.groups = vte.VTE_GEMV_MFMA, 16, 8, 2, 4, 1
    pl.rows = 32 if (N + 15) // 16 > 256 else 16
    d2 = vte.vte_desc_gemv_planned(ctx, dW, n2, Y2, B, N, K, vte.VTE_EPI_NONE, pl)
    p = H.pctx_of_width(ctx, 128)
    H.run_on(ctx, d1, p)
    H.run_on(ctx, d2, p)
    assert np.array_equal(h_f, H.to_bits(h2)) and np.array_equal(h_f, w["E"][tok])
    assert np.array_equal(n_f, H.to_bits(n2))
    assert np.array_equal(y_f, H.to_bits(Y2))
    # the oracle, each operator on the GPU's own input
    bf16_close(n_f, oracle.rmsnorm(w["E"][tok], w["gamma"], 1e-6), "fused norm, batch %d" % B)
    bf16_close(y_f, oracle.gemv(W, n_f), "fused gemv, batch %d, N %d" % (B, N))
    for d in (fused, d1, d2):
        vte.vte_desc_destroy(d)


@pytest.mark.parametrize("B", [1, 4, 8, 16])
def test_chain_with_the_boundary_in_the_qkv_launch_teacher_forced(H, ctx, chain_4096, B):
    """The five-launch step against the oracle, operator by operator on the GPU's own inputs, six
    teacher-forced steps; the first step takes its tokens from the buffer, the later ones finish them
    from the LM head's candidates (the token buffer is overwritten with the oracle's to check that)."""
    shp, w, wd = chain_4096
    ch = H.DecodeChain(ctx, wd, shp, B, want_logits=True, feedback=True, fused_gather=True, fused_argmax=True, fused_qkv=True)
    vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
    tok = inputs.tokens(23, inputs.T_TOK0, B, shp.V)
    ch.set_tokens(tok)
    near = 0
    for step in range(6):
        for k in (ch.order_first if step == 0 else ch.order_next):
            last = vte.vte_submit(vs, ch.desc[k])
        vte.vte_token_wait(ctx, last)
        s = ch.snapshot()
        if step > 0:                                       # the tokens the launch finished from the candidates
            assert np.array_equal(ch.tok.cpu().numpy(), prev_next)
            tok = prev_next
        o = oracle.decode_step(w, tok, shp, want_logits=True)
        assert np.array_equal(s["h0"], o["h0"])
        bf16_close(s["n"], oracle.rmsnorm(s["h0"], w["gamma"]), "n")
        bf16_close(s["qkv"], oracle.gemv(w["Wqkv"], s["n"]), "qkv")
        bf16_close(s["o"], oracle.gemv(w["Wo"], np.ascontiguousarray(s["qkv"][:, :shp.D])), "o")
        bf16_close(s["act"], oracle.gemv_silu_mul(w["Wgu"], s["o"]), "act")
        bf16_close(s["d"], oracle.gemv(w["Wd"], s["act"]), "d")
        lg, t_ref, margin = oracle.lmhead_argmax(w["Wlm"], s["d"])
        eps_logit = np.abs(s["logits"].astype(np.float64) - lg).max()
        assert eps_logit < 1e-3
        # what the next launch must find: the greedy token of these logits (ties to the lowest index)
        prev_next = np.array([int(np.flatnonzero(r == r.max())[0]) for r in s["logits"]], dtype=np.int32)
        for b in range(B):
            if prev_next[b] != t_ref[b]:
                assert margin[b] <= 2 * eps_logit
                near += 1
    assert near <= 1
    vte.vte_vstream_destroy(vs)
    ch.close()


@pytest.mark.parametrize("B", [3, 4, 8, 16])
def test_chain_with_the_boundary_in_the_qkv_launch_equals_the_six_launch_chain(H, ctx, chain_4096, B):
    """Five launches per step (token finish, gather and RMSNorm in the QKV launch's prologue) leave the same
    tokens, activations and logits as the chain whose boundary is a launch of its own, step after step
    (from batch 3 the stand-alone QKV launch runs the same matrix-core plan; below that it is the
    dot-product kind, another tree)."""
    shp, w, wd = chain_4096
    tok = inputs.tokens(17, inputs.T_TOK0, B, shp.V)
    steps = 6
    snaps, toks = [], []
    for fused in (False, True):
        ch = H.DecodeChain(ctx, wd, shp, B, want_logits=True, feedback=True, fused_gather=True, fused_argmax=True, fused_qkv=fused)
        if fused:
            assert ch.order_next == ["qkv_next", "o", "gateup", "down", "lmhead"] and ch.order_first[0] == "qkv_first"
        ch.set_tokens(tok)
        vs = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
        vte.vte_vstream_pin(vs, H.pctx_of_width(ctx, 64 if fused else 256))
        ch.submit_burst(vs, steps)
        vte.vte_vstream_sync(vs)
        snaps.append(ch.snapshot())
        toks.append(ch.tok.cpu().numpy().copy())
        vte.vte_vstream_destroy(vs)
        ch.close()
    assert np.array_equal(toks[0], toks[1])
    for k in ("h0", "n", "qkv", "o", "act", "d"):
        assert np.array_equal(snaps[0][k], snaps[1][k]), k
    assert np.array_equal(snaps[0]["logits"].view(np.uint32), snaps[1]["logits"].view(np.uint32))
    assert not np.array_equal(toks[0], tok)


def test_fused_qkv_launch_rejects_what_it_is_not_built_for(H, ctx, chain_4096, small_chain):
    shp, w, wd = chain_4096
    Y = H.dev_empty((17, 64))
    tok = torch.zeros(17, dtype=torch.int32, device="cuda")
    with pytest.raises(vte.VteError):                             # batch above 16
        vte.vte_desc_gemv_rmsnorm_gather(ctx, wd["Wqkv"], wd["E"], tok, wd["gamma"], Y, None, None, 17, shp.V, 64, shp.D, 1e-6)
    with pytest.raises(vte.VteError):                             # fewer than one tile of outputs
        vte.vte_desc_gemv_rmsnorm_gather(ctx, wd["Wqkv"], wd["E"], tok, wd["gamma"], Y, None, None, 8, shp.V, 8, shp.D, 1e-6)
    s_shp, s_w, s_wd = small_chain
    with pytest.raises(vte.VteError):                             # another hidden size
        vte.vte_desc_gemv_rmsnorm_gather(ctx, s_wd["Wqkv"], s_wd["E"], tok, s_wd["gamma"], Y, None, None, 8, s_shp.V, 64, s_shp.D, 1e-6)
    ch = H.DecodeChain(ctx, wd, shp, 2, fused_gather=True)
    with pytest.raises(vte.VteError):                             # candidates must come from an LM-head descriptor
        vte.vte_desc_gemv_rmsnorm_gather_argmax(ctx, wd["Wqkv"], wd["E"], ch.desc["qkv"], None, wd["gamma"], ch.qkv, None, None,
                                                shp.V, shp.Nqkv, shp.D, 1e-6)
    ch.close()


def test_chain_bits_do_not_depend_on_allocation(H, ctx, small_chain):
    shp, w, wd = small_chain
    B = 8
    ch = H.DecodeChain(ctx, wd, shp, B, want_logits=True)
    tok0 = inputs.tokens(3, inputs.T_TOK0, B, shp.V)
    rng = np.random.default_rng(0)
    ids = all_pctx(ctx)

    def replay(choice):
        toks, tok = [], tok0
        for step in range(8):
            ch.set_tokens(tok)
            ch.run_step_on(choice(step))
            s = ch.snapshot()
            toks.append((s["next"].copy(), s["logits"].copy(), s["d"].copy()))
            tok = s["next"]
        return toks

    base = replay(lambda s: H.pctx_of_width(ctx, 256))
    for trial in range(4):                                # a different pCtx for every launch
        other = replay(lambda s: [int(rng.choice(ids)) for _ in ch.order])
        for (t0, l0, d0), (t1, l1, d1) in zip(base, other):
            assert np.array_equal(t0, t1)
            assert np.array_equal(l0.view(np.uint32), l1.view(np.uint32))
            assert np.array_equal(d0, d1)
    ch.close()

