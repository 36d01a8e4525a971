"""Host logic of the runtime driven through the C ABI with the fake backend (no GPU).

Covers the statements of Sec. 4.2-4.5: pool shape and the printed remainder
example, conflict rules, the four pCtx states, token chains, readiness before
binding, unchanged descriptors, validated proposals, failed submissions,
reservation and gate closing, pipelined device-side edges.
"""
import ctypes as C
import os
import re

import pytest

from paper_2603_15042_amd import vte

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 0x100000  # fake, 16-byte aligned "device" addresses: never dereferenced on the fake backend


def make_ctx(mode=vte.VTE_MODE_STRICT, total=256, leaf=32, lookahead=16, remainders=vte.VTE_REMAINDERS_ALL):
    cfg = vte.vte_pool_cfg_default()
    cfg.backend = vte.VTE_BACKEND_FAKE
    cfg.with_remainders = remainders
    cfg.total_cus = total
    cfg.leaf_cus = leaf
    cfg.mode = mode
    cfg.lookahead = lookahead
    return vte.vte_init(0, cfg)


@pytest.fixture
def ctx():
    c = make_ctx()
    yield c
    vte.vte_shutdown(c)


@pytest.fixture
def pctx():
    c = make_ctx(vte.VTE_MODE_PIPELINED)
    yield c
    vte.vte_shutdown(c)


def norm_desc(c, rows=8, cols=1024):
    return vte.vte_desc_rmsnorm(c, A, A + 0x1000, A + 0x2000, rows, cols, 1e-6)


def infos(c):
    return [vte.vte_pool_info(c, i) for i in range(vte.vte_pool_count(c))]


def mask_int(info):
    return sum(int(w) << (32 * i) for i, w in enumerate(info.mask))


# ---------- the boundary ---------------------------------------------------------------
def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "vte.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(vte_[a-z_0-9]+)\s*\(", text))
    declared -= {"vte_policy_vtbl"}
    assert len(declared) > 50
    lib = vte.load()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(vte.EXPORTS)


def test_errors_are_codes_not_exceptions_across_the_abi():
    lib = vte.load()
    assert lib.vte_pool_count(None, None) == vte.VTE_EINVAL
    assert b"null" in lib.vte_last_error()
    cfg = vte.vte_pool_cfg_default()
    cfg.backend = vte.VTE_BACKEND_FAKE
    cfg.layout = 7
    with pytest.raises(vte.VteError) as e:
        vte.vte_init(0, cfg)
    assert e.value.code == vte.VTE_EINVAL


# ---------- pool (Sec. 4.3) -----------------------------------------------------------------
def test_pool_shape_on_mi355x_numbers(ctx):
    ps = infos(ctx)
    nodes = [p for p in ps if p.kind == vte.VTE_PCTX_NODE]
    rems = [p for p in ps if p.kind == vte.VTE_PCTX_REMAINDER]
    assert sorted(p.width for p in nodes) == [32] * 8 + [64] * 4 + [128] * 2 + [256]
    assert sorted(p.width for p in rems) == [192] * 4 + [224] * 8
    assert len(ps) == 27
    full = (1 << 256) - 1
    for p in nodes:
        assert bin(mask_int(p)).count("1") == p.width
        if p.child[0] >= 0:  # internal node covers the union of its children
            assert mask_int(p) == mask_int(ps[p.child[0]]) | mask_int(ps[p.child[1]])
            assert mask_int(ps[p.child[0]]) & mask_int(ps[p.child[1]]) == 0
        if p.parent < 0:
            assert mask_int(p) == full and p.remainder == -1
        else:  # remainder spans exactly every other CU
            assert mask_int(ps[p.remainder]) == full & ~mask_int(p)
    # the two halves complement each other without a duplicate allocation
    halves = [p for p in nodes if p.width == 128]
    assert halves[0].remainder == halves[1].id and halves[1].remainder == halves[0].id
    # a leaf is a run of 32 consecutive mask bits (4 CUs on each of the 8 XCDs on the device)
    leaf = [p for p in nodes if p.width == 32][3]
    m = mask_int(leaf)
    assert m == ((1 << 32) - 1) << (m & -m).bit_length() - 1


def test_bounded_pool_keeps_one_remainder_per_level():
    cfg = vte.vte_pool_cfg_default()
    assert cfg.with_remainders == vte.VTE_REMAINDERS_PER_LEVEL       # the default stays under the queue limit
    c = make_ctx(remainders=vte.VTE_REMAINDERS_PER_LEVEL)
    try:
        ps = infos(c)
        assert len(ps) == 17
        rems = [p for p in ps if p.kind == vte.VTE_PCTX_REMAINDER]
        assert sorted(p.width for p in rems) == [192, 224]
        assert sorted(set(p.width for p in ps)) == [32, 64, 128, 192, 224, 256]
        for r in rems:                                                 # still the exact complement of its node
            assert mask_int(r) == ((1 << 256) - 1) & ~mask_int(ps[r.parent])
        for a in ps:
            for b in ps:
                assert vte.vte_pool_conflict(c, a.id, b.id) == bool(mask_int(a) & mask_int(b))
    finally:
        vte.vte_shutdown(c)
    c = make_ctx(remainders=vte.VTE_REMAINDERS_NONE)
    assert vte.vte_pool_count(c) == 15
    vte.vte_shutdown(c)


def test_pool_reproduces_the_papers_remainder_example():
    total, node_w, rem_w = [int(v) for v in open(os.path.join(ROOT, "tests", "golden", "pool_remainder_example.txt"))
                            .read().split("\n")[1].split()]
    c = make_ctx(total=total, leaf=node_w)
    try:
        ps = infos(c)
        leaf = next(p for p in ps if p.kind == vte.VTE_PCTX_NODE and p.width == node_w)
        assert ps[leaf.remainder].width == rem_w
        assert bin(mask_int(ps[leaf.remainder])).count("1") == rem_w
        assert mask_int(ps[leaf.remainder]) & mask_int(leaf) == 0
    finally:
        vte.vte_shutdown(c)


@pytest.mark.parametrize("total,leaf", [(256, 32), (256, 64), (132, 8), (64, 16)])
def test_conflict_by_traversal_equals_mask_intersection(total, leaf):
    c = make_ctx(total=total, leaf=leaf)
    try:
        ps = infos(c)
        for a in ps:
            for b in ps:
                assert vte.vte_pool_conflict(c, a.id, b.id) == bool(mask_int(a) & mask_int(b)), (a.id, b.id)
    finally:
        vte.vte_shutdown(c)


def test_lease_excludes_ancestors_descendants_and_remainder_rules(ctx):
    ps = infos(ctx)
    d = norm_desc(ctx)
    n64 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 64, 1)
    t = vte.vte_bind_and_launch(ctx, d, n64)
    assert vte.vte_pool_info(ctx, n64).state == vte.VTE_PCTX_LEASED
    busy, free = [], []
    for p in ps:
        if p.id == n64:
            continue
        try:
            tt = vte.vte_bind_and_launch(ctx, d, p.id)
            vte.vte_fake_complete(ctx, tt)
            vte.vte_token_wait(ctx, tt)
            free.append(p.id)
        except vte.VteError as e:
            assert e.code == vte.VTE_EBUSY
            busy.append(p.id)
    m = mask_int(ps[n64])
    assert sorted(busy) == sorted(p.id for p in ps if p.id != n64 and mask_int(p) & m)
    assert ps[n64].remainder in free            # the 192-CU remainder runs beside the node
    assert ps[n64].parent in busy and ps[n64].child[0] in busy
    vte.vte_fake_complete(ctx, t)
    vte.vte_token_wait(ctx, t)
    # leasing the remainder excludes the node's ancestors and the sibling branches, not its subtree
    r = ps[n64].remainder
    t = vte.vte_bind_and_launch(ctx, d, r)
    for p in ps:
        if p.id == r:
            continue
        inside = p.kind == vte.VTE_PCTX_NODE and (mask_int(p) & ~m) == 0
        try:
            tt = vte.vte_bind_and_launch(ctx, d, p.id)
            vte.vte_fake_complete(ctx, tt)
            vte.vte_token_wait(ctx, tt)
            assert inside, p.id
        except vte.VteError as e:
            assert e.code == vte.VTE_EBUSY and not inside
    vte.vte_fake_complete(ctx, t)
    vte.vte_token_wait(ctx, t)
    st = vte.vte_stats(ctx)
    assert st.lease_conflicts > 0 and st.completed == st.submitted


# ---------- pCtx lifecycle -------------------------------------------------------------------
def test_idle_leased_draining_idle(ctx):
    d = norm_desc(ctx)
    root = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 256)
    assert vte.vte_pool_info(ctx, root).state == vte.VTE_PCTX_IDLE
    t1 = vte.vte_bind_and_launch(ctx, d, root)
    t2 = vte.vte_bind_and_launch(ctx, d, root)     # lease reused
    i = vte.vte_pool_info(ctx, root)
    assert (i.state, i.outstanding, i.gate_open) == (vte.VTE_PCTX_LEASED, 2, 1)
    vte.vte_pctx_close_gate(ctx, root)
    i = vte.vte_pool_info(ctx, root)
    assert (i.state, i.gate_open) == (vte.VTE_PCTX_DRAINING, 0)
    with pytest.raises(vte.VteError) as e:          # no new admissions while draining
        vte.vte_bind_and_launch(ctx, d, root)
    assert e.value.code == vte.VTE_EBUSY
    vte.vte_fake_complete(ctx, t1)
    vte.vte_token_wait(ctx, t1)
    assert vte.vte_pool_info(ctx, root).state == vte.VTE_PCTX_DRAINING   # submitted work continues
    assert not vte.vte_token_query(ctx, t2)
    vte.vte_fake_complete(ctx, t2)
    vte.vte_token_wait(ctx, t2)
    i = vte.vte_pool_info(ctx, root)
    assert (i.state, i.outstanding, i.gate_open) == (vte.VTE_PCTX_IDLE, 0, 1)
    st = vte.vte_stats(ctx)
    assert st.leases_opened == 1 and st.leases_reused == 1 and st.gates_closed == 1


def test_reservation_excludes_unrelated_and_survives_use(ctx):
    d = norm_desc(ctx)
    lat = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
    n64 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 64, 0)
    ps = infos(ctx)
    vte.vte_pctx_reserve(ctx, n64, lat)
    assert vte.vte_pool_info(ctx, n64).state == vte.VTE_PCTX_RESERVED
    for other in (n64, ps[n64].parent, ps[n64].child[0]):   # explicit (unrelated) launches are shut out
        with pytest.raises(vte.VteError) as e:
            vte.vte_bind_and_launch(ctx, d, other)
        assert e.value.code == vte.VTE_EBUSY
    t = vte.vte_bind_and_launch(ctx, d, ps[n64].remainder)  # the rest of the device stays usable
    vte.vte_vstream_pin(lat, n64)
    tok = vte.vte_submit(lat, d)
    vte.vte_dispatcher_quiesce(ctx)
    assert vte.vte_pool_info(ctx, n64).state == vte.VTE_PCTX_LEASED      # owner dispatches without waiting
    vte.vte_fake_complete(ctx, tok)
    vte.vte_token_wait(ctx, tok)
    assert vte.vte_pool_info(ctx, n64).state == vte.VTE_PCTX_RESERVED    # standing reservation
    vte.vte_pctx_unreserve(ctx, n64)
    assert vte.vte_pool_info(ctx, n64).state == vte.VTE_PCTX_IDLE
    vte.vte_fake_complete(ctx, t)
    vte.vte_token_wait(ctx, t)


def test_lookahead_reclamation_drains_then_reserves(ctx):
    d = norm_desc(ctx)
    lat = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY)
    be = vte.vte_vstream_create(ctx, vte.VTE_CLASS_BEST_EFFORT)
    ps = infos(ctx)
    root = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 256)
    vte.vte_vstream_pin(be, root)
    t_be = vte.vte_submit(be, d)
    vte.vte_dispatcher_quiesce(ctx)
    assert vte.vte_pool_info(ctx, root).state == vte.VTE_PCTX_LEASED
    h = vte.vte_hint(vte.vte_vstream_id(lat), 128, 1e-3, 0.0)
    vte.vte_hint_submit(ctx, h)          # default Prepare: close overlapping gates, reserve a 128
    assert vte.vte_pool_info(ctx, root).state == vte.VTE_PCTX_DRAINING
    target = [p.id for p in infos(ctx) if p.reserved_for == vte.vte_vstream_id(lat)]
    assert len(target) == 1 and ps[target[0]].width == 128
    assert vte.vte_pool_info(ctx, target[0]).state == vte.VTE_PCTX_IDLE  # pending until the drain ends
    t_be2 = vte.vte_submit(be, d)        # new best-effort work is not admitted meanwhile
    vte.vte_dispatcher_quiesce(ctx)
    assert len([e for e in vte.vte_fake_log(ctx)]) == 1
    vte.vte_fake_complete(ctx, t_be)
    vte.vte_token_wait(ctx, t_be)
    vte.vte_dispatcher_quiesce(ctx)
    assert vte.vte_pool_info(ctx, target[0]).state == vte.VTE_PCTX_RESERVED
    assert vte.vte_pool_info(ctx, root).state == vte.VTE_PCTX_IDLE
    # the pinned best-effort op now conflicts with the reservation and stays ready
    assert not vte.vte_token_query(ctx, t_be2)
    vte.vte_vstream_pin(be, ps[target[0]].remainder)
    vte.vte_dispatcher_quiesce(ctx)
    log = vte.vte_fake_log(ctx)
    assert log[-1].token == t_be2 and log[-1].pctx == ps[target[0]].remainder
    vte.vte_fake_complete(ctx, t_be2)
    vte.vte_token_wait(ctx, t_be2)


# ---------- tokens and readiness (Sec. 4.2, 4.4) ----------------------------------------------
def test_empty_stream_is_satisfied_and_tail_chains(ctx):
    vs = vte.vte_vstream_create(ctx)
    vte.vte_vstream_sync(vs)                       # empty stream: returns at once
    assert vte.vte_token_query(ctx, 0)
    d = norm_desc(ctx)
    toks = [vte.vte_submit(vs, d) for _ in range(4)]
    assert toks == sorted(toks) and len(set(toks)) == 4
    vte.vte_dispatcher_quiesce(ctx)
    log = vte.vte_fake_log(ctx)
    assert [e.token for e in log] == toks[:1]      # strict: successors wait for observed completion
    for i, t in enumerate(toks):
        assert not vte.vte_token_query(ctx, t)
        vte.vte_fake_complete(ctx, t)
        vte.vte_token_wait(ctx, t)
        vte.vte_dispatcher_quiesce(ctx)
        assert [e.token for e in vte.vte_fake_log(ctx)] == toks[:min(i + 2, 4)]
    vte.vte_vstream_sync(vs)
    with pytest.raises(vte.VteError):
        vte.vte_token_query(ctx, 10 ** 9)           # never issued


def test_cross_stream_dependency_is_a_fixed_completion_point(ctx):
    a, b = vte.vte_vstream_create(ctx), vte.vte_vstream_create(ctx)
    d = norm_desc(ctx)
    n0 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 0)
    n1 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 1)
    vte.vte_vstream_pin(a, n0)
    vte.vte_vstream_pin(b, n1)
    ta1 = vte.vte_submit(a, d)
    tb = vte.vte_submit_after(b, d, [ta1])          # waits for the point captured now ...
    ta2 = vte.vte_submit(a, d)                      # ... a later op on `a` cannot retarget it
    vte.vte_dispatcher_quiesce(ctx)
    assert [e.token for e in vte.vte_fake_log(ctx)] == [ta1]
    vte.vte_fake_complete(ctx, ta1)
    vte.vte_token_wait(ctx, ta1)
    vte.vte_dispatcher_quiesce(ctx)
    assert sorted(e.token for e in vte.vte_fake_log(ctx)) == sorted([ta1, tb, ta2])  # tb did not wait for ta2
    for t in (tb, ta2):
        vte.vte_fake_complete(ctx, t)
    vte.vte_device_sync(ctx)


def test_descriptor_is_submitted_unchanged(ctx):
    vs = vte.vte_vstream_create(ctx)
    W, X, Y = A, A + 0x4000000, A + 0x5000000
    d = vte.vte_desc_gemv(ctx, W, X, Y, 4, 4096, 4096, vte.VTE_EPI_NONE)
    v0 = vte.vte_desc_info(d)
    args0 = vte.vte_desc_args(d)
    ptrs = [int.from_bytes(args0[i:i + 8], "little") for i in (0, 8, 16)]
    assert ptrs == [W, X, Y]                        # pointer values copied by value
    vte.vte_fake_set_autocomplete(ctx, 1)
    toks = [vte.vte_submit(vs, d) for _ in range(6)]
    vte.vte_vstream_sync(vs)
    v1 = vte.vte_desc_info(d)
    assert (v0.hash, list(v0.grid), list(v0.block), v0.lds_bytes) == (v1.hash, list(v1.grid), list(v1.block), v1.lds_bytes)
    assert vte.vte_desc_args(d) == args0
    log = vte.vte_fake_log(ctx)
    assert [e.token for e in log] == toks
    assert all(e.desc_hash == v0.hash for e in log)  # what the backend saw, every time


def test_structure_depends_on_shape_only():
    # same shape -> same grid/block/LDS whatever the pool looks like
    views = []
    for total, leaf in ((256, 32), (64, 16), (132, 8)):
        c = make_ctx(total=total, leaf=leaf)
        d = vte.vte_desc_gemv(c, A, A, A, 8, 14336 * 2, 4096, vte.VTE_EPI_SILU_MUL)
        v = vte.vte_desc_info(d)
        n = vte.vte_desc_info(vte.vte_desc_rmsnorm(c, A, A, A, 8, 4096, 1e-6))
        views.append((list(v.grid), list(v.block), v.lds_bytes, v.profile_key, list(n.grid), list(n.block)))
        vte.vte_shutdown(c)
    assert views[0] == views[1] == views[2]
    c = make_ctx()
    # the reshaped baseline does change with the CU count it is given
    blocks = [list(vte.vte_desc_info(vte.vte_desc_rmsnorm_reshaped(c, A, A, A, 8, 1024, 1e-6, w)).block) for w in (32, 64, 128, 256)]
    assert blocks == [[64, 1, 1], [128, 1, 1], [256, 1, 1], [512, 1, 1]]
    grids = [list(vte.vte_desc_info(vte.vte_desc_gemv_splitk(c, A, A, A, A, 1, 4096, 4096, 0, s)).grid) for s in (1, 2, 4, 8)]
    assert [g[1] for g in grids] == [1, 2, 4, 8] and len({g[0] for g in grids}) == 1
    vte.vte_shutdown(c)


def _plan(kind, bt, rows, ks, pf, mw, groups):
    p = vte.vte_gemv_plan()
    p.batch_tile, p.rows, p.ksteps, p.prefetch, p.max_waves, p.groups, p.kind = bt, rows, ks, pf, mw, groups, kind
    return p


def test_default_plans_by_batch_and_width_of_the_output(ctx):
    """The decomposition is a function of (B, N, K, epilogue) alone: which kernel family serves which
    batch, and that every default plan builds."""
    def kind_bt(B, N, K, epi=0):
        p = vte.vte_gemv_default_plan(B, N, K, epi, 1)
        vte.vte_desc_destroy(vte.vte_desc_gemv(ctx, A, A, A, B, N, K, epi))
        return p.kind, p.batch_tile
    assert kind_bt(1, 4096, 4096)[0] == vte.VTE_GEMV_DOT2
    assert kind_bt(8, 4096, 4096) == (vte.VTE_GEMV_MFMA, 16)
    assert kind_bt(24, 4096, 4096) == (vte.VTE_GEMV_MFMA, 32)
    assert kind_bt(24, 128256, 4096) == (vte.VTE_GEMV_MFMA_ROWS, 32)       # wide output: rows split, X through LDS
    assert kind_bt(64, 4096, 14336) == (vte.VTE_GEMV_MFMA, 64)             # narrow output: K split, four column tiles
    assert kind_bt(64, 28672, 4096, vte.VTE_EPI_SILU_MUL) == (vte.VTE_GEMV_MFMA_ROWS, 64)
    assert kind_bt(33, 128256, 4096) == (vte.VTE_GEMV_MFMA_ROWS, 64)
    big = vte.vte_gemv_default_plan(8, 128256, 4096, 0, 1)                 # 1024-element chunks: four waves hold all of X
    assert (big.ksteps, big.max_waves) == (8, 4)
    long_k = vte.vte_gemv_default_plan(8, 128256, 8192, 0, 1)              # not for longer rows
    assert long_k.ksteps == 4


def test_plans_that_do_not_fit_are_rejected(ctx):
    R, M = vte.VTE_GEMV_MFMA_ROWS, vte.VTE_GEMV_MFMA
    for B, N, K, plan in (
        (64, 4096, 4096, _plan(R, 16, 32, 1, 2, 8, 1)),      # the row-split kind has batch_tile 32 or 64
        (40, 4096, 4096, _plan(R, 32, 32, 1, 2, 8, 1)),      # and takes the whole batch in one tile
        (64, 4096, 4096, _plan(R, 64, 32, 1, 3, 8, 1)),      # a combination that is not built
        (64, 8, 4096, _plan(R, 64, 32, 1, 2, 8, 1)),         # less than one tile of outputs
        (64, 4096, 4096, _plan(M, 16, 16, 4, 2, 8, 1)),      # batch_tile 16 takes at most 16 rows
        (64, 4096, 4096, _plan(vte.VTE_GEMV_DOT2, 16, 4, 2, 1, 8, 1)),
        (8, 4096, 4096, _plan(7, 16, 16, 4, 2, 8, 1)),       # unknown kind
        (8, 4096, 1 << 26, _plan(M, 16, 16, 4, 2, 8, 1)),    # a workgroup's 16 weight rows span 2 GiB: 32-bit offsets
    ):
        with pytest.raises(vte.VteError) as e:
            vte.vte_desc_gemv_planned(ctx, A, A, A, B, N, K, 0, plan)
        assert e.value.code == vte.VTE_EINVAL
    vte.vte_desc_destroy(vte.vte_desc_gemv_planned(ctx, A, A, A, 8, 4096, 1 << 24, 0, _plan(M, 16, 16, 4, 2, 8, 1)))
    with pytest.raises(vte.VteError):                        # no split-K baseline above batch 32
        vte.vte_desc_gemv_splitk(ctx, A, A, A, A, 33, 4096, 4096, 0, 2)
    with pytest.raises(vte.VteError):
        vte.vte_splitk_workspace_bytes(65, 4096, 2)
    # the shape-derived split: a factor from the shape alone, a split launch with S workgroup rows, a finish launch
    assert vte.vte_gemv_fixed_split(64, 4096, 4096) == 1 and vte.vte_gemv_fixed_split(64, 4096, 14336) == 7
    assert vte.vte_gemv_fixed_split(32, 4096, 4096) == 1 and vte.vte_gemv_fixed_split(64, 128256, 4096) == 1
    d1 = vte.vte_desc_gemv_split(ctx, A, A, 0, A, 64, 4096, 4096, 0, 4)
    d2 = vte.vte_desc_gemv_split_finish(ctx, d1, A)
    assert vte.vte_desc_info(d1).grid[1] == 4 and vte.vte_desc_info(d2).grid[1] == 64
    with pytest.raises(vte.VteError):
        vte.vte_desc_gemv_split_finish(ctx, d2, A)           # not a split descriptor
    with pytest.raises(vte.VteError):
        vte.vte_desc_gemv_split(ctx, A, A, 0, A, 64, 4096, 4096, 0, 3)   # S must divide K


def test_the_qkv_launch_with_the_step_boundary_in_its_prologue_has_a_shape_derived_geometry(ctx):
    """vte_desc_gemv_rmsnorm_gather{,_argmax}: 256 threads, 16 or 32 rows per workgroup from N alone; built for
    K = 4096 and batch <= 16; the candidates come from an LM-head descriptor of the same context."""
    d = vte.vte_desc_gemv_rmsnorm_gather(ctx, A, A, A, A, A, None, None, 8, 128256, 6144, 4096, 1e-6)
    v = vte.vte_desc_info(d)
    assert v.kernel == vte.VTE_K_GEMV_NORM and list(v.grid) == [192, 1, 1] and list(v.block) == [256, 1, 1]
    d2 = vte.vte_desc_gemv_rmsnorm_gather(ctx, A, A, A, A, A, A, A, 16, 1000, 4096, 4096, 1e-6)
    assert list(vte.vte_desc_info(d2).grid) == [256, 1, 1]
    assert vte.vte_desc_info(d2).profile_key != v.profile_key
    lm = vte.vte_desc_lmhead_argmax(ctx, A, A, A, None, A, 8, 128256, 4096)
    d3 = vte.vte_desc_gemv_rmsnorm_gather_argmax(ctx, A, A, lm, A, A, A, None, None, 128256, 6144, 4096, 1e-6)
    assert list(vte.vte_desc_info(d3).grid) == [192, 1, 1] and vte.vte_desc_info(d3).bytes > v.bytes   # the candidates are read too
    plain = vte.vte_desc_gemv(ctx, A, A, A, 8, 6144, 4096, 0)
    for call in (
        lambda: vte.vte_desc_gemv_rmsnorm_gather(ctx, A, A, A, A, A, None, None, 17, 1000, 6144, 4096, 1e-6),    # batch
        lambda: vte.vte_desc_gemv_rmsnorm_gather(ctx, A, A, A, A, A, None, None, 8, 1000, 6144, 2048, 1e-6),     # hidden size
        lambda: vte.vte_desc_gemv_rmsnorm_gather(ctx, A, A, A, A, A, None, None, 8, 1000, 8, 4096, 1e-6),        # less than a tile
        lambda: vte.vte_desc_gemv_rmsnorm_gather(ctx, A, A, A, A, A, None, None, 8, 1 << 18, 6144, 4096, 1e-6),  # table of 2 GiB
        lambda: vte.vte_desc_gemv_rmsnorm_gather(ctx, A, A, None, A, A, None, None, 8, 1000, 6144, 4096, 1e-6),  # no tokens
        lambda: vte.vte_desc_gemv_rmsnorm_gather(ctx, A, A + 2, A, A, A, None, None, 8, 1000, 6144, 4096, 1e-6), # alignment
        lambda: vte.vte_desc_gemv_rmsnorm_gather_argmax(ctx, A, A, plain, A, A, A, None, None, 1000, 6144, 4096, 1e-6),
    ):
        with pytest.raises(vte.VteError) as e:
            call()
        assert e.value.code == vte.VTE_EINVAL
    for x in (d, d2, d3, lm, plain):
        vte.vte_desc_destroy(x)


def test_bad_shapes_are_rejected(ctx):
    for call in (
        lambda: vte.vte_desc_rmsnorm(ctx, A, A, A, 8, 1020, 1e-6),          # cols % 8
        lambda: vte.vte_desc_rmsnorm(ctx, A, A, A, 0, 1024, 1e-6),
        lambda: vte.vte_desc_rmsnorm(ctx, A + 2, A, A, 8, 1024, 1e-6),      # alignment
        lambda: vte.vte_desc_gemv(ctx, A, A, A, 65, 64, 64, 0),             # B > 64
        lambda: vte.vte_desc_gemv(ctx, A, A, A, 17, 8, 64, 0),              # batch 17-32 needs a full tile of outputs
        lambda: vte.vte_desc_gemv(ctx, A, A, A, 1, 63, 64, vte.VTE_EPI_SILU_MUL),
        lambda: vte.vte_desc_gemv(ctx, A, A, A, 1, 64, 60, 0),
        lambda: vte.vte_desc_gemv_splitk(ctx, A, A, A, A, 1, 64, 4096, 0, 3),
        lambda: vte.vte_desc_lmhead_argmax(ctx, A, A, A, None, None, 1, 64, 64),
        lambda: vte.vte_desc_gemm(ctx, A, A, A, 100, 256, 64),
        lambda: vte.vte_desc_gather(ctx, A, A, A, 2, 10, 12),
    ):
        with pytest.raises(vte.VteError) as e:
            call()
        assert e.value.code == vte.VTE_EINVAL


# ---------- binding and submission (Sec. 4.4) ----------------------------------------------------
def test_failed_submission_leaves_op_ready(ctx):
    vs = vte.vte_vstream_create(ctx)
    d = norm_desc(ctx)
    vte.vte_fake_fail_next_submits(ctx, 2)
    t = vte.vte_submit(vs, d)
    for _ in range(100):                             # each dispatcher pass retries the ready op once
        vte.vte_dispatcher_quiesce(ctx)
        if vte.vte_fake_log(ctx):
            break
    log = vte.vte_fake_log(ctx)
    assert [e.token for e in log] == [t]             # third attempt went through
    st = vte.vte_stats(ctx)
    assert st.submit_failures == 2 and st.leases_opened == 1   # nothing was committed by the failures
    assert vte.vte_pool_info(ctx, log[0].pctx).outstanding == 1
    vte.vte_fake_complete(ctx, t)
    vte.vte_vstream_sync(vs)
    # explicit launch: the failure is reported and nothing is leased
    vte.vte_fake_fail_next_submits(ctx, 1)
    with pytest.raises(vte.VteError) as e:
        vte.vte_bind_and_launch(ctx, d, 0)
    assert e.value.code == vte.VTE_EHIP
    assert vte.vte_pool_info(ctx, 0).state == vte.VTE_PCTX_IDLE


def test_submission_that_always_fails_fails_the_op_and_its_dependants(ctx):
    """A failed submission leaves the op ready (Sec. 4.4), but not for ever: after a bounded number
    of attempts the op is retired as failed, its waiters get the backend's error on their own
    thread, and every op that depends on it fails with it."""
    vs, other = vte.vte_vstream_create(ctx), vte.vte_vstream_create(ctx)
    d = norm_desc(ctx)
    vte.vte_fake_fail_next_submits(ctx, 1 << 20)
    t1 = vte.vte_submit(vs, d)
    t2 = vte.vte_submit(vs, d)                         # stream order: depends on t1
    t3 = vte.vte_submit_after(other, d, [t1])          # cross-stream edge onto t1
    for t in (t1, t2, t3):
        with pytest.raises(vte.VteError) as e:
            vte.vte_token_wait(ctx, t)                 # returns instead of blocking
        assert e.value.code == vte.VTE_EHIP and "injected submission failure" in str(e.value)
    with pytest.raises(vte.VteError) as e:
        vte.vte_token_query(ctx, t2)
    assert e.value.code == vte.VTE_EHIP and "predecessor failed" in str(e.value)
    st = vte.vte_stats(ctx)
    assert st.failed == 3 and st.submit_failures == 8 and st.completed == 0 and st.leases_opened == 0
    assert vte.vte_fake_log(ctx) == []                 # nothing ever reached the backend
    assert all(i.state == vte.VTE_PCTX_IDLE and i.outstanding == 0 for i in infos(ctx))
    # the stream reports its failed tail once and is usable again; so is the device-wide wait
    with pytest.raises(vte.VteError):
        vte.vte_vstream_sync(vs)
    with pytest.raises(vte.VteError) as e:
        vte.vte_device_sync(ctx)
    assert e.value.code == vte.VTE_EHIP
    vte.vte_fake_fail_next_submits(ctx, 0)
    vte.vte_fake_set_autocomplete(ctx, 1)
    t4 = vte.vte_submit(vs, d)
    vte.vte_token_wait(ctx, t4)
    vte.vte_vstream_sync(vs)
    vte.vte_device_sync(ctx)                           # the failure was reported; nothing new failed
    assert vte.vte_stats(ctx).completed == 1


def test_completion_that_reports_a_device_error_fails_the_token(ctx):
    """A completion record that comes back with an error is not a successful launch: the token is
    retired as failed with the backend's message and HIP code, the lease is released, successors
    do not run, and the error reaches a caller that was already blocked in the wait."""
    import threading
    vs = vte.vte_vstream_create(ctx)
    d = norm_desc(ctx)
    t1 = vte.vte_submit(vs, d)
    t2 = vte.vte_submit(vs, d)
    vte.vte_dispatcher_quiesce(ctx)
    assert [e.token for e in vte.vte_fake_log(ctx)] == [t1]     # STRICT: t2 waits for t1
    got = {}

    def waiter():
        try:
            vte.vte_token_wait(ctx, t1)
            got["rc"] = 0
        except vte.VteError as e:
            got["rc"], got["msg"], got["hip"] = e.code, str(e), vte.vte_last_hip_error()

    th = threading.Thread(target=waiter)
    th.start()
    vte.vte_fake_complete_error(ctx, t1)
    th.join(10)
    assert not th.is_alive()
    assert got["rc"] == vte.VTE_EHIP and "injected device error" in got["msg"] and got["hip"] == 719
    with pytest.raises(vte.VteError) as e:
        vte.vte_token_wait(ctx, t2)                    # never submitted: its predecessor failed
    assert e.value.code == vte.VTE_EHIP
    assert [e.token for e in vte.vte_fake_log(ctx)] == [t1]
    st = vte.vte_stats(ctx)
    assert st.failed == 2 and st.completed == 1
    assert all(i.state == vte.VTE_PCTX_IDLE and i.outstanding == 0 for i in infos(ctx))
    with pytest.raises(vte.VteError) as e:
        vte.vte_device_sync(ctx)
    assert e.value.code == vte.VTE_EHIP
    vte.vte_device_sync(ctx)                           # reported once


def test_policy_callbacks_and_stale_proposal(ctx):
    calls = {"pick": 0, "select": 0, "bad": True}
    root = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 256)
    leaf = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 32, 5)

    def pick(user, ready, n, S):
        calls["pick"] += 1
        assert n >= 1 and S.contents.count == 27
        return 0

    def select(user, op, el, n, S):
        calls["select"] += 1
        ids = [el[i] for i in range(n)]
        if calls["bad"]:
            calls["bad"] = False
            blocked = next(i for i in range(27) if i not in ids)   # a pCtx outside E
            return blocked
        assert root not in ids                                     # overlaps the explicit lease below
        return leaf if leaf in ids else -1

    vt = vte.vte_policy_vtbl(vte.PICK_FN(pick), vte.SELECT_FN(select), vte.PREPARE_FN())
    vte.vte_set_policy(ctx, vt, None)
    d = norm_desc(ctx)
    other = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 32, 0)
    t0 = vte.vte_bind_and_launch(ctx, d, other)
    vs = vte.vte_vstream_create(ctx)
    t = vte.vte_submit(vs, d)
    for _ in range(100):
        vte.vte_dispatcher_quiesce(ctx)
        if len(vte.vte_fake_log(ctx)) == 2:
            break
    log = vte.vte_fake_log(ctx)
    assert log[-1].token == t and log[-1].pctx == leaf
    assert vte.vte_stats(ctx).stale_proposals == 1 and calls["select"] >= 2
    for tok in (t0, t):
        vte.vte_fake_complete(ctx, tok)
    vte.vte_device_sync(ctx)
    vte.vte_set_policy(ctx, None)


def test_default_policy_takes_widest_non_conflicting(ctx):
    d = norm_desc(ctx)
    ps = infos(ctx)
    a, b = vte.vte_vstream_create(ctx), vte.vte_vstream_create(ctx, vte.VTE_CLASS_BEST_EFFORT)
    ta = vte.vte_submit(a, d)
    vte.vte_dispatcher_quiesce(ctx)
    log = vte.vte_fake_log(ctx)
    assert ps[log[0].pctx].width == 256
    tb = vte.vte_submit(b, d)
    vte.vte_dispatcher_quiesce(ctx)
    assert len(vte.vte_fake_log(ctx)) == 1           # everything overlaps the root: stays ready
    vte.vte_fake_complete(ctx, ta)
    vte.vte_token_wait(ctx, ta)
    vte.vte_dispatcher_quiesce(ctx)
    assert vte.vte_fake_log(ctx)[-1].token == tb
    vte.vte_fake_complete(ctx, tb)
    vte.vte_device_sync(ctx)


def test_queue_state_policy_uses_profiles(ctx):
    d = norm_desc(ctx)
    g = vte.vte_desc_gemm(ctx, A, A, A, 512, 512, 512)
    key = vte.vte_desc_info(d).profile_key
    for w, t in ((32, 10e-6), (64, 6e-6), (128, 5.2e-6), (192, 5.1e-6), (224, 5.05e-6), (256, 5e-6)):
        vte.vte_profile_set(ctx, key, w, t)
    assert vte.vte_profile_get(ctx, key, 128) == pytest.approx(5.2e-6)
    with pytest.raises(vte.VteError):
        vte.vte_profile_get(ctx, key, 48)
    vte.vte_set_builtin_policy(ctx, vte.VTE_POLICY_QUEUE_STATE, 0.1, 0)
    lat, be = vte.vte_vstream_create(ctx, vte.VTE_CLASS_LATENCY), vte.vte_vstream_create(ctx, vte.VTE_CLASS_BEST_EFFORT)
    ps = infos(ctx)
    t0 = vte.vte_submit(lat, d)                      # alone on the device: the fastest width
    vte.vte_dispatcher_quiesce(ctx)
    assert ps[vte.vte_fake_log(ctx)[-1].pctx].width == 256
    vte.vte_fake_complete(ctx, t0)
    vte.vte_device_sync(ctx)
    g1 = vte.vte_submit(be, g)                       # nothing latency-critical around: whole device
    g2 = vte.vte_submit(be, g)                       # (waits for g1 in stream order)
    vte.vte_dispatcher_quiesce(ctx)
    assert ps[vte.vte_fake_log(ctx)[-1].pctx].width == 256
    t1 = vte.vte_submit(lat, d)                      # everything overlaps the root lease: stays ready
    vte.vte_dispatcher_quiesce(ctx)
    assert vte.vte_fake_log(ctx)[-1].token == g1
    vte.vte_fake_complete(ctx, g1)
    vte.vte_token_wait(ctx, g1)
    vte.vte_dispatcher_quiesce(ctx)
    log = {e.token: e.pctx for e in vte.vte_fake_log(ctx)}
    p1, p2 = log[t1], log[g2]
    assert ps[p1].width == 128                       # sharing: narrowest width within 10% of the best
    assert ps[p2].width == 128 and p2 == ps[p1].remainder   # best effort takes the widest that is left
    vte.vte_fake_complete(ctx, t1)
    vte.vte_fake_complete(ctx, g2)
    vte.vte_device_sync(ctx)


def test_queue_state_policy_keeps_a_chain_on_one_width(pctx):
    """The width decision is taken for the recurring chain, not per launch: a tiny
    launch does not drag the heavy ones onto a narrow pCtx, and a launch whose good
    pCtx is blocked only by its own vstream's lease waits for that lease to drain."""
    c = pctx
    small = norm_desc(c)
    big = vte.vte_desc_gemm(c, A, A, A, 512, 512, 512)
    ks, kb = vte.vte_desc_info(small).profile_key, vte.vte_desc_info(big).profile_key
    for w in (32, 64, 128, 192, 224, 256):
        vte.vte_profile_set(c, ks, w, 4e-6)                      # flat: launch-bound
        vte.vte_profile_set(c, kb, w, 100e-6 * 256 / w)          # scales with width
    vte.vte_set_builtin_policy(c, vte.VTE_POLICY_QUEUE_STATE, 0.1, 0)
    lat = vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY)
    ps = infos(c)
    toks = []
    for _ in range(3):
        toks += [vte.vte_submit(lat, small), vte.vte_submit(lat, big)]
    vte.vte_dispatcher_quiesce(c)
    log = vte.vte_fake_log(c)
    assert [e.token for e in log] == toks and {ps[e.pctx].width for e in log[1:]} == {256}
    first = log[0].pctx                                          # bound before the chain was known
    for t in toks:
        vte.vte_fake_complete(c, t)
    vte.vte_vstream_sync(lat)
    assert ps[first].width in (32, 256)


# ---------- pipelined binding -----------------------------------------------------------------------
def test_pipelined_binds_ahead_with_device_side_edges(pctx):
    c = pctx
    d = norm_desc(c)
    vs = vte.vte_vstream_create(c)
    toks = [vte.vte_submit(vs, d) for _ in range(5)]
    vte.vte_dispatcher_quiesce(c)
    log = vte.vte_fake_log(c)
    assert [e.token for e in log] == toks            # all bound before anything completed
    assert len({e.pctx for e in log}) == 1           # same pCtx: stream order carries the edge
    assert all(e.waited_on_pctx == -1 for e in log)
    for t in toks:
        vte.vte_fake_complete(c, t)
    vte.vte_vstream_sync(vs)
    # successive ops on different pCtxs: the edge becomes a device-side wait on the predecessor
    n0 = vte.vte_pool_find(c, vte.VTE_PCTX_NODE, 128, 0)
    n1 = vte.vte_pool_find(c, vte.VTE_PCTX_NODE, 128, 1)
    vte.vte_vstream_pin(vs, n0)
    t0 = vte.vte_submit(vs, d)
    vte.vte_dispatcher_quiesce(c)
    vte.vte_vstream_pin(vs, n1)
    t1 = vte.vte_submit(vs, d)
    vte.vte_dispatcher_quiesce(c)
    log = vte.vte_fake_log(c)[-2:]
    assert (log[0].token, log[0].pctx, log[1].token, log[1].pctx, log[1].waited_on_pctx) == (t0, n0, t1, n1, n0)
    vte.vte_fake_complete(c, t0)
    vte.vte_fake_complete(c, t1)
    vte.vte_vstream_sync(vs)


def test_pipelined_lookahead_is_bounded():
    c = make_ctx(vte.VTE_MODE_PIPELINED, lookahead=3)
    try:
        d = norm_desc(c)
        vs = vte.vte_vstream_create(c)
        toks = [vte.vte_submit(vs, d) for _ in range(6)]
        vte.vte_dispatcher_quiesce(c)
        assert len(vte.vte_fake_log(c)) == 3
        vte.vte_fake_complete(c, toks[0])
        vte.vte_token_wait(c, toks[0])
        vte.vte_dispatcher_quiesce(c)
        assert len(vte.vte_fake_log(c)) == 4
        for t in toks[1:]:
            vte.vte_dispatcher_quiesce(c)
            vte.vte_fake_complete(c, t)
            vte.vte_token_wait(c, t)
        recs = vte.vte_stats_read(c)
        assert [r.token for r in recs] == toks
        assert all(r.t_submit <= r.t_ready <= r.t_bound <= r.t_done for r in recs)
    finally:
        vte.vte_shutdown(c)


def test_out_of_order_completion_across_pctxs(ctx):
    d = norm_desc(ctx)
    a = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 64, 0)
    b = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 64, 3)
    ta, tb = vte.vte_bind_and_launch(ctx, d, a), vte.vte_bind_and_launch(ctx, d, b)
    vte.vte_fake_complete(ctx, tb)
    vte.vte_token_wait(ctx, tb)
    assert not vte.vte_token_query(ctx, ta)
    assert vte.vte_pool_info(ctx, b).state == vte.VTE_PCTX_IDLE and vte.vte_pool_info(ctx, a).state == vte.VTE_PCTX_LEASED
    vte.vte_fake_complete(ctx, ta)
    vte.vte_device_sync(ctx)
    with pytest.raises(vte.VteError):
        vte.vte_fake_complete(ctx, ta)               # not in flight any more


# ---------- events and data-movement descriptors (Sec. 4.2) ----------------------------------------
def test_event_is_an_immutable_completion_point_and_wait_orders_a_stream(ctx):
    a, b = vte.vte_vstream_create(ctx), vte.vte_vstream_create(ctx)
    d = norm_desc(ctx)
    assert vte.vte_event_record(a) == 0                      # empty stream: already satisfied
    vte.vte_vstream_wait_event(b, 0)                         # waiting on it adds nothing
    n0 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 0)
    n1 = vte.vte_pool_find(ctx, vte.VTE_PCTX_NODE, 128, 1)
    vte.vte_vstream_pin(a, n0)
    vte.vte_vstream_pin(b, n1)
    ta1 = vte.vte_submit(a, d)
    ev = vte.vte_event_record(a)                             # generation: the tail as of now
    assert ev == ta1
    ta2 = vte.vte_submit(a, d)                               # later work on `a` does not move the event
    assert vte.vte_event_record(a) == ta2
    vte.vte_vstream_wait_event(b, ev)
    tb1 = vte.vte_submit(b, d)                               # carries the wait ...
    tb2 = vte.vte_submit(b, d)                               # ... and tb2 follows tb1 in stream order
    vte.vte_dispatcher_quiesce(ctx)
    assert [e.token for e in vte.vte_fake_log(ctx)] == [ta1]
    vte.vte_fake_complete(ctx, ta1)
    vte.vte_token_wait(ctx, ta1)
    vte.vte_dispatcher_quiesce(ctx)
    assert sorted(e.token for e in vte.vte_fake_log(ctx)) == sorted([ta1, ta2, tb1])   # tb1 did not wait for ta2
    for t in (ta2, tb1):
        vte.vte_fake_complete(ctx, t)
    vte.vte_token_wait(ctx, tb1)
    vte.vte_dispatcher_quiesce(ctx)
    assert vte.vte_fake_log(ctx)[-1].token == tb2
    vte.vte_fake_complete(ctx, tb2)
    vte.vte_device_sync(ctx)
    with pytest.raises(vte.VteError):
        vte.vte_vstream_wait_event(b, 10 ** 9)               # never issued
    vte.vte_vstream_wait_event(b, ta1)                       # satisfied long ago: nothing to wait for
    t = vte.vte_submit(b, d)
    vte.vte_dispatcher_quiesce(ctx)
    assert vte.vte_fake_log(ctx)[-1].token == t
    vte.vte_fake_complete(ctx, t)
    vte.vte_device_sync(ctx)


def test_memcpy_and_memset_descriptors(ctx):
    d = vte.vte_desc_memcpy(ctx, A + 0x100000, A, 1 << 20)
    v = vte.vte_desc_info(d)
    assert v.kernel == vte.VTE_K_MEMCPY and list(v.grid) == [64, 1, 1] and list(v.block) == [256, 1, 1] and v.bytes == 2 << 20
    m = vte.vte_desc_memset32(ctx, A, 0xDEADBEEF, 48)
    v = vte.vte_desc_info(m)
    assert v.kernel == vte.VTE_K_MEMSET and list(v.grid) == [1, 1, 1] and v.bytes == 48
    args = vte.vte_desc_args(m)
    assert int.from_bytes(args[0:8], "little") == A and int.from_bytes(args[8:16], "little") == 48
    assert int.from_bytes(args[16:20], "little") == 0xDEADBEEF
    for call in (lambda: vte.vte_desc_memcpy(ctx, A, A + 0x1000, 0), lambda: vte.vte_desc_memcpy(ctx, A, A + 0x1000, 24),
                 lambda: vte.vte_desc_memcpy(ctx, A + 4, A + 0x1000, 32), lambda: vte.vte_desc_memset32(ctx, A + 8, 0, 32),
                 lambda: vte.vte_desc_memset32(ctx, None, 0, 32)):
        with pytest.raises(vte.VteError) as e:
            call()
        assert e.value.code == vte.VTE_EINVAL
