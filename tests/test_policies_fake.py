"""The two policy instantiations of Sec. 5 (Throughput-Oriented, Algorithm 1; TPOT-First)
driven through the C ABI on the fake backend (no GPU).

A joint plan needs several ready ops in one dispatch round: the tests park the
dispatcher behind a custom Pick that defers, submit, then switch to the built-in policy.
"""
import time

import pytest

from paper_2603_15042_amd import vte
from test_runtime_fake import A, make_ctx, infos

WIDTHS = (32, 64, 128, 192, 224, 256)


def park(c):
    keep = {"pick": vte.PICK_FN(lambda user, ready, n, S: -1)}
    vt = vte.vte_policy_vtbl()
    vt.pick = keep["pick"]
    vte.vte_set_policy(c, vt)
    return keep, vt


def set_profile(c, desc, times):
    """times: width -> seconds, or a callable of the width."""
    key = vte.vte_desc_info(desc).profile_key
    for w in WIDTHS:
        vte.vte_profile_set(c, key, w, times(w) if callable(times) else times[w])


def bound(c):
    return {e.token: e.pctx for e in vte.vte_fake_log(c)}


def assert_disjoint(c, ids):
    for i, a in enumerate(ids):
        for b in ids[i + 1:]:
            assert not vte.vte_pool_conflict(c, a, b)


def finish(c, toks):
    for t in toks:
        vte.vte_fake_complete(c, t)
    vte.vte_device_sync(c)


# ---------- Throughput-Oriented (Algorithm 1) ---------------------------------------------------
def test_tput_plan_flat_ops_stay_narrow_and_scaling_ops_widen():
    c = make_ctx()
    try:
        flat = vte.vte_desc_rmsnorm(c, A, A, A, 8, 1024, 1e-6)
        lin1 = vte.vte_desc_gemv(c, A, A, A, 1, 4096, 4096, 0)
        lin2 = vte.vte_desc_gemv(c, A, A, A, 1, 6144, 4096, 0)
        set_profile(c, flat, lambda w: 4e-6)                 # gains nothing from more CUs
        set_profile(c, lin1, lambda w: 1e-3 * 32 / w)        # scales perfectly
        set_profile(c, lin2, lambda w: 2e-3 * 32 / w)
        keep = park(c)
        vs = [vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT) for _ in range(3)]
        toks = [vte.vte_submit(v, d) for v, d in zip(vs, (flat, lin1, lin2))]
        vte.vte_dispatcher_quiesce(c)
        assert vte.vte_fake_log(c) == []
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        vte.vte_dispatcher_quiesce(c)
        b = bound(c)
        assert sorted(b) == sorted(toks)                     # concurrency first: all three run
        ps = infos(c)
        assert ps[b[toks[0]]].width == 32
        assert sorted(ps[b[t]].width for t in toks) == [32, 64, 128]   # nothing usable is left over
        assert_disjoint(c, [b[t] for t in toks])
        finish(c, toks)
        del keep
    finally:
        vte.vte_shutdown(c)


def test_tput_plan_weighs_a_stream_by_its_recurring_chain_not_by_the_launch_at_hand():
    """Sec. 5 "Performance Profiles": a stream that alternates a flat launch (a norm) with one that scales
    (a projection) is planned by the profile of the chain.  Planned by the launch that happens to be ready,
    the flat one would keep the stream on a leaf while a co-tenant takes the rest of the device."""
    c = make_ctx(remainders=vte.VTE_REMAINDERS_NONE)
    try:
        flat = vte.vte_desc_rmsnorm(c, A, A, A, 8, 1024, 1e-6)
        lin = vte.vte_desc_gemv(c, A, A, A, 1, 4096, 4096, 0)
        ten = vte.vte_desc_gemv(c, A, A, A, 1, 6144, 4096, 0)
        set_profile(c, flat, lambda w: 4e-6)                      # gains nothing from more CUs
        set_profile(c, lin, lambda w: 1e-3 * 32 / w)              # scales perfectly
        set_profile(c, ten, lambda w: 1e-3 * (32 / w) ** 0.3)     # the co-tenant: sublinear
        chain, other = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT), vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        first = vte.vte_submit(chain, lin)                        # the chain's history: the scaling launch has run
        vte.vte_dispatcher_quiesce(c)
        finish(c, [first])
        keep = park(c)
        t_flat, t_ten = vte.vte_submit(chain, flat), vte.vte_submit(other, ten)
        vte.vte_dispatcher_quiesce(c)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        vte.vte_dispatcher_quiesce(c)
        b, ps = bound(c), infos(c)
        assert ps[b[t_flat]].width == 128 and ps[b[t_ten]].width == 128, (ps[b[t_flat]].width, ps[b[t_ten]].width)
        assert_disjoint(c, [b[t_flat], b[t_ten]])
        finish(c, [t_flat, t_ten])
        # a stream whose whole history is flat stays narrow (the first test of this file), chain or not
        del keep
    finally:
        vte.vte_shutdown(c)


def test_tput_plan_prefers_the_steeper_profile():
    c = make_ctx(remainders=vte.VTE_REMAINDERS_NONE)
    try:
        steep = vte.vte_desc_gemv(c, A, A, A, 1, 4096, 4096, 0)
        shallow = vte.vte_desc_gemv(c, A, A, A, 1, 6144, 4096, 0)
        set_profile(c, steep, lambda w: 1e-3 * 32 / w)
        set_profile(c, shallow, lambda w: 1e-3 * (32 / w) ** 0.3)   # sublinear: P(m) = (m/32)^0.3
        keep = park(c)
        vs = [vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT) for _ in range(2)]
        t_sh = vte.vte_submit(vs[0], shallow)                # the older op does not get the larger share for its age
        t_st = vte.vte_submit(vs[1], steep)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        vte.vte_dispatcher_quiesce(c)
        b, ps = bound(c), infos(c)
        assert ps[b[t_st]].width == 128 and ps[b[t_sh]].width == 128   # both halves: every expansion had positive gain
        finish(c, [t_sh, t_st])
        # three ops on four 64-CU quarters: the steep one gets the half, the others a quarter each
        keep2 = park(c)
        third = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        toks = [vte.vte_submit(vs[0], shallow), vte.vte_submit(third, shallow), vte.vte_submit(vs[1], steep)]
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        vte.vte_dispatcher_quiesce(c)
        b = bound(c)
        assert [ps[b[t]].width for t in toks] == [64, 64, 128]
        assert_disjoint(c, [b[t] for t in toks])
        finish(c, toks)
        del keep, keep2
    finally:
        vte.vte_shutdown(c)


def test_tput_plan_without_profiles_assumes_perfect_scaling_and_takes_the_device(ctx=None):
    c = make_ctx()
    try:
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        d = vte.vte_desc_rmsnorm(c, A, A, A, 8, 1024, 1e-6)
        vs = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        t = vte.vte_submit(vs, d)
        vte.vte_dispatcher_quiesce(c)
        assert infos(c)[bound(c)[t]].width == 256
        finish(c, [t])
    finally:
        vte.vte_shutdown(c)


def test_tput_plan_more_ready_ops_than_leaves_binds_the_oldest():
    c = make_ctx(total=64, leaf=32, remainders=vte.VTE_REMAINDERS_NONE)   # two leaves
    try:
        d = vte.vte_desc_rmsnorm(c, A, A, A, 8, 1024, 1e-6)
        keep = park(c)
        vs = [vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT) for _ in range(3)]
        toks = [vte.vte_submit(v, d) for v in vs]
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        vte.vte_dispatcher_quiesce(c)
        b = bound(c)
        assert sorted(b) == toks[:2]                         # age order decides who waits
        assert_disjoint(c, list(b.values()))
        vte.vte_fake_complete(c, toks[0])
        vte.vte_token_wait(c, toks[0])
        vte.vte_dispatcher_quiesce(c)
        assert toks[2] in bound(c)                           # the freed leaf goes to the op that waited
        finish(c, toks[1:])
        del keep
    finally:
        vte.vte_shutdown(c)


def test_tput_plan_waits_for_its_own_lease_rather_than_settling_for_less():
    c = make_ctx(vte.VTE_MODE_PIPELINED)
    try:
        d = vte.vte_desc_gemv(c, A, A, A, 1, 4096, 4096, 0)
        set_profile(c, d, lambda w: 1e-3 * 32 / w)
        half0 = vte.vte_pool_find(c, vte.VTE_PCTX_NODE, 128, 0)
        half1 = vte.vte_pool_find(c, vte.VTE_PCTX_NODE, 128, 1)
        other = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        vte.vte_vstream_pin(other, half0)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        t_other = vte.vte_submit(other, d)
        vte.vte_dispatcher_quiesce(c)
        vs = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        t1 = vte.vte_submit(vs, d)
        vte.vte_dispatcher_quiesce(c)
        assert bound(c)[t1] == half1                         # the widest thing that does not overlap the pinned job
        finish_one = lambda t: (vte.vte_fake_complete(c, t), vte.vte_token_wait(c, t))
        finish_one(t_other)                                  # the device is now free but for vs's own lease
        t2 = vte.vte_submit(vs, d)
        vte.vte_dispatcher_quiesce(c)
        assert t2 not in bound(c)                            # planned onto the root: stays ready while t1 runs
        finish_one(t1)
        vte.vte_dispatcher_quiesce(c)
        assert infos(c)[bound(c)[t2]].width == 256
        finish(c, [t2])
    finally:
        vte.vte_shutdown(c)


# ---------- TPOT-First -------------------------------------------------------------------------------
def decode_descs(c):
    norm = vte.vte_desc_rmsnorm(c, A, A, A, 8, 4096, 1e-6)
    head = vte.vte_desc_gemv(c, A, A, A, 8, 4096, 4096, 0)
    return norm, head


def test_tpot_first_sizes_an_exclusive_standing_pctx_from_profiles():
    c = make_ctx()
    try:
        norm, head = decode_descs(c)
        set_profile(c, norm, lambda w: 0.1)                  # seconds: the fake backend never finishes by itself,
        set_profile(c, head, lambda w: 1.9 * 32 / w)         # so nothing here is at risk; token: 2.0 / 1.05 / 0.575 s
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPOT_FIRST, 0.1)
        dec = vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY)
        vte.vte_vstream_set_tpot(dec, 1.2, 2)                # 64 CUs: 1.05 s * 1.1 <= 1.2 s; 32 CUs: too slow
        assert vte.vte_vstream_tpot_info(dec).standing_pctx == -1   # nothing to size it from yet
        keep = park(c)
        toks = [vte.vte_submit(dec, norm), vte.vte_submit(dec, head)]
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPOT_FIRST, 0.1)
        vte.vte_dispatcher_quiesce(c)
        info = vte.vte_vstream_tpot_info(dec)
        st = info.standing_pctx
        ps = infos(c)
        assert st >= 0 and ps[st].width == 64 and ps[st].kind == vte.VTE_PCTX_NODE
        assert ps[st].reserved_for == vte.vte_vstream_id(dec)
        assert bound(c)[toks[0]] == st                       # the decode runs on its reservation
        # best-effort work plans around it: never on anything that overlaps the standing pCtx
        be = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        gemm = vte.vte_desc_gemm(c, A, A, A, 256, 256, 64)
        t_be = vte.vte_submit(be, gemm)
        vte.vte_dispatcher_quiesce(c)
        p_be = bound(c)[t_be]
        assert not vte.vte_pool_conflict(c, p_be, st)
        assert ps[p_be].width == 192                         # everything but the standing quarter
        vte.vte_fake_complete(c, toks[0])
        vte.vte_token_wait(c, toks[0])
        vte.vte_dispatcher_quiesce(c)
        assert bound(c)[toks[1]] == st
        finish(c, [toks[1], t_be])
        info = vte.vte_vstream_tpot_info(dec)
        assert info.tokens_done == 1 and info.escalations == 0
        assert infos(c)[st].state == vte.VTE_PCTX_RESERVED   # standing: kept between tokens
        # removing the target releases it
        vte.vte_vstream_set_tpot(dec, 0.0, 0)
        assert infos(c)[st].state == vte.VTE_PCTX_IDLE and infos(c)[st].reserved_for == -1
    finally:
        vte.vte_shutdown(c)


def test_tpot_first_second_standing_pctx_packs_beside_the_first_and_displaces_the_best_effort_lease():
    """Two decode streams and a best-effort GEMM: the second standing leaf is the sibling of the first
    (another pipe) although the GEMM's lease overlaps it and sits on that pipe — the reservation drains
    that lease anyway — and the GEMM's next launch takes the 192-CU remainder beside the quarter."""
    c = make_ctx()
    try:
        norm, head = decode_descs(c)
        set_profile(c, norm, lambda w: 0.1)
        set_profile(c, head, lambda w: 0.5 * 32 / w)         # a token takes 0.6 s on 32 CUs: the leaf suffices
        gemm = vte.vte_desc_gemm(c, A, A, A, 256, 256, 64)
        set_profile(c, gemm, lambda w: 10.0 * 32 / w)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPOT_FIRST, 0.1)
        d1 = vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY)
        d2 = vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY)
        be = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        for d in (d1, d2):
            vte.vte_vstream_set_tpot(d, 1.0, 2)
        t1 = [vte.vte_submit(d1, norm), vte.vte_submit(d1, head)]
        vte.vte_dispatcher_quiesce(c)
        st1 = vte.vte_vstream_tpot_info(d1).standing_pctx
        ps = infos(c)
        assert st1 >= 0 and ps[st1].width == 32
        g1 = vte.vte_submit(be, gemm)                        # plans around the first leaf: its 224-CU complement
        vte.vte_dispatcher_quiesce(c)
        p_g1 = bound(c)[g1]
        assert ps[p_g1].width == 224 and not vte.vte_pool_conflict(c, p_g1, st1)
        t2 = [vte.vte_submit(d2, norm), vte.vte_submit(d2, head)]
        vte.vte_dispatcher_quiesce(c)
        st2 = vte.vte_vstream_tpot_info(d2).standing_pctx
        assert st2 >= 0 and ps[st2].width == 32 and st2 != st1
        assert ps[st2].parent == ps[st1].parent              # the sibling: one quarter holds both
        assert ps[st2].pipe != ps[st1].pipe
        assert infos(c)[p_g1].gate_open == 0                 # the GEMM's lease drains
        vte.vte_fake_complete(c, g1)
        vte.vte_token_wait(c, g1)
        g2 = vte.vte_submit(be, gemm)
        vte.vte_dispatcher_quiesce(c)
        p_g2 = bound(c)[g2]
        assert ps[p_g2].width == 192
        assert len({ps[st1].pipe, ps[st2].pipe, ps[p_g2].pipe}) == 3
        for t in t1[:1] + t2[:1]:
            vte.vte_fake_complete(c, t)
            vte.vte_token_wait(c, t)
        vte.vte_dispatcher_quiesce(c)                        # the second op of each token is bound now
        assert bound(c)[t1[1]] == st1 and bound(c)[t2[1]] == st2
        finish(c, t1[1:] + t2[1:] + [g2])
    finally:
        vte.vte_shutdown(c)


def test_tpot_first_prepares_a_wider_pctx_when_the_token_is_at_risk():
    c = make_ctx()
    try:
        norm, head = decode_descs(c)
        set_profile(c, norm, lambda w: 0.05)
        set_profile(c, head, lambda w: 0.6 * 32 / w)         # token: 0.65 s at 32, 0.35 at 64, 0.2 at 128, 0.125 at 256
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPOT_FIRST, 0.0)
        dec = vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY)
        be = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        vte.vte_vstream_set_tpot(dec, 0.4, 2)                # standing: 64 CUs
        gemm = vte.vte_desc_gemm(c, A, A, A, 256, 256, 64)
        keep = park(c)
        t_n, t_h = vte.vte_submit(dec, norm), vte.vte_submit(dec, head)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPOT_FIRST, 0.0)
        vte.vte_dispatcher_quiesce(c)
        st = vte.vte_vstream_tpot_info(dec).standing_pctx
        ps = infos(c)
        assert ps[st].width == 64 and bound(c)[t_n] == st
        t_be = vte.vte_submit(be, gemm)
        vte.vte_dispatcher_quiesce(c)
        p_be = bound(c)[t_be]
        assert ps[p_be].width == 192
        assert not vte.vte_vstream_tpot_info(dec).at_risk    # 0.05 + 0.3 s of work against a 0.4 s deadline
        time.sleep(0.15)                                     # the norm "runs" late: 0.15 + 0.05 + 0.3 > 0.4
        vte.vte_dispatcher_quiesce(c)
        info = vte.vte_vstream_tpot_info(dec)
        assert info.at_risk and info.escalations == 1
        esc = info.escalated_pctx
        # smallest wider pCtx predicted to meet the deadline: 0.15 + 0.05 + 0.6*32/w <= 0.4 needs w >= 128
        assert ps[esc].width == 128 and vte.vte_pool_conflict(c, esc, st)
        assert infos(c)[esc].reserved_for == vte.vte_vstream_id(dec)
        assert infos(c)[p_be].state == vte.VTE_PCTX_DRAINING   # the overlapping best-effort lease is being drained
        t_be2 = vte.vte_submit(be, gemm)
        vte.vte_dispatcher_quiesce(c)
        assert t_be2 not in bound(c)                         # gate closed: nothing new behind it
        vte.vte_fake_complete(c, t_be)
        vte.vte_token_wait(c, t_be)
        vte.vte_dispatcher_quiesce(c)
        assert infos(c)[esc].state == vte.VTE_PCTX_IDLE      # pending: the decode's own lease on `st` is still active below it
        assert not vte.vte_pool_conflict(c, bound(c)[t_be2], esc)   # best-effort work went on beside the prepared pCtx
        vte.vte_fake_complete(c, t_n)
        vte.vte_token_wait(c, t_n)
        vte.vte_dispatcher_quiesce(c)
        assert bound(c)[t_h] == esc                          # Select binds the at-risk decode to the prepared pCtx
        finish(c, [t_h, t_be2])
        vte.vte_dispatcher_quiesce(c)
        info = vte.vte_vstream_tpot_info(dec)
        assert info.tokens_done == 1 and info.escalated_pctx == -1   # given back once the stream is idle
        assert infos(c)[esc].reserved_for == -1 and infos(c)[st].state == vte.VTE_PCTX_RESERVED
    finally:
        vte.vte_shutdown(c)


def test_tpot_first_uses_the_standing_pctx_while_preparation_is_incomplete():
    c = make_ctx()
    try:
        norm, head = decode_descs(c)
        set_profile(c, norm, lambda w: 0.05)
        set_profile(c, head, lambda w: 0.6 * 32 / w)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPOT_FIRST, 0.0)
        dec = vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY)
        be = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        vte.vte_vstream_set_tpot(dec, 0.4, 2)
        gemm = vte.vte_desc_gemm(c, A, A, A, 256, 256, 64)
        keep = park(c)
        t_n, t_h = vte.vte_submit(dec, norm), vte.vte_submit(dec, head)
        t_be = vte.vte_submit(be, gemm)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPOT_FIRST, 0.0)
        vte.vte_dispatcher_quiesce(c)
        st = vte.vte_vstream_tpot_info(dec).standing_pctx
        time.sleep(0.2)
        vte.vte_dispatcher_quiesce(c)
        esc = vte.vte_vstream_tpot_info(dec).escalated_pctx
        assert esc >= 0
        vte.vte_fake_complete(c, t_n)                        # the decode is ready, the best-effort job still drains
        vte.vte_token_wait(c, t_n)
        vte.vte_dispatcher_quiesce(c)
        assert bound(c)[t_h] == st                           # an available allocation instead of waiting
        finish(c, [t_h, t_be])
        assert vte.vte_vstream_tpot_info(dec).deadline_misses in (0, 1)
    finally:
        vte.vte_shutdown(c)


def test_set_tpot_rejects_bad_arguments_and_busy_streams():
    c = make_ctx()
    try:
        vs = vte.vte_vstream_create(c)
        with pytest.raises(vte.VteError):
            vte.vte_vstream_set_tpot(vs, -1.0, 2)
        with pytest.raises(vte.VteError):
            vte.vte_vstream_set_tpot(vs, 1e-3, 0)
        t = vte.vte_submit(vs, vte.vte_desc_rmsnorm(c, A, A, A, 8, 1024, 1e-6))
        with pytest.raises(vte.VteError) as e:
            vte.vte_vstream_set_tpot(vs, 1e-3, 2)
        assert e.value.code == vte.VTE_EBUSY
        vte.vte_dispatcher_quiesce(c)
        finish(c, [t])
        with pytest.raises(vte.VteError):
            vte.vte_set_builtin_policy(c, 4)
    finally:
        vte.vte_shutdown(c)


def test_submit_batch_is_a_chain_seen_at_once():
    c = make_ctx(vte.VTE_MODE_PIPELINED)
    try:
        d1 = vte.vte_desc_rmsnorm(c, A, A, A, 8, 1024, 1e-6)
        d2 = vte.vte_desc_gemv(c, A, A, A, 8, 4096, 4096, 0)
        vs = vte.vte_vstream_create(c)
        arr = vte.desc_array([d1, d2, d1, d2])
        last = vte.vte_submit_batch(vs, arr)
        vte.vte_dispatcher_quiesce(c)
        log = vte.vte_fake_log(c)
        assert [e.token for e in log] == [last - 3, last - 2, last - 1, last]   # stream order, consecutive tokens
        h1, h2 = vte.vte_desc_info(d1).hash, vte.vte_desc_info(d2).hash
        assert [e.desc_hash for e in log] == [h1, h2, h1, h2]
        assert len({e.pctx for e in log}) == 1
        finish(c, [e.token for e in log])
        other = make_ctx()
        try:
            foreign = vte.vte_desc_rmsnorm(other, A, A, A, 8, 1024, 1e-6)
            with pytest.raises(vte.VteError) as e:
                vte.vte_submit_batch(vs, vte.desc_array([d1, foreign]))
            assert e.value.code == vte.VTE_EINVAL
            vte.vte_dispatcher_quiesce(c)
            assert len(vte.vte_fake_log(c)) == 4               # validated as a whole: nothing was submitted
        finally:
            vte.vte_shutdown(other)
    finally:
        vte.vte_shutdown(c)


# ---------- dispatch pipes ---------------------------------------------------------------------------
@pytest.mark.parametrize("remainders", [vte.VTE_REMAINDERS_NONE, vte.VTE_REMAINDERS_PER_LEVEL, vte.VTE_REMAINDERS_ALL])
def test_disjoint_pctxs_meant_to_run_together_sit_on_different_pipes(remainders):
    c = make_ctx(remainders=remainders)
    try:
        ps = infos(c)
        assert all(0 <= p.pipe < 4 for p in ps)
        nodes = lambda w: [p for p in ps if p.kind == vte.VTE_PCTX_NODE and p.width == w]
        assert len({p.pipe for p in nodes(128)}) == 2                  # the two halves
        assert len({p.pipe for p in nodes(64)}) == 4                   # the four quarters
        for q in nodes(64):                                            # a quarter and the opposite half
            other = [h for h in nodes(128) if not vte.vte_pool_conflict(c, h.id, q.id)][0]
            assert q.pipe != other.pipe
        for p in ps:                                                   # a node and the remainder that complements it
            if p.kind == vte.VTE_PCTX_NODE and p.remainder >= 0:
                assert ps[p.remainder].pipe != p.pipe, (p.id, p.remainder)
        # queues are dealt to pipes in creation order: the k-th created belongs to pipe k % 4
        order = vte.vte_pool_creation_order(c)
        assert sorted(i for i in order if i >= 0) == list(range(len(ps)))
        assert all(i < 0 or ps[i].pipe == k % 4 for k, i in enumerate(order))
        assert sum(1 for i in order if i < 0) <= 3                     # few placeholder queues
    finally:
        vte.vte_shutdown(c)


def test_tput_plan_avoids_a_pipe_another_tenant_dispatches_on():
    c = make_ctx(remainders=vte.VTE_REMAINDERS_NONE)
    try:
        ps = infos(c)
        flat = vte.vte_desc_rmsnorm(c, A, A, A, 8, 1024, 1e-6)
        set_profile(c, flat, lambda w: 4e-6)                           # flat profile: stays on a leaf
        leaves = [p for p in ps if p.width == 32]
        busy = leaves[0]
        other = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        vte.vte_vstream_pin(other, busy.id)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        t0 = vte.vte_submit(other, flat)
        vte.vte_dispatcher_quiesce(c)
        vs = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        t1 = vte.vte_submit(vs, flat)
        vte.vte_dispatcher_quiesce(c)
        got = ps[bound(c)[t1]]
        assert got.width == 32 and got.pipe != busy.pipe
        finish(c, [t0, t1])
    finally:
        vte.vte_shutdown(c)


def test_tput_plan_does_not_renew_a_lease_while_an_older_op_has_nowhere_to_go():
    c = make_ctx(vte.VTE_MODE_PIPELINED)
    try:
        d = vte.vte_desc_gemv(c, A, A, A, 1, 4096, 4096, 0)
        set_profile(c, d, lambda w: 1e-3 * 32 / w)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        hog, late = vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT), vte.vte_vstream_create(c, vte.VTE_CLASS_BEST_EFFORT)
        t1 = vte.vte_submit(hog, d)
        vte.vte_dispatcher_quiesce(c)
        ps = infos(c)
        assert ps[bound(c)[t1]].width == 256                 # alone: the whole device
        t_late = vte.vte_submit(late, d)                     # nothing is left for it ...
        t2 = vte.vte_submit(hog, d)                          # ... and the holder's next op could reuse the lease
        vte.vte_dispatcher_quiesce(c)
        assert t_late not in bound(c) and t2 not in bound(c)  # it does not: the older op waits, so the lease drains
        vte.vte_fake_complete(c, t1)
        vte.vte_token_wait(c, t1)
        vte.vte_dispatcher_quiesce(c)
        b = bound(c)
        assert ps[b[t_late]].width + ps[b[t2]].width == 256 and not vte.vte_pool_conflict(c, b[t_late], b[t2])   # planned together
        finish(c, [t_late, t2])
    finally:
        vte.vte_shutdown(c)


def test_tput_plan_keeps_a_stream_on_its_open_lease_and_packs_newcomers_beside_taken_buddies():
    """Two seats of the plan that keep the pool whole: the next op of a vstream whose predecessor is
    still in flight is seated where that predecessor runs (a narrower free pCtx would make the stream
    hold two allocations), and a newcomer takes, among equally wide pCtxs on free pipes, the one
    nearest to a block that is already broken up, so that a whole half stays free for a tenant that scales."""
    c = make_ctx(vte.VTE_MODE_PIPELINED, remainders=vte.VTE_REMAINDERS_PER_LEVEL)
    try:
        flat = vte.vte_desc_rmsnorm(c, A, A, A, 8, 1024, 1e-6)
        set_profile(c, flat, lambda w: 4e-6)                 # gains nothing from more CUs: MinBind decides
        ps = infos(c)
        quarters = [p.id for p in ps if p.kind == vte.VTE_PCTX_NODE and p.width == 64]
        a, b = vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY), vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY)
        vte.vte_set_builtin_policy(c, vte.VTE_POLICY_TPUT_PLAN)
        # stream a sits on the first quarter of the SECOND half (pinned for its first op only)
        vte.vte_vstream_pin(a, quarters[2])
        t1 = vte.vte_submit(a, flat)
        vte.vte_dispatcher_quiesce(c)
        vte.vte_vstream_pin(a, -1)
        t2 = vte.vte_submit(a, flat)                         # predecessor in flight on that quarter; every leaf elsewhere is free
        vte.vte_dispatcher_quiesce(c)
        assert bound(c)[t1] == quarters[2] and bound(c)[t2] == quarters[2]
        # a newcomer that wants exactly a quarter: the other quarter of the second half, not one of the first
        heavy = vte.vte_desc_gemv(c, A, A, A, 1, 4096, 4096, 0)
        set_profile(c, heavy, {32: 2e-3, 64: 1e-3, 128: 1e-3, 192: 1e-3, 224: 1e-3, 256: 1e-3})
        t3 = vte.vte_submit(b, heavy)
        vte.vte_dispatcher_quiesce(c)
        got = bound(c)[t3]
        assert got == quarters[3], (got, quarters)           # completes the broken half instead of breaking the whole one
        finish(c, [t1, t2, t3])
    finally:
        vte.vte_shutdown(c)
