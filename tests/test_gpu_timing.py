"""GPU: device timing of selected launches (sampled, on the kernel's own dispatch) leaves results alone.
Needs an MI355X.  A context of its own: two pools alive at once exceed the queues the device keeps resident."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2603_15042_amd import inputs, vte

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    from paper_2603_15042_amd import harness
    return harness


# ---------- device timing of selected launches -------------------------------------------------
@pytest.mark.parametrize("mode", [vte.VTE_MODE_STRICT, vte.VTE_MODE_PIPELINED])
def test_timed_launches_are_sampled_and_leave_the_result_alone(H, mode):
    rows, cols = 4096, 4096
    x = inputs.normal_bf16(5, inputs.T_X, (rows, cols))
    g = inputs.normal_bf16(5, inputs.T_GAMMA, (cols,))
    dx, dg = H.to_dev(x), H.to_dev(g)
    y_ref, y = H.dev_empty((rows, cols)), H.dev_empty((rows, cols))
    torch.zeros(1, device="cuda")
    cfg = vte.vte_pool_cfg_default()
    cfg.mode = mode
    cfg.lookahead = 8
    cfg.device_timing_mask = 1 << vte.VTE_K_RMSNORM
    cfg.device_timing_stride = 4
    c2 = vte.vte_init(0, cfg)
    try:
        d = vte.vte_desc_rmsnorm(c2, dx, dg, y, rows, cols, 1e-6)
        root = vte.vte_pool_find(c2, vte.VTE_PCTX_NODE, 256)
        d_ref = vte.vte_desc_rmsnorm(c2, dx, dg, y_ref, rows, cols, 1e-6)
        vte.vte_token_wait(c2, vte.vte_bind_and_launch(c2, d_ref, root))
        alone = vte.vte_profile_measure_on(c2, d, root, 5, 20)
        vs = vte.vte_vstream_create(c2, vte.VTE_CLASS_LATENCY)
        vte.vte_set_builtin_policy(c2, vte.VTE_POLICY_WIDEST)
        vte.vte_stats_reset(c2)
        y.fill_(0x7FC1)
        torch.cuda.synchronize()
        vte.vte_token_wait(c2, vte.vte_submit_batch(vs, vte.desc_array([d] * 16)))
        recs = [r for r in vte.vte_stats_read(c2) if r.kernel == vte.VTE_K_RMSNORM]
        assert len(recs) == 16
        timed = [r.gpu_seconds for r in recs if r.gpu_seconds > 0]
        assert len(timed) == 4                              # every fourth
        for t in timed:                                     # the kernel's own duration, not a queueing time
            assert 0.3 * alone < t < 3.0 * alone + 20e-6, (t, alone)
        torch.cuda.synchronize()
        assert np.array_equal(H.to_bits(y), H.to_bits(y_ref))
    finally:
        vte.vte_shutdown(c2)


def test_pipelined_binding_makes_few_completion_records(H):
    """A stream marker idles its stream for a few microseconds, so PIPELINED binding makes one only
    where progress needs it: behind a quarter of the lookahead window, behind a launch a caller waits
    for, or when nothing recorded is pending — not behind every launch, as STRICT binding must."""
    rows, cols = 4096, 4096
    dx = H.to_dev(inputs.normal_bf16(5, inputs.T_X, (rows, cols)))
    dg = H.to_dev(inputs.normal_bf16(5, inputs.T_GAMMA, (cols,)))
    y = H.dev_empty((rows, cols))
    counts = {}
    for mode in (vte.VTE_MODE_PIPELINED, vte.VTE_MODE_STRICT):
        cfg = vte.vte_pool_cfg_default()
        cfg.mode = mode
        cfg.lookahead = 64
        c = vte.vte_init(0, cfg)
        try:
            d = vte.vte_desc_rmsnorm(c, dx, dg, y, rows, cols, 1e-6)
            vs = vte.vte_vstream_create(c, vte.VTE_CLASS_LATENCY)
            vte.vte_set_builtin_policy(c, vte.VTE_POLICY_WIDEST)
            vte.vte_stats_reset(c)
            n = 512
            mid = vte.vte_submit_batch(vs, vte.desc_array([d] * (n // 2)))
            last = vte.vte_submit_batch(vs, vte.desc_array([d] * (n // 2)))
            vte.vte_token_wait(c, mid)                    # a wait in the middle of the stream returns
            vte.vte_token_wait(c, last)
            st = vte.vte_stats(c)
            assert st.completed == n
            counts[mode] = st.completion_records
        finally:
            vte.vte_shutdown(c)
    assert counts[vte.VTE_MODE_STRICT] == 512
    assert counts[vte.VTE_MODE_PIPELINED] <= 512 // 8, counts
