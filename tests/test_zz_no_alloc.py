"""The allocation-free LM head + greedy token (vte_lmhead_argmax_static) against the descriptor
pair it is a variant of (vte_desc_lmhead_argmax + vte_desc_argmax_finish): same kernels and
plan, so tokens and fp32 logits must be equal bit for bit.  Two calls in a row share the
library's static scratch array; the second is smaller, so stale candidates of the first lie
behind its own."""
import numpy as np
import pytest
import torch

from paper_2603_15042_amd import harness as H, inputs, vte

pytestmark = pytest.mark.gpu


def _reference(ctx, W, X, B, V, K):
    tok = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    logits = torch.zeros((B, V), dtype=torch.float32, device="cuda")
    ws = H.dev_zeros_bytes(vte.vte_lmhead_workspace_bytes(B, V, K))
    lm = vte.vte_desc_lmhead_argmax(ctx, W, X, tok, logits, ws, B, V, K)
    fin = vte.vte_desc_argmax_finish(ctx, lm)
    p = H.pctx_of_width(ctx, 256)
    H.run_on(ctx, lm, p)
    H.run_on(ctx, fin, p)
    torch.cuda.synchronize()
    out = tok.cpu().numpy().copy(), logits.cpu().numpy().copy()
    vte.vte_desc_destroy(fin)
    vte.vte_desc_destroy(lm)
    return out


def _static(W, X, B, V, K, with_logits=True):
    tok = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    logits = torch.zeros((B, V), dtype=torch.float32, device="cuda") if with_logits else None
    torch.cuda.synchronize()
    vte.vte_lmhead_argmax_static(0, W, X, tok, logits, B, V, K)   # null stream; no allocation inside
    torch.cuda.synchronize()
    return tok.cpu().numpy().copy(), (logits.cpu().numpy().copy() if with_logits else None)


def test_static_lmhead_equals_the_descriptor_pair_on_two_calls_in_a_row():
    assert vte.vte_static_scratch_bytes() == 1 << 20
    ctx = H.make_ctx()
    try:
        cases = [(8, 20011, 1024, 7), (3, 4099, 512, 8)]       # the second is smaller in B, V and K
        inputs_dev = []
        for B, V, K, seed in cases:
            W = H.to_dev(inputs.normal_bf16(seed, 1, (V, K), 0.0, K ** -0.5))
            X = H.to_dev(inputs.normal_bf16(seed, 2, (B, K)))
            inputs_dev.append((W, X))
        got = [_static(W, X, B, V, K) for (B, V, K, _), (W, X) in zip(cases, inputs_dev)]   # back to back
        for (B, V, K, _), (W, X), (tok_s, lg_s) in zip(cases, inputs_dev, got):
            tok_r, lg_r = _reference(ctx, W, X, B, V, K)
            assert np.array_equal(tok_s, tok_r), (B, V, K, tok_s, tok_r)
            assert np.array_equal(lg_s.view(np.uint32), lg_r.view(np.uint32)), (B, V, K)
            assert np.array_equal(tok_r, np.argmax(lg_r, axis=1).astype(np.int32))   # a real maximum, not a stale one
        # without the logits dump, and at a batch of the row-split kind
        B, V, K = 40, 8200, 1024
        W = H.to_dev(inputs.normal_bf16(9, 1, (V, K), 0.0, K ** -0.5))
        X = H.to_dev(inputs.normal_bf16(9, 2, (B, K)))
        tok_s, _ = _static(W, X, B, V, K, with_logits=False)
        tok_r, _ = _reference(ctx, W, X, B, V, K)
        assert np.array_equal(tok_s, tok_r)
    finally:
        vte.vte_shutdown(ctx)


def test_static_lmhead_rejects_what_does_not_fit_and_bad_arguments():
    W = torch.zeros(16, dtype=torch.int16, device="cuda")
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(vte.VteError) as e:   # 2^21 rows at batch 3: 4.7 MB of candidates; rejected before any launch
        vte.vte_lmhead_argmax_static(0, W, W, tok, None, 3, 1 << 21, 4096)
    assert e.value.code == vte.VTE_EINVAL and "scratch" in str(e.value)
    with pytest.raises(vte.VteError):
        vte.vte_lmhead_argmax_static(0, W, W, None, None, 3, 1000, 512)
    with pytest.raises(vte.VteError):
        vte.vte_lmhead_argmax_static(0, W, W, tok, None, 65, 1000, 512)
