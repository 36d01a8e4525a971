"""Shared pieces of the GPU parity tests: one context per module, tolerance rule."""
import numpy as np

from paper_2603_15042_amd import inputs


def f64(bits):
    return inputs.bf16_to_f32(bits).astype(np.float64)


def bf16_close(gpu_bits, ref, what=""):
    """Tolerance on bf16 outputs against the UNROUNDED double reference:
    |y - ref| <= 2e-2, or within half a bf16 ulp of ref plus fp32-accumulation slack
    (half an ulp exceeds 2e-2 once |ref| >= 8).  Returns (max abs err, max err in ulps)."""
    y = f64(gpu_bits)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(y - ref)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -126))) - 7)
    ok = (err <= 2e-2) | (err <= 0.5 * ulp * (1 + 1e-3) + 1e-6 * np.abs(ref))
    assert np.all(np.isfinite(y)), what
    assert np.all(ok), "%s: max abs err %.4g, worst %.3f ulp" % (what, err.max(), (err / ulp).max())
    return float(err.max()), float((err / ulp).max())
