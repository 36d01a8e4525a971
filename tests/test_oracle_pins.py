"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each pin is a closed form, exact rational arithmetic (fractions.Fraction), a
library routine (numpy float64 matmul / argmax) or a special case with a known
answer.  Together they are chosen so that a dropped term, a transposed
operand, a wrong index, a missing eps, a biased-vs-unbiased variance mix-up or
a double rounding in the bf16 conversion fails at least one of them.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2603_15042_amd import inputs


# ---------- independent helpers written for the tests only ----------------------
def bits_to_fraction(h):
    """Exact rational value of a (finite) bf16 bit pattern."""
    h = int(h)
    s = -1 if h >> 15 else 1
    e = (h >> 7) & 0xFF
    m = h & 0x7F
    if e == 0:
        return s * Fraction(m, 1 << 7) * Fraction(2) ** (-126)
    return s * (1 + Fraction(m, 1 << 7)) * Fraction(2) ** (e - 127)


def np_round_bf16(x):
    """float64 -> bf16 bits by integer rounding of the binary64 fraction (normal range only)."""
    u = np.ascontiguousarray(x, dtype=np.float64).view(np.uint64).copy()
    lsb = (u >> np.uint64(45)) & np.uint64(1)
    u += np.uint64((1 << 44) - 1) + lsb
    u &= ~np.uint64((1 << 45) - 1)
    f = u.view(np.float64).astype(np.float32)
    return (f.view(np.uint32) >> 16).astype(np.uint16)


def f(bits):
    return inputs.bf16_to_f32(bits).astype(np.float64)


# ---------- bf16 conversions ------------------------------------------------------
def test_bf16_roundtrip_all_patterns():
    allb = np.arange(65536, dtype=np.uint16)
    v = oracle.bf16_to_f64(allb)
    fin = np.isfinite(v)
    # value equals the float32 whose upper half is the pattern
    assert np.array_equal(v[fin], f(allb)[fin])
    back = oracle.f64_to_bf16(v[fin])
    assert np.array_equal(back, allb[fin])
    # a few exact rationals
    for h in (0x3F80, 0x4049, 0xC2F7, 0x0001, 0x0080, 0x7F7F):
        assert Fraction(float(v[h])) == bits_to_fraction(h)


def test_bf16_rounding_ties_and_single_rounding():
    one = 1.0
    ulp = 2.0 ** -7
    cases = {
        one + ulp / 2: 0x3F80,             # tie -> even (1.0)
        one + 3 * ulp / 2: 0x3F82,         # tie -> even (1 + 2 ulp)
        one + ulp / 2 + 2.0 ** -40: 0x3F81,  # just above a tie: must go up (a float32 detour would lose it)
        one + ulp / 2 - 2.0 ** -40: 0x3F80,
        -(one + ulp / 2 + 2.0 ** -40): 0xBF81,
        255.5: 0x4380,                     # 255.5 -> tie between 255 and 256 -> 256 (even)
        0.0: 0x0000,
        2.0 ** -133: 0x0001,               # smallest subnormal
        2.0 ** -134: 0x0000,               # tie to even at the bottom
        3.3895313892515355e38: 0x7F7F,     # largest finite bf16
    }
    for val, want in cases.items():
        got = int(oracle.f64_to_bf16(np.array([val]))[0])
        assert got == want, (val, hex(got), hex(want))
    rng = np.random.default_rng(1)
    x = rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))
    assert np.array_equal(oracle.f64_to_bf16(x), np_round_bf16(x))


# ---------- RMSNorm ------------------------------------------------------------------
@pytest.mark.parametrize("n", [8, 1024, 4096, 1000])
def test_rmsnorm_unit_rms_rows(n):
    eps = 1e-6
    sign = np.where(np.arange(n) % 3 == 0, -1.0, 1.0)
    for c in (1.0, 0.5, 4.0):
        x = inputs.bf16_bits((sign * c).astype(np.float32))[None, :]
        g = inputs.bf16_bits(np.ones(n, np.float32))
        ref = oracle.rmsnorm(x, g, eps)
        want = sign * c / math.sqrt(c * c + eps)
        assert np.allclose(ref[0], want, rtol=1e-15, atol=0)
    # c = 1 rounds to exactly +-1.0 in bf16
    x = inputs.bf16_bits(sign.astype(np.float32))[None, :]
    out = oracle.f64_to_bf16(oracle.rmsnorm(x, inputs.bf16_bits(np.ones(n, np.float32)), eps))
    assert np.array_equal(f(out)[0], sign)


def test_rmsnorm_one_hot_zero_row_and_gamma():
    n, eps = 1024, 1e-6
    g = inputs.uniform_bf16(3, inputs.T_GAMMA, (n,), 0.5, 1.5)
    x = np.zeros((3, n), np.float32)
    x[0, 17] = 3.0
    x[1, 1023] = -0.25
    xb = inputs.bf16_bits(x)
    ref = oracle.rmsnorm(xb, g, eps)
    gv = f(g)
    assert ref[0, 17] == pytest.approx(3.0 / math.sqrt(9.0 / n + eps) * gv[17], rel=1e-15)
    assert ref[1, 1023] == pytest.approx(-0.25 / math.sqrt(0.0625 / n + eps) * gv[1023], rel=1e-15)
    assert abs(ref[0, 17] / gv[17] - 32.0) < 1e-2      # -> sqrt(n) as eps -> 0
    mask = np.ones((3, n), bool)
    mask[0, 17] = mask[1, 1023] = False
    assert np.all(ref[mask] == 0.0)                     # zero row stays finite and zero
    assert np.all(np.isfinite(ref))


def test_rmsnorm_exact_rational_small():
    n, eps = 7, Fraction(1, 1000000)
    x, g = inputs.rmsnorm_case(seed=5, rows=3, cols=n)
    ref = oracle.rmsnorm(x, g, float(eps))
    for r in range(3):
        xs = [bits_to_fraction(h) for h in x[r]]
        ms = sum(v * v for v in xs) / n + Fraction(float(eps))   # eps as the double the oracle receives
        for i in range(n):
            want = float(xs[i] * bits_to_fraction(g[i])) / math.sqrt(float(ms))
            assert ref[r, i] == pytest.approx(want, rel=4e-16 * 8, abs=0)


def test_rmsnorm_mean_not_sum_and_row_independence():
    x, g = inputs.rmsnorm_case(seed=0, rows=8, cols=1024)
    ref = oracle.rmsnorm(x, g)
    xv, gv = f(x), f(g)
    want = xv * gv / np.sqrt((xv * xv).mean(axis=1, keepdims=True) + 1e-6)
    assert np.allclose(ref, want, rtol=1e-13, atol=0)
    # output rows have RMS ~ RMS(gamma-weighted unit rows)
    one = oracle.rmsnorm(x[3:4], g)
    assert np.array_equal(one[0], ref[3])


# ---------- LayerNorm ---------------------------------------------------------------
def test_layernorm_constant_and_alternating_rows():
    n, eps = 1024, 1e-6
    _, g, b = inputs.layernorm_case(seed=2, rows=1, cols=n)
    const = inputs.bf16_bits(np.full((1, n), 2.5, np.float32))
    ref = oracle.layernorm(const, g, b, eps)
    assert np.array_equal(ref[0], f(b))                 # (x - mu) == 0 exactly
    alt = np.where(np.arange(n) % 2 == 0, 1.0, -1.0)
    ref = oracle.layernorm(inputs.bf16_bits(alt.astype(np.float32))[None, :], g, b, eps)
    want = alt * f(g) / math.sqrt(1.0 + eps) + f(b)
    assert np.allclose(ref[0], want, rtol=1e-14, atol=1e-16)


def test_layernorm_biased_variance_and_shift_invariance():
    x, g, b = inputs.layernorm_case(seed=4, rows=4, cols=96)
    ref = oracle.layernorm(x, g, b, 1e-6)
    xv = f(x)
    mu = xv.mean(axis=1, keepdims=True)
    var = ((xv - mu) ** 2).mean(axis=1, keepdims=True)   # divide by n, not n-1
    want = (xv - mu) / np.sqrt(var + 1e-6) * f(g) + f(b)
    assert np.allclose(ref, want, rtol=1e-12, atol=1e-15)
    unb = (xv - mu) / np.sqrt(var * 96 / 95 + 1e-6) * f(g) + f(b)
    assert not np.allclose(ref, unb, rtol=1e-4, atol=0)
    # exact rational check of one row
    xs = [bits_to_fraction(h) for h in x[1]]
    m = sum(xs) / 96
    v = sum((t - m) ** 2 for t in xs) / 96
    for i in (0, 50, 95):
        want_i = float(xs[i] - m) / math.sqrt(float(v) + 1e-6) * float(bits_to_fraction(g[i])) + float(bits_to_fraction(b[i]))
        assert ref[1, i] == pytest.approx(want_i, rel=1e-13, abs=1e-15)


# ---------- GEMV -----------------------------------------------------------------------
def test_gemv_identity_permutation_ones():
    K = 512
    X = inputs.normal_bf16(7, inputs.T_XB, (4, K))
    eye = inputs.bf16_bits(np.eye(K, dtype=np.float32))
    y = oracle.gemv(eye, X)
    assert np.array_equal(oracle.f64_to_bf16(y), X)      # Y = X bit-exactly
    perm = np.random.default_rng(0).permutation(K)
    P = np.zeros((K, K), np.float32)
    P[np.arange(K), perm] = 1.0                          # row n picks x[perm[n]]
    y = oracle.gemv(inputs.bf16_bits(P), X)
    assert np.array_equal(oracle.f64_to_bf16(y), X[:, perm])
    ones = inputs.bf16_bits(np.ones((3, 4096), np.float32))
    y = oracle.gemv(ones, inputs.bf16_bits(np.ones((2, 4096), np.float32)))
    assert np.all(y == 4096.0) and y.shape == (2, 3)


def test_gemv_layout_is_N_by_K_and_matches_blas():
    W, X = inputs.gemv_case(seed=0, B=3, N=40, K=256)
    y = oracle.gemv(W, X)
    want = f(X) @ f(W).T                                 # numpy float64 matmul
    assert y.shape == (3, 40)
    assert np.allclose(y, want, rtol=1e-12, atol=1e-13)
    # single nonzero weight W[n0,k0] picks X[:,k0] into column n0 only
    Wz = np.zeros((40, 256), np.float32)
    Wz[5, 200] = 2.0
    y = oracle.gemv(inputs.bf16_bits(Wz), X)
    assert np.array_equal(y[:, 5], 2.0 * f(X)[:, 200])
    assert np.count_nonzero(y) == np.count_nonzero(f(X)[:, 200])


def test_gemv_exact_rational_and_reverse_order():
    W, X = inputs.gemv_case(seed=9, B=2, N=5, K=64)
    y = oracle.gemv(W, X)
    for b in range(2):
        for n in range(5):
            exact = sum(bits_to_fraction(W[n, k]) * bits_to_fraction(X[b, k]) for k in range(64))
            mag = sum(abs(bits_to_fraction(W[n, k]) * bits_to_fraction(X[b, k])) for k in range(64))
            assert abs(Fraction(float(y[b, n])) - exact) <= mag * Fraction(64, 2 ** 53)
    W, X = inputs.gemv_case(seed=1, B=4, N=64, K=4096)
    fwd, rev = oracle.gemv(W, X), oracle.gemv_reverse(W, X)
    scale = oracle.gemv_abs(W, X)
    assert np.all(np.abs(fwd - rev) <= 1e-12 * scale)
    assert np.all(scale >= np.abs(fwd))


def test_gemv_exact_integer_inputs_any_order():
    # integers: every product and partial sum is exactly representable -> order cannot matter
    W = inputs.int_bf16(3, inputs.T_W, (16, 1024), -8, 8)
    X = inputs.int_bf16(3, inputs.T_XB, (2, 1024), -8, 8, -2)
    fwd, rev = oracle.gemv(W, X), oracle.gemv_reverse(W, X)
    assert np.array_equal(fwd, rev)
    want = (f(X).astype(np.float64) @ f(W).T.astype(np.float64))
    assert np.array_equal(fwd, want)
    assert np.array_equal(fwd * 4, np.round(fwd * 4))


def test_thread_count_does_not_change_results():
    W, X = inputs.gemv_case(seed=2, B=2, N=37, K=512)
    a = oracle.gemv(W, X, threads=1)
    for t in (2, 3, 8):
        assert np.array_equal(a, oracle.gemv(W, X, threads=t))
    x, g = inputs.rmsnorm_case(seed=1, rows=5, cols=64)
    assert np.array_equal(oracle.rmsnorm(x, g, threads=1), oracle.rmsnorm(x, g, threads=4))


# ---------- SiLU epilogue ---------------------------------------------------------------
def test_silu_limits_and_gate_up():
    assert oracle.silu(0.0) == 0.0
    assert oracle.silu(40.0) == pytest.approx(40.0, rel=1e-15)
    assert -1e-15 < oracle.silu(-40.0) <= 0.0
    assert oracle.silu(1.0) == pytest.approx(1.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    assert oracle.silu(-2.0) == pytest.approx(-2.0 / (1.0 + math.exp(2.0)), rel=1e-15)
    F_, K = 12, 128
    W = inputs.normal_bf16(4, inputs.T_WGU, (2 * F_, K), 0.0, 0.1)
    X = inputs.normal_bf16(4, inputs.T_XB, (3, K))
    act = oracle.gemv_silu_mul(W, X)
    y = f(X) @ f(W).T
    g, u = y[:, :F_], y[:, F_:]                          # gate rows first, then up rows
    assert np.allclose(act, g / (1 + np.exp(-g)) * u, rtol=1e-12, atol=1e-15)
    Wz = W.copy()
    Wz[F_:] = 0                                          # u = 0 -> act = 0
    assert np.all(oracle.gemv_silu_mul(Wz, X) == 0.0)
    Wz = W.copy()
    Wz[:F_] = 0                                          # g = 0 -> silu = 0
    assert np.all(oracle.gemv_silu_mul(Wz, X) == 0.0)


# ---------- argmax / LM head --------------------------------------------------------------
@pytest.mark.parametrize("V", [1, 2, 7, 64, 1000, 4097])
def test_argmax_brute_force(V):
    rng = np.random.default_rng(V)
    lg = rng.standard_normal((4, V))
    for b, pos in enumerate({0, V - 1, V // 2, min(V - 1, 63)}):
        if b < 4:
            lg[b, pos] = 10.0 + b
    tok, margin = oracle.argmax(lg)
    assert np.array_equal(tok, np.argmax(lg, axis=1).astype(np.int32))
    if V >= 2:
        srt = np.sort(lg, axis=1)
        assert np.allclose(margin, srt[:, -1] - srt[:, -2], rtol=0, atol=0)
    # duplicated maxima -> lowest index; all-equal -> 0
    if V >= 7:
        d = np.zeros((2, V))
        d[0, [5, 3, V - 1]] = 2.0
        tok, margin = oracle.argmax(d)
        assert tok[0] == 3 and tok[1] == 0 and margin[0] == 0.0 and margin[1] == 0.0
        d[0, :] = -np.inf
        d[0, 6] = -1e300
        d[1, 2] = np.nan                                   # NaN never wins
        d[1, 4] = 1e-300
        tok, _ = oracle.argmax(d)
        assert tok[0] == 6 and tok[1] == 4
    allnan = np.full((1, V), np.nan)
    assert oracle.argmax(allnan)[0][0] == 0


def test_lmhead_planted_token():
    V, K = 777, 128
    W = inputs.normal_bf16(6, inputs.T_WLM, (V, K), 0.0, 0.02)
    H = inputs.normal_bf16(6, inputs.T_XB, (3, K))
    # plant: row v* of W equals 0.5 * h_b  => logit = 0.5*|h|^2, far above N(0, 0.02^2 |h|^2)
    for b, v in enumerate((0, 400, 776)):
        W[v] = oracle.f64_to_bf16(0.5 * f(H[b]))
    logits, tok, margin = oracle.lmhead_argmax(W, H)
    assert list(tok) == [0, 400, 776]
    assert np.allclose(logits, f(H) @ f(W).T, rtol=1e-12, atol=1e-14)
    assert np.all(margin > 0)
    _, tok2, _ = oracle.lmhead_argmax(W, H, want_logits=False)
    assert np.array_equal(tok, tok2)


# ---------- gather / GEMM sample / chain ---------------------------------------------------
def test_gather_rows():
    E = inputs.normal_bf16(1, inputs.T_EMB, (50, 32))
    tok = np.array([49, 0, 7, 7], np.int32)
    assert np.array_equal(oracle.gather(E, tok), E[tok])
    shp = inputs.DecodeShapes(D=32, Nqkv=48, F=64, V=50)
    assert np.array_equal(inputs.embedding_rows(1, shp, tok), E[tok])


def test_gemm_sample_matches_blas_and_layout():
    A = inputs.normal_bf16(0, inputs.T_GEMM_A, (48, 96))
    Bm = inputs.normal_bf16(0, inputs.T_GEMM_B, (40, 96))
    C = f(A) @ f(Bm).T                                      # C = A B^T, both K-contiguous
    rows = np.array([0, 47, 13])
    cols = np.array([39, 1])
    assert np.allclose(oracle.gemm_rows(A, Bm, rows), C[rows], rtol=1e-12, atol=1e-12)
    assert np.allclose(oracle.gemm_cols(A, Bm, cols), C[:, cols].T, rtol=1e-12, atol=1e-12)


def test_decode_step_is_the_listed_composition():
    shp = inputs.DecodeShapes(D=64, Nqkv=96, F=160, V=300)
    w = inputs.decode_weights(11, shp)
    # larger weights so that activations do not vanish through the short chain
    for k in ("Wqkv", "Wo", "Wgu", "Wd"):
        w[k] = inputs.normal_bf16(11, hash(k) % 1000 + 100, w[k].shape, 0.0, 0.15)
    tok = inputs.tokens(11, inputs.T_TOK0, 3, shp.V)
    o = oracle.decode_step(w, tok, shp, want_logits=True)
    r = np_round_bf16
    h0 = w["E"][tok]
    hv = f(h0)
    n = r(hv * f(w["gamma"]) / np.sqrt((hv * hv).mean(1, keepdims=True) + 1e-6))
    qkv = r(f(n) @ f(w["Wqkv"]).T)
    a = qkv[:, :shp.D]                                    # the Q slice feeds the O projection
    ob = r(f(a) @ f(w["Wo"]).T)
    gu = f(ob) @ f(w["Wgu"]).T
    g, u = gu[:, :shp.F], gu[:, shp.F:]
    act = r(g / (1 + np.exp(-g)) * u)
    d = r(f(act) @ f(w["Wd"]).T)
    logits = f(d) @ f(w["Wlm"]).T

    def close_bits(a_, b_, name):
        # numpy's blocked float64 sums may differ in the last bits and flip a rounding tie: allow 1 ulp on <1%
        diff = a_.astype(np.int32) - b_.astype(np.int32)
        assert np.all(np.abs(diff) <= 1), name
        assert np.mean(diff != 0) < 0.01, name
    assert np.array_equal(o["h0"], h0)
    close_bits(o["n"], n, "n")
    close_bits(o["qkv"], qkv, "qkv")
    # downstream of a possible 1-ulp flip compare stage by stage from the oracle's own inputs
    close_bits(o["o"], r(f(o["qkv"][:, :shp.D]) @ f(w["Wo"]).T), "o")
    gu = f(o["o"]) @ f(w["Wgu"]).T
    close_bits(o["act"], r(gu[:, :shp.F] / (1 + np.exp(-gu[:, :shp.F])) * gu[:, shp.F:]), "act")
    close_bits(o["d"], r(f(o["act"]) @ f(w["Wd"]).T), "d")
    lg = f(o["d"]) @ f(w["Wlm"]).T
    assert np.allclose(o["logits"], lg, rtol=1e-11, atol=1e-13)
    assert np.array_equal(o["next"], np.argmax(lg, axis=1))
    assert np.count_nonzero(f(o["act"])) > 0.9 * o["act"].size
    assert logits.shape == (3, shp.V)


# ---------- softmax probability of a token (Sec. 7.2) ---------------------------------------------
def test_softmax_prob_closed_forms():
    V = 1000
    # all logits equal -> 1 / V, whatever the level
    for level in (0.0, -50.0, 80.0):
        p = oracle.softmax_prob(np.full((2, V), level, np.float32), [0, V - 1])
        assert np.allclose(p, 1.0 / V, rtol=1e-14)
    # two live entries with logits 0 and ln 3, everything else -inf -> 1/4 and 3/4
    lg = np.full((2, V), -np.inf, np.float32)
    lg[:, 7] = 0.0
    lg[:, 900] = np.float32(np.log(3.0))
    p = oracle.softmax_prob(lg, [7, 900])
    ln3 = float(np.float32(np.log(3.0)))
    assert abs(p[0] - 1.0 / (1.0 + np.exp(ln3))) < 1e-15 and abs(p[1] - np.exp(ln3) / (1.0 + np.exp(ln3))) < 1e-15
    assert abs(p.sum() - 1.0) < 1e-15
    assert oracle.softmax_prob(lg, [3, 3]).tolist() == [0.0, 0.0]      # a dead entry has probability 0
    # one live entry -> 1; a token outside the vocabulary -> 0
    one = np.full((1, 64), -np.inf, np.float32)
    one[0, 5] = 12.5
    assert oracle.softmax_prob(one, [5])[0] == 1.0
    assert oracle.softmax_prob(one, [64])[0] == 0.0 and oracle.softmax_prob(one, [-1])[0] == 0.0


def test_softmax_prob_against_an_independent_evaluation():
    import scipy.special
    rng = np.random.default_rng(4)
    lg = (rng.standard_normal((5, 4097)) * 8).astype(np.float32)
    tok = rng.integers(0, 4097, size=5)
    ref = scipy.special.softmax(lg.astype(np.float64), axis=1)[np.arange(5), tok]
    got = oracle.softmax_prob(lg, tok)
    assert np.allclose(got, ref, rtol=1e-12, atol=0)
    # shifting a row by a constant changes nothing (logits on a 2^-10 grid, so the shifted float32 values are exact)
    grid = (rng.integers(-8192, 8192, size=(5, 4097)) / 1024.0).astype(np.float32)
    shifted = (grid.astype(np.float64) + 64.0).astype(np.float32)
    assert np.array_equal(shifted.astype(np.float64) - 64.0, grid.astype(np.float64))
    assert np.allclose(oracle.softmax_prob(shifted, tok), oracle.softmax_prob(grid, tok), rtol=1e-12)
    # the probabilities of all tokens of a row sum to one
    row = lg[:1].repeat(64, axis=0)
    assert abs(oracle.softmax_prob(row, np.arange(64)).sum() - scipy.special.softmax(lg[0].astype(np.float64))[:64].sum()) < 1e-13
