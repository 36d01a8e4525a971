"""CPU checks of the matrix-core tree emulator (tests/tree_emulator.py) against what arithmetic fixes:
it is test infrastructure for the GPU tests, so a slip in it must not go unnoticed here."""
import numpy as np

import oracle
import tree_emulator as te
from paper_2603_15042_amd import inputs


def _bits(a):
    return inputs.bf16_bits(np.asarray(a, np.float32))


def test_small_integers_sum_exactly_whatever_the_grouping():
    rng = np.random.default_rng(0)
    W = rng.integers(-8, 9, size=(24, 200)).astype(np.float32)
    X = rng.integers(-8, 9, size=(5, 200)).astype(np.float32)
    exact = (X.astype(np.int64) @ W.astype(np.int64).T).astype(np.float32)
    assert np.array_equal(te.gemv_rows_sums(_bits(W), _bits(X)), exact)
    assert np.array_equal(te.gemv_ksplit_sums(_bits(W), _bits(X), 1, 8), exact)
    assert np.array_equal(te.gemv_dot2_sums(_bits(W), _bits(X), 1), exact)


def test_zero_groups_and_a_ragged_tail_leave_the_accumulator_alone():
    W = np.zeros((3, 40), np.float32); X = np.ones((2, 40), np.float32)
    W[:, 3] = [1.5, -2.0, 0.25]; W[:, 36] = [4.0, 4.0, 4.0]
    got = te.gemv_rows_sums(_bits(W), _bits(X))
    assert np.array_equal(got, np.tile(np.array([5.5, 2.0, 4.25], np.float32), (2, 1)))


def test_a_single_group_cuts_small_products_at_2_to_the_minus_24_of_the_largest():
    # 1 + 2^-25: the small product lies wholly below the grid 2^(0-24) and is dropped, not rounded in
    W = np.array([[1.0, 2.0 ** -13] + [0.0] * 6], np.float32); X = np.array([[1.0, 2.0 ** -12] + [0.0] * 6], np.float32)
    assert te.gemv_rows_sums(_bits(W), _bits(X))[0, 0] == np.float32(1.0)
    # 1 + 2^-23 is on the grid and survives; -(1) + ... checks the sign handling
    X2 = np.array([[1.0, 2.0 ** -10] + [0.0] * 6], np.float32)
    assert te.gemv_rows_sums(_bits(W), _bits(X2))[0, 0] == np.float32(1.0 + 2.0 ** -23)
    assert te.gemv_rows_sums(_bits(-W), _bits(X2))[0, 0] == np.float32(-(1.0 + 2.0 ** -23))


def test_emulated_sums_stay_within_the_error_bound_of_the_plain_definition():
    N, K, B = 64, 1160, 7
    W, X = inputs.gemv_case(seed=3, B=B, N=N, K=K)
    ref = inputs.bf16_to_f32(W).astype(np.float64) @ inputs.bf16_to_f32(X).astype(np.float64).T   # [N, B]
    mag = np.abs(inputs.bf16_to_f32(W)).astype(np.float64) @ np.abs(inputs.bf16_to_f32(X)).astype(np.float64).T
    for got in (te.gemv_rows_sums(W, X), te.gemv_ksplit_sums(W, X, 4, 8), te.gemv_ksplit_sums(W, X, 8, 4), te.gemv_dot2_sums(W, X, 2)):
        err = np.abs(got.astype(np.float64).T - ref)
        assert np.all(err <= (K / 8 + 8) * 2.0 ** -23 * mag)          # one rounding and one cut per group of 8
    bf16_err = np.abs(inputs.bf16_to_f32(te._f32_to_bf16(te.gemv_rows_sums(W, X))).astype(np.float64).T - ref)
    assert np.all(bf16_err <= 2e-2)
    assert oracle.gemv(W, X).shape == (B, N)


def test_a_smaller_accumulator_is_dropped_toward_minus_infinity_at_the_groups_grid():
    # group 1 leaves acc = -1.5 * 2^-24; group 2 is the single product 1 * 1 (grid 2^-24): the accumulator
    # becomes -2 grid units, not -1 (toward zero) and not rounded: 1 - 2^-23
    W = np.zeros((1, 16), np.float32); X = np.zeros((1, 16), np.float32)
    W[0, 0], X[0, 0] = -1.5 * 2.0 ** -12, 2.0 ** -12
    W[0, 8], X[0, 8] = 1.0, 1.0
    assert te.gemv_rows_sums(_bits(W), _bits(X))[0, 0] == np.float32(1.0 - 2.0 ** -23)
    # the same with a positive remainder: +1.5 * 2^-24 -> +1 unit
    W[0, 0] = 1.5 * 2.0 ** -12
    assert te.gemv_rows_sums(_bits(W), _bits(X))[0, 0] == np.float32(1.0)   # 1 + 2^-24 exactly: a tie, to even


def test_the_row_split_kernel_walks_k_from_a_start_fixed_by_the_outputs_block_of_512():
    """gemv_rows_kernel_sums: output block j (512 outputs) starts at step (j mod 32) * steps // 32 and wraps
    around; block 0 is the plain ascending chain.  Planted values whose sum depends on the order show the
    start, and exact inputs do not care."""
    rng = np.random.default_rng(3)
    K, N = 4096, 1100                                     # 32 steps: block 1 starts at step 1, block 2 at step 2
    W = rng.integers(-4, 5, size=(N, K)).astype(np.float32)
    X = rng.integers(-4, 5, size=(2, K)).astype(np.float32)
    exact = (X.astype(np.int64) @ W.astype(np.int64).T).astype(np.float32)
    assert np.array_equal(te.gemv_rows_kernel_sums(_bits(W), _bits(X)), exact)
    # 1 in step 0, 2^-24 in step 1, -1 in step 31: ascending from step 0 the small term is lost beside the 1
    # (sum 0); started at step 1 or 2 it meets 0 or survives the cancellation of 1 and -1
    W = np.zeros((N, K), np.float32)
    W[:, 0], W[:, 128], W[:, 31 * 128] = 1.0, 2.0 ** -24, -1.0
    X = np.ones((1, K), np.float32)
    got = te.gemv_rows_kernel_sums(_bits(W), _bits(X))[0]
    assert np.all(te.gemv_rows_sums(_bits(W), _bits(X))[0] == 0.0)
    assert np.all(got[:512] == 0.0) and np.all(got[512:] == np.float32(2.0 ** -24))
    # 1160 elements are 10 steps: blocks 0 to 3 start at step 0 (3 * 10 // 32 = 0), block 4 at step 1
    Ws, Xs = inputs.normal_bf16(3, inputs.T_W, (2100, 1160), 0.0, 1.0), inputs.normal_bf16(3, inputs.T_XB, (3, 1160))
    a, b = te.gemv_rows_kernel_sums(Ws, Xs), te.gemv_rows_sums(Ws, Xs)
    assert np.array_equal(a[:, :2048], b[:, :2048]) and not np.array_equal(a[:, 2048:], b[:, 2048:])


def test_a_sum_that_cancels_down_a_binade_keeps_the_guard_bit():
    """One accumulation step as the device performed it (v_mfma_f32_16x16x32_bf16, one group of 8 products;
    operands and results read back from the row-split kernel): the accumulator 4.0066504 sets the grid, the
    group's total is negative and takes the sum just below 4.  The exact sum lies 0.493 ulp below 0x407f0149
    and 0.507 ulp above 0x407f0148; the instruction returns the former.  A rule that drops the group's
    total to the accumulator's 32-bit window before adding (no guard bit) returns the latter."""
    acc = np.array([[np.uint32(0x4080367b)]], dtype=np.uint32).view(np.float32)
    w = np.array([[0x3b03, 0x3d52, 0xb5e8, 0xbc01, 0xbb2b, 0xb882, 0xbc93, 0x3abd]], dtype=np.uint16)
    x = np.array([[0xbe8d, 0xbddc, 0xbf43, 0x3fa9, 0x3ed2, 0x3f31, 0x3e5b, 0xbf0d]], dtype=np.uint16)
    got = te.mfma_chain(acc.copy(), te._bf16_to_f32(w), te._bf16_to_f32(x), 0, 8)
    assert got.view(np.uint32)[0, 0] == 0x407f0149
    # the same step is the correctly rounded sum here (exact arithmetic in rationals)
    from fractions import Fraction
    exact = Fraction(float(acc[0, 0])) + sum(Fraction(float(a)) * Fraction(float(b))
                                             for a, b in zip(te._bf16_to_f32(w)[0], te._bf16_to_f32(x)[0]))
    lo, hi = np.array([0x407f0148, 0x407f0149], dtype=np.uint32).view(np.float32)
    assert abs(Fraction(float(hi)) - exact) < abs(Fraction(float(lo)) - exact)
