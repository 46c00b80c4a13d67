"""Pins for the oracle's decompression and update (Algorithm 2, lines 7 and 8): Delta = P^ Q+^T and
x+ = x - Delta.  Each pin fails for a plausible mistake: a transposed factor, a wrong sign, a dropped
rank term, an update that adds instead of subtracting."""
import numpy as np
import pytest


def _rng(seed):
    return np.random.default_rng(seed)


def test_delta_of_small_integer_factors_is_the_exact_integer_product(ref):
    """Integers up to 8 in the factors: every product and partial sum is an integer below 2^24,
    exact in fp32, so the result must equal the integer matrix product bit for bit."""
    rng = _rng(0)
    n, m, r = 19, 23, 5                                           # non-square, odd: a transposed operand would not fit
    P = rng.integers(-8, 9, size=(n, r))
    Q = rng.integers(-8, 9, size=(m, r))
    want = P @ Q.T
    got = ref.decompress(P.astype(np.float32), Q.astype(np.float32))
    assert got.shape == (n, m)
    assert np.array_equal(got, want.astype(np.float32))


def test_rank_one_delta_is_the_rounded_outer_product(ref):
    """r = 1: fma(a, b, 0) is the correctly rounded product, i.e. numpy's fp32 multiplication."""
    rng = _rng(1)
    a = rng.standard_normal((31, 1)).astype(np.float32)
    b = rng.standard_normal((17, 1)).astype(np.float32)
    assert np.array_equal(ref.decompress(a, b), a * b.T)


def test_delta_is_close_to_the_fp64_product_and_uses_every_rank_term(ref):
    rng = _rng(2)
    n, m, r = 40, 70, 8
    P = rng.standard_normal((n, r)).astype(np.float32)
    Q = rng.standard_normal((m, r)).astype(np.float32)
    exact = P.astype(np.float64) @ Q.astype(np.float64).T
    got = ref.decompress(P, Q)
    bound = r * 2.0 ** -24 * (np.abs(P).astype(np.float64) @ np.abs(Q).astype(np.float64).T)   # r roundings of the chain
    assert np.all(np.abs(got - exact) <= bound + 1e-30)
    # dropping the last rank term would be far outside that bound
    short = P[:, :-1].astype(np.float64) @ Q[:, :-1].astype(np.float64).T
    assert np.max(np.abs(got - short)) > 100 * bound.max()


def test_update_subtracts_delta_with_one_rounding(ref):
    rng = _rng(3)
    n, m, r = 12, 33, 4
    x = rng.standard_normal((n, m)).astype(np.float32)
    P = rng.standard_normal((n, r)).astype(np.float32)
    Q = rng.standard_normal((m, r)).astype(np.float32)
    delta = ref.decompress(P, Q)
    got = ref.apply_update(x, P, Q)
    assert np.array_equal(got, x - delta)                         # fp32 subtraction, same Delta
    assert not np.array_equal(got, x + delta)
    # x = Delta is sent to exactly zero
    assert np.array_equal(ref.apply_update(delta, P, Q), np.zeros_like(delta))


def test_p_is_delta_plus_residual(ref):
    """Algorithm 2 line 9 takes p - Delta; the Delta that is applied to the parameters is the same
    one: entry by entry, residual = fl(p - Delta)."""
    rng = _rng(4)
    n, m, r = 25, 64, 3
    p = rng.standard_normal((n, m)).astype(np.float32)
    Q0 = rng.standard_normal((m, r)).astype(np.float32)
    Ph = ref.orthonormalise(ref.lowrank_P(p, Q0))
    Qn = ref.lowrank_Q(p, Ph)
    assert np.array_equal(ref.residual(p, Ph, Qn), p - ref.decompress(Ph, Qn))


def test_exact_rank_r_input_is_removed_by_its_own_update(ref):
    """A matrix of rank <= r is reproduced by one step of the compressor (exact-recovery property of
    subspace iteration), so x = p leaves x - Delta at rounding level."""
    rng = _rng(5)
    n, m, r = 48, 96, 4
    p = (rng.standard_normal((n, r)) @ rng.standard_normal((r, m))).astype(np.float32)
    Q0 = rng.standard_normal((m, r)).astype(np.float32)
    Ph = ref.orthonormalise(ref.lowrank_P(p, Q0))
    Qn = ref.lowrank_Q(p, Ph)
    left = ref.apply_update(p, Ph, Qn)
    assert np.max(np.abs(left)) <= 1e-5 * np.abs(p).max()
