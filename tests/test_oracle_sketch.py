"""Pins of the count-sketch oracle (oracle/sketch_ref.c) against what Section 4.2.2, Proposition 2
and Algorithm 4 fix, and against library routines that are not the oracle's own:

  * the fp16 conversion against numpy's float16 cast (all 65536 patterns one way, many values the other);
  * the hash against the pinned Philox routine and the uniformity / balance a hash must have;
  * compress and decode against the explicit w x n sign matrix on integer data (exact arithmetic);
  * linearity C(e1 + e2) = C(e1) + C(e2) (Section 4.2.2);
  * unbiasedness and the closed-form variance (||e||^2 - e_p^2) / w of the estimate over seeds
    (Proposition 2; the classical count-sketch variance for v = 1);
  * a collision-free sketch: the estimate is exact, and the step is EFSGD (Algorithm 1) with the
    same compressor; with beta > 0 it is Algorithm 4 written out densely in numpy fp64;
  * conservation: g + e = Delta + e+ for every beta when nothing collides (Algorithm 4 lines 5, 9).
"""
import numpy as np
import pytest

from oracle import conef_ref as R


def sign_matrix(bucket, sign, w):
    Pi = np.zeros((w, bucket.size), np.float64)
    Pi[bucket, np.arange(bucket.size)] = sign
    return Pi


def collision_free_seed(n, w, mat=0):
    for seed in range(1, 100000):
        b, _ = R.cs_hash(seed, mat, n, w)
        if np.unique(b).size == n:
            return seed
    raise AssertionError("no collision-free seed found")


# ------------------------------------------------------------------ fp16
def test_f16_to_f32_matches_numpy_on_every_pattern():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = h.view(np.float16).astype(np.float32)
    got = np.array([R.f16_to_f32(int(v)) for v in h], np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f32_to_f16_matches_numpy_round_to_nearest_even():
    rng = np.random.default_rng(3)
    parts = [rng.standard_normal(20000).astype(np.float32) * np.float32(s)
             for s in (1.0, 1e-3, 1e-5, 3e-8, 100.0, 40000.0)]
    # exact halves between neighbouring fp16 values (ties), subnormal range included, and the overflow edge
    h = rng.integers(0, 0x7BFF, 4000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    ties = ((lo + hi) / 2).astype(np.float32)
    edge = np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e9, -1e9, np.inf, -np.inf, 2.0 ** -24, 2.0 ** -25,
                     2.0 ** -25 * 1.0001, 2.0 ** -14, 2.0 ** -14 * 0.9999], np.float32)
    x = np.concatenate(parts + [ties, -ties, edge])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([R.f32_to_f16(float(v)) for v in x], np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ hash
def test_hash_is_the_stated_function_of_the_pinned_generator():
    seed, mat, n, w = 0x123456789ABCDEF, 3, 50, 17
    b, s = R.cs_hash(seed, mat, n, w)
    for i in range(n):
        out = R.philox4x32_10([i, mat, 0xFFFFFFFF, 0xFFFFFFFF], [seed & 0xFFFFFFFF, seed >> 32])
        assert b[i] == (int(out[0]) * w) >> 32
        assert s[i] == (-1 if int(out[1]) & 1 else 1)


def test_hash_is_uniform_and_signs_are_balanced():
    n, w = 200000, 64
    b, s = R.cs_hash(11, 0, n, w)
    assert b.min() >= 0 and b.max() < w
    counts = np.bincount(b, minlength=w)
    chi2 = float(((counts - n / w) ** 2 / (n / w)).sum())
    assert chi2 < 63 + 6 * np.sqrt(2 * 63)            # chi-square with 63 degrees of freedom, ~6 sigma
    assert abs(int(s.sum())) < 6 * np.sqrt(n)
    # bucket and sign are independent of each other and differ between matrices and seeds
    assert abs(float(np.corrcoef(b, s)[0, 1])) < 0.02
    b2, s2 = R.cs_hash(11, 1, n, w)
    b3, _ = R.cs_hash(12, 0, n, w)
    assert (b2 == b).mean() < 0.03 and (b3 == b).mean() < 0.03 and abs(float((s2 * s.astype(np.int32)).mean())) < 0.02


# ------------------------------------------------------------------ compress / decode
@pytest.mark.parametrize("n,m,w", [(37, 11, 5), (64, 8, 64), (20, 3, 1)])
def test_compress_and_decode_are_the_sign_matrix_on_integers(n, m, w):
    rng = np.random.default_rng(n)
    x = rng.integers(-50, 51, (n, m)).astype(np.float32)
    b, s = R.cs_hash(7, 2, n, w)
    Pi = sign_matrix(b, s, w)
    table = rng.integers(-8, 9, (w, m)).astype(np.float32)
    old = table.astype(np.float64)
    R.cs_update(x, b, s, 0.5, table)                     # beta = 0.5: every value stays an exact binary fraction
    assert np.array_equal(table.astype(np.float64), 0.5 * old + Pi @ x.astype(np.float64))
    e = R.cs_decode(table, b, s, n)
    assert np.array_equal(e.astype(np.float64), Pi.T @ table.astype(np.float64))
    # the same through an fp16 table (integers and halves of this size are exact in fp16)
    t16 = old.astype(np.float16).view(np.uint16).copy()
    R.cs_update(x, b, s, 0.5, t16)
    assert np.array_equal(t16.view(np.float16).astype(np.float64), 0.5 * old + Pi @ x.astype(np.float64))
    assert np.array_equal(R.cs_decode(t16, b, s, n), e)


def test_sketch_is_linear():
    rng = np.random.default_rng(5)
    n, m, w = 50, 7, 9
    b, s = R.cs_hash(3, 0, n, w)
    x1 = rng.integers(-99, 100, (n, m)).astype(np.float32)
    x2 = rng.integers(-99, 100, (n, m)).astype(np.float32)
    t1, t2, t12 = (np.zeros((w, m), np.float32) for _ in range(3))
    R.cs_update(x1, b, s, 0.0, t1)
    R.cs_update(x2, b, s, 0.0, t2)
    R.cs_update(x1 + x2, b, s, 0.0, t12)
    assert np.array_equal(t12, t1 + t2)


def test_bucket_rows_are_added_in_ascending_row_order():
    # 1e8 + 1 - 1e8 in fp32 is 0 when added left to right and 1 in any order that pairs the large terms first
    n, m, w = 3, 1, 1
    b, s = np.zeros(n, np.int32), np.ones(n, np.int8)
    x = np.array([[1e8], [1.0], [-1e8]], np.float32)
    t = np.zeros((w, m), np.float32)
    R.cs_update(x, b, s, 0.0, t)
    assert t[0, 0] == 0.0
    x = np.array([[1e8], [-1e8], [1.0]], np.float32)
    t[:] = 0
    R.cs_update(x, b, s, 0.0, t)
    assert t[0, 0] == 1.0


def test_estimate_is_unbiased_with_the_closed_form_variance():
    """Proposition 2 for v = 1: E[estimate] = e and Var[estimate_p] = (||e||^2 - e_p^2) / w, taken over the
    hash (here: over seeds), column by column of the row sketch."""
    rng = np.random.default_rng(9)
    n, m, w, trials = 40, 3, 8, 4000
    e = rng.standard_normal((n, m)).astype(np.float32) * np.float32(2.0)
    tot, sq = np.zeros((n, m)), np.zeros((n, m))
    for seed in range(trials):
        b, s = R.cs_hash(1000 + seed, 0, n, w)
        t = np.zeros((w, m), np.float32)
        R.cs_update(e, b, s, 0.0, t)
        d = R.cs_decode(t, b, s, n).astype(np.float64) - e
        tot += d
        sq += d * d
    var = ((e.astype(np.float64) ** 2).sum(0, keepdims=True) - e.astype(np.float64) ** 2) / w
    assert np.all(np.abs(tot / trials) < 5 * np.sqrt(var / trials))                 # unbiased
    assert np.all(np.abs(sq / trials / var - 1.0) < 0.25)                            # variance (5 sigma ~ 0.2)


# ------------------------------------------------------------------ the step
def dense_partial_step(g, e, Q, beta):
    """Algorithm 4 with the identity as error compressor, in fp64 with numpy's QR."""
    p = g + (1.0 - beta) * e
    P = p @ Q
    Ph, Rr = np.linalg.qr(P)
    Ph = Ph * np.sign(np.diag(Rr))
    Qn = p.T @ Ph
    delta = Ph @ Qn.T
    return Ph, Qn, beta * e + p - delta, delta


@pytest.mark.parametrize("beta", [0.0, 0.5, 0.9])
def test_collision_free_sketch_gives_the_dense_partial_error_feedback_step(beta):
    rng = np.random.default_rng(21)
    n, m, r, w = 12, 40, 3, 4096
    seed = collision_free_seed(n, w)
    st = R.SketchState.fresh(n, m, w, False, rng.standard_normal((m, r)).astype(np.float32))
    b, s = R.cs_hash(seed, 0, n, w)
    e = np.zeros((n, m))
    Q = st.Q.astype(np.float64)
    for t in range(4):
        g = (rng.standard_normal((n, m)) * 0.1).astype(np.float32)
        e_before = R.cs_decode(st.table, b, s, n).astype(np.float64)
        Ph, Qn = R.cs_step_matrix(g, st, r, beta, seed, 0)
        Ph64, Qn64, e, delta = dense_partial_step(g.astype(np.float64), e, Q, beta)
        Q = Qn64
        assert np.abs(Ph - Ph64).max() < 2e-5
        assert np.abs(Qn - Qn64).max() < 2e-5 * max(1.0, np.abs(Qn64).max())
        e_after = R.cs_decode(st.table, b, s, n).astype(np.float64)
        assert np.abs(e_after - e).max() < 1e-5
        # conservation (Algorithm 4 lines 5 and 9 added up): g + e_t = Delta + e_{t+1}
        assert np.abs(g + e_before - R.decompress(Ph, Qn) - e_after).max() < 1e-6
    if beta == 0.0:
        # beta = 0 and no collisions: the oracle's own EFSGD step (Algorithm 1) from the same start
        rng = np.random.default_rng(21)
        Q0 = rng.standard_normal((m, r)).astype(np.float32)
        e32 = np.zeros((n, m), np.float32)
        st2 = R.SketchState.fresh(n, m, w, False, Q0)
        Qe = Q0
        for t in range(3):
            g = (rng.standard_normal((n, m)) * 0.1).astype(np.float32)
            Pa, Qa = R.cs_step_matrix(g, st2, r, 0.0, seed, 0)
            Pb, Qe = R.step_matrix_efsgd(g, e32, Qe)
            assert np.array_equal(Pa, Pb) and np.array_equal(Qa, Qe)
            assert np.array_equal(R.cs_decode(st2.table, b, s, n), e32)


def test_partial_step_with_collisions_follows_algorithm_4_through_the_sign_matrix():
    """With collisions the table must be beta * S + Pi (p - Delta) and p must use the decoded estimate."""
    rng = np.random.default_rng(33)
    n, m, r, w, beta = 30, 16, 2, 7, 0.75
    b, s = R.cs_hash(99, 4, n, w)
    Pi = sign_matrix(b, s, w)
    st = R.SketchState.fresh(n, m, w, False, rng.standard_normal((m, r)).astype(np.float32))
    S = np.zeros((w, m))
    for t in range(3):
        g = (rng.standard_normal((n, m)) * 0.1).astype(np.float32)
        Q = st.Q.astype(np.float64)
        Ph, Qn = R.cs_step_matrix(g, st, r, beta, 99, 4)
        p = g + (1.0 - beta) * (Pi.T @ S)
        P = p @ Q
        Ph64, Rr = np.linalg.qr(P)
        Ph64 = Ph64 * np.sign(np.diag(Rr))
        Qn64 = p.T @ Ph64
        S = beta * S + Pi @ (p - Ph64 @ Qn64.T)
        assert np.abs(Ph - Ph64).max() < 2e-5 and np.abs(Qn - Qn64).max() < 2e-5 * max(1.0, np.abs(Qn64).max())
        assert np.abs(st.table - S).max() < 1e-5


def test_fp16_table_step_rounds_the_fp32_step_once():
    rng = np.random.default_rng(8)
    n, m, r, w, beta = 25, 24, 2, 6, 0.9
    Q0 = rng.standard_normal((m, r)).astype(np.float32)
    g = (rng.standard_normal((n, m)) * 0.1).astype(np.float32)
    a = R.SketchState.fresh(n, m, w, False, Q0)
    h = R.SketchState.fresh(n, m, w, True, Q0)
    R.cs_step_matrix(g, a, r, beta, 5, 0)
    R.cs_step_matrix(g, h, r, beta, 5, 0)
    # from the zero table both runs see the same p, so the fp16 table is the fp32 table rounded once
    assert np.array_equal(h.table, a.table.astype(np.float16).view(np.uint16))
    # bf16 gradients are widened exactly
    gb = (g.view(np.uint32) >> 16).astype(np.uint16)
    gw = (gb.astype(np.uint32) << 16).view(np.float32)
    c = R.SketchState.fresh(n, m, w, False, Q0)
    d = R.SketchState.fresh(n, m, w, False, Q0)
    Pc, Qc = R.cs_step_matrix(gb, c, r, beta, 5, 0)
    Pd, Qd = R.cs_step_matrix(gw, d, r, beta, 5, 0)
    assert np.array_equal(Pc, Pd) and np.array_equal(Qc, Qd) and np.array_equal(c.table, d.table)
