"""Pins of the column-form count-sketch oracle (oracle/sketch_col_ref.c; Section 5.3, "row or column"): sketching the
columns of a matrix is sketching the rows of its transpose, so every routine must give, bit for bit, what the row form
(pinned in test_oracle_sketch.py against the explicit sign matrix, Proposition 2 and dense error feedback) gives on the
transposed data; the step is then pinned by its parts, by the factors in numpy fp64 and by the conservation
g + e = Delta + e+ when no two columns share a bucket."""
import numpy as np
import pytest

from oracle import conef_ref as R


def _table(rng, n, w, fp16):
    t = (rng.standard_normal((n, w)) * 0.05).astype(np.float32)
    return t.astype(np.float16).view(np.uint16) if fp16 else t


def _t(a):
    return np.array(a.T, order="C", copy=True)


@pytest.mark.parametrize("fp16", [False, True])
@pytest.mark.parametrize("n,m,w", [(37, 53, 11), (8, 300, 300), (64, 5, 1)])
def test_every_routine_is_the_row_form_on_the_transpose(fp16, n, m, w):
    rng = np.random.default_rng([n, m, w, int(fp16)])
    seed, mat, beta = 991, 2, 0.75
    g = rng.standard_normal((n, m)).astype(np.float32)
    tab = _table(rng, n, w, fp16)
    b, s = R.cs_hash(seed, mat, m, w)                       # one hash per column
    # estimate
    e = R.csc_decode(tab, b, s, m)
    assert np.array_equal(e.view(np.uint32), _t(R.cs_decode(_t(tab), b, s, m)).view(np.uint32))
    # accumulation
    p = R.csc_form_p(g, tab, b, s, beta)
    assert np.array_equal(p.view(np.uint32), _t(R.cs_form_p(_t(g), _t(tab), b, s, beta)).view(np.uint32))
    # error step
    x = rng.standard_normal((n, m)).astype(np.float32)
    mine, theirs = tab.copy(), _t(tab)
    R.csc_update(x, b, s, beta, mine)
    R.cs_update(_t(x), b, s, beta, theirs)
    assert np.array_equal(mine, _t(theirs))
    assert not np.array_equal(mine, tab)


def test_step_is_its_parts_and_its_factors_are_those_of_p():
    rng = np.random.default_rng(5)
    n, m, w, r, beta, seed, mat = 40, 96, 20, 4, 0.5, 77, 1
    g = rng.standard_normal((n, m)).astype(np.float32)
    tab = _table(rng, n, w, False)
    Q0 = rng.standard_normal((m, r)).astype(np.float32)
    b, s = R.cs_hash(seed, mat, m, w)
    p = R.csc_form_p(g, tab, b, s, beta)
    new = tab.copy()
    Ph, Qn = R.csc_step_matrix(g, new, Q0, r, beta, seed, mat)
    # factors: numpy fp64 from the same p
    P64 = p.astype(np.float64) @ Q0.astype(np.float64)
    Qr, _ = np.linalg.qr(P64)
    assert np.abs(Ph.astype(np.float64).T @ Ph.astype(np.float64) - np.eye(r)).max() < 1e-5
    assert np.abs(Qr @ (Qr.T @ Ph.astype(np.float64)) - Ph).max() < 1e-5           # same column space
    assert np.abs(Qn - p.astype(np.float64).T @ Ph.astype(np.float64)).max() < 1e-4
    # error step: the pinned routine on p - Delta
    want = tab.copy()
    R.csc_update(R.residual(p, Ph, Qn), b, s, beta, want)
    assert np.array_equal(new, want)


def test_without_collisions_nothing_is_lost():
    """As many buckets as columns and a hash without collisions (found by search over seeds): the sketch is a signed
    permutation of the columns, so g + e = Delta + e+ up to fp32 rounding, with beta = 0."""
    n, m, r = 12, 6, 2
    seed = next(sd for sd in range(10000) if len(set(R.cs_hash(sd, 0, m, 4 * m)[0])) == m)
    w = 4 * m
    b, s = R.cs_hash(seed, 0, m, w)
    rng = np.random.default_rng(8)
    tab = np.zeros((n, w), np.float32)
    Q = rng.standard_normal((m, r)).astype(np.float32)
    for t in range(3):
        g = rng.standard_normal((n, m)).astype(np.float32)
        e = R.csc_decode(tab, b, s, m)
        Ph, Q = R.csc_step_matrix(g, tab, Q, r, 0.0, seed, 0)
        delta = Ph.astype(np.float64) @ Q.astype(np.float64).T
        e_new = R.csc_decode(tab, b, s, m)
        assert np.abs(g.astype(np.float64) + e - delta - e_new).max() < 1e-5
    assert np.abs(e_new).max() > 0.1
