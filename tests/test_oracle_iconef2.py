"""Pins of the iConEF-v2 oracle (oracle/iconef2_ref.c) against what Algorithm 3 (Section 3.2, the branch
e~+ = Q(p - Delta)) fixes, with the unscaled random block of Section 5.3 as the first error compressor:

  * with nothing kept by the first error compressor (k_e = 0) the step is the plain ConEF step with the same gradient
    compressor (pinned elsewhere), bit for bit: Algorithm 3 with e~ = 0 throughout is Algorithm 2;
  * the block start is the stated function of the pinned Philox generator (recomputed here with Python integers),
    covers its range 0 .. N - k_e uniformly and is not the gradient compressor's block;
  * from zero state Delta is the plain step's, e~+ is g on its block outside Delta's block and 0 inside it, and q+
    is the (pinned) quantiser applied to g with both kept sets zeroed;
  * p = Delta + e~+ + q+ + r entry by entry with r = 0 on both kept sets and |r| at most one step of the block's
    quantiser elsewhere, from a non-zero state too, where p = g + e~ + q is recomputed from the stored state with
    numpy;
  * over several steps the sum of all Delta plus the last e~ + q equals the sum of all gradients up to the summed
    quantiser steps: this fails, by far, if e~ is added back at any block but the one it was taken from, or with
    the wrong sign, or not at all;
  * the kept block is a contraction: E||x - Q(x)||^2 = sum_j (1 - pi_j) x_j^2 with pi_j the inclusion probability
    of coordinate j under a uniformly drawn start (closed form), checked on average over steps.
"""
import numpy as np
import pytest

from oracle import conef_ref as R


def fresh(N, bits, block, ke):
    return np.zeros(ke, np.float32), np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)


def dense(N, idx, vals):
    out = np.zeros(N, np.float64)
    out[idx] = vals
    return out


@pytest.mark.parametrize("bits,block", [(4, 64), (8, 128), (2, 32)])
def test_nothing_kept_by_the_first_error_compressor_is_the_plain_step(bits, block):
    rng = np.random.default_rng(12)
    N, k, G, seed = 1000, 90, 10, 31
    e0, c, s = fresh(N, bits, block, 0)
    pc, ps = c.copy(), s.copy()
    c2, s2, pc2, ps2 = c.copy(), s.copy(), c.copy(), s.copy()
    for t in range(3):
        g = rng.standard_normal((1, N)).astype(np.float32)
        assert np.array_equal(R.i2_rb_step_matrix(g, e0, c, s, k, bits, block, seed, 2, t),
                              R.rb_step_matrix(g, pc, ps, k, bits, block, 0.0, seed, 2, t))
        assert np.array_equal(c, pc) and np.array_equal(s, ps)
        assert np.array_equal(R.i2_rk_step_matrix(g, e0, c2, s2, G, bits, block, seed, 2, t),
                              R.rk_step_matrix(g, pc2, ps2, G, bits, block, 0.0, seed, 2, t))
        assert np.array_equal(c2, pc2) and np.array_equal(s2, ps2)
    assert np.any(c != 0)


def test_block_start_is_the_stated_function_of_the_generator():
    seed = 0x1234_5678_9ABC_DEF0
    key = np.array([seed & 0xFFFFFFFF, seed >> 32], np.uint32)
    for mat, step, N, ke in [(0, 0, 1000, 50), (7, 3, 12345, 1), (5, (1 << 40) + 9, 4096, 4096), (1, (1 << 64) - 1, 300, 299)]:
        out = R.philox4x32_10(np.array([mat, 0xFFFFFFFE, step & 0xFFFFFFFF, step >> 32], np.uint32), key)
        r = int(out[0]) | (int(out[1]) << 32)
        assert R.i2_start(seed, mat, step, N, ke) == (r * (N - ke + 1)) >> 64
    # step - 1 at step 0 wraps
    assert R.i2_start(seed, 1, -1, 300, 299) == R.i2_start(seed, 1, (1 << 64) - 1, 300, 299)


def test_block_start_is_uniform_and_not_the_gradient_compressors():
    N, ke, seed, T = 1000, 100, 5, 9010
    starts = np.array([R.i2_start(seed, 0, t, N, ke) for t in range(T)])
    assert starts.min() >= 0 and starts.max() <= N - ke
    counts = np.bincount(starts * 17 // (N - ke + 1), minlength=17).astype(np.float64)
    expect = np.bincount(np.arange(N - ke + 1) * 17 // (N - ke + 1), minlength=17) * (T / (N - ke + 1))
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 40.8                                  # 99.9 % point of chi-square with 16 degrees of freedom
    grad_starts = np.array([R.rb_start(seed, 0, t, N, ke) for t in range(T)])
    assert np.mean(starts == grad_starts) < 0.01
    assert abs(np.corrcoef(starts, grad_starts)[0, 1]) < 0.05
    # other matrices and seeds draw other blocks
    assert np.mean(starts[:500] == np.array([R.i2_start(seed, 1, t, N, ke) for t in range(500)])) < 0.02


@pytest.mark.parametrize("compressor", ["block", "strata"])
def test_first_step_from_zero_state(compressor):
    rng = np.random.default_rng(3)
    N, k, G, ke, bits, block, seed, mat, step = 960, 96, 10, 48, 4, 64, 77, 3, 11
    g = rng.standard_normal((1, N)).astype(np.float32)
    e, c, s = fresh(N, bits, block, ke)
    pc, ps = c.copy(), s.copy()
    if compressor == "block":
        d = R.i2_rb_step_matrix(g, e, c, s, k, bits, block, seed, mat, step)
        d_plain = R.rb_step_matrix(g, pc, ps, k, bits, block, 0.0, seed, mat, step)
        kept = np.arange(R.rb_start(seed, mat, step, N, k), R.rb_start(seed, mat, step, N, k) + k)
    else:
        d = R.i2_rk_step_matrix(g, e, c, s, G, bits, block, seed, mat, step)
        d_plain = R.rk_step_matrix(g, pc, ps, G, bits, block, 0.0, seed, mat, step)
        kept = R.rk_indices(seed, mat, step, N, G)
    assert np.array_equal(d, d_plain) and np.array_equal(d, g.ravel()[kept])
    s2 = R.i2_start(seed, mat, step, N, ke)
    x = g.ravel().copy()
    x[kept] = 0.0
    assert np.array_equal(e, x[s2:s2 + ke])
    x[s2:s2 + ke] = 0.0
    wc, ws = R.quantise(x, bits, block, seed, mat, step)
    assert np.array_equal(c, wc) and np.array_equal(s, ws)
    assert not np.array_equal(c, pc)                    # the plain step's vector also holds what e~+ took


@pytest.mark.parametrize("compressor", ["block", "strata"])
@pytest.mark.parametrize("bits,block", [(4, 128), (8, 64)])
def test_what_is_kept_plus_what_is_stored_is_p(compressor, bits, block):
    rng = np.random.default_rng(8)
    N, k, G, ke, seed, mat = 1024, 100, 10, 60, 9, 1
    e, c, s = fresh(N, bits, block, ke)
    for t in range(4):
        g = rng.standard_normal((1, N)).astype(np.float32)
        # p from the stored state, with numpy
        p = R.form_p(g, c, s, bits, block).ravel().copy()
        prev = R.i2_start(seed, mat, t - 1, N, ke)
        p[prev:prev + ke] = p[prev:prev + ke] + e
        if compressor == "block":
            d = R.i2_rb_step_matrix(g, e, c, s, k, bits, block, seed, mat, t)
            kept = np.arange(R.rb_start(seed, mat, t, N, k), R.rb_start(seed, mat, t, N, k) + k)
        else:
            d = R.i2_rk_step_matrix(g, e, c, s, G, bits, block, seed, mat, t)
            kept = R.rk_indices(seed, mat, t, N, G)
        assert np.array_equal(d, p[kept])
        s2 = R.i2_start(seed, mat, t, N, ke)
        mine = np.setdiff1d(np.arange(s2, s2 + ke), kept)
        e_dense = np.zeros(N, np.float32)
        e_dense[s2:s2 + ke] = e
        assert np.array_equal(e_dense[mine], p[mine]) and np.all(e_dense[np.intersect1d(np.arange(s2, s2 + ke), kept)] == 0)
        q = R.decode(c, s, N, bits, block)
        r = p.astype(np.float64) - dense(N, kept, d) - e_dense - q
        assert np.all(r[kept] == 0) and np.all(r[s2:s2 + ke] == 0)
        step_of = np.repeat(s.astype(np.float64) / R.levels(bits), block)[:N]
        assert np.all(np.abs(r) <= step_of * (1 + 1e-6))
        assert np.abs(r).max() > 0
    assert np.any(e != 0)


def test_nothing_is_lost_over_several_steps():
    rng = np.random.default_rng(21)
    N, k, ke, bits, block, seed, mat, T = 2048, 200, 300, 8, 64, 4, 0, 12
    e, c, s = fresh(N, bits, block, ke)
    sum_g, sum_d, slack = np.zeros(N), np.zeros(N), np.zeros(N)
    for t in range(T):
        g = rng.standard_normal((1, N)).astype(np.float32)
        d = R.i2_rb_step_matrix(g, e, c, s, k, bits, block, seed, mat, t)
        start = R.rb_start(seed, mat, t, N, k)
        sum_g += g.ravel()
        sum_d[start:start + k] += d
        slack += np.repeat(s.astype(np.float64) / R.levels(bits), block)[:N]
    last = R.i2_start(seed, mat, T - 1, N, ke)
    held = R.decode(c, s, N, bits, block).astype(np.float64)
    held[last:last + ke] += e
    gap = np.abs(sum_g - sum_d - held)
    assert np.all(gap <= slack + 1e-4)                  # fp32 roundings of the accumulation on top of the quantiser's steps
    assert gap.max() < 0.5 and np.abs(e).max() > 1.0    # ... which is below one misplaced entry of e~:
    wrong = R.decode(c, s, N, bits, block).astype(np.float64)
    wrong[(last + 7) % (N - ke):(last + 7) % (N - ke) + ke] += e
    assert np.abs(sum_g - sum_d - wrong).max() > 1.0


def test_the_kept_block_contracts_by_its_inclusion_probabilities():
    rng = np.random.default_rng(30)
    N, ke, seed, T = 400, 80, 17, 6000
    x = rng.standard_normal(N)
    j = np.arange(N)
    # number of starts s in 0 .. N - ke with s <= j < s + ke
    pi = (np.minimum(j, N - ke) - np.maximum(j - ke + 1, 0) + 1) / (N - ke + 1)
    want = ((1 - pi) * x ** 2).sum()
    got = 0.0
    for t in range(T):
        s0 = R.i2_start(seed, 0, t, N, ke)
        got += (x ** 2).sum() - (x[s0:s0 + ke] ** 2).sum()
    assert abs(got / T - want) <= 0.02 * want
    assert want < (x ** 2).sum() * (1 - 0.5 * ke / N)   # a contraction (Assumption 4): delta < 1
