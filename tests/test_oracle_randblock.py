"""Pins of the random-block oracle (oracle/randblock_ref.c) against what Section 5.3 and Algorithms 2 / 4 fix:

  * the block start is the stated function of the pinned Philox, lies in [0, N - k], is uniform over
    that range (chi-square over steps) and differs between matrices;
  * Delta is p = g + (1 - beta) e on the block and nothing else is sent;
  * beta = 0: the new error is exactly zero on the block ("the error has zeros there") and, with an error
    compressor that is exact on the data (8-bit codes of small integers with block maximum 127; a
    collision-free sketch), g + e_t = Delta + e_{t+1} entry by entry (Algorithm 2 lines 5, 6, 9 added up);
  * beta > 0: inside the block the quantiser's argument is beta * e, outside g + e: every decoded entry lies
    within one quantisation step of it; the sketch keeps beta S plus the sketch of p outside the block.
"""
import numpy as np
import pytest

from oracle import conef_ref as R


def test_block_start_is_the_stated_function_of_the_generator_and_in_range():
    seed, N, k = 0xFEEDFACE12345678, 1000, 100
    for mat in (0, 3):
        for step in (0, 1, 2 ** 40 + 5):
            out = R.philox4x32_10([mat, 0xFFFFFFFF, step & 0xFFFFFFFF, step >> 32], [seed & 0xFFFFFFFF, seed >> 32])
            r = int(out[0]) | (int(out[1]) << 32)
            assert R.rb_start(seed, mat, step, N, k) == (r * (N - k + 1)) >> 64
    assert R.rb_start(1, 0, 0, 50, 50) == 0                       # k = N: the whole matrix
    big = [R.rb_start(9, 1, t, 2 ** 34, 2 ** 20) for t in range(200)]
    assert 0 <= min(big) and max(big) <= 2 ** 34 - 2 ** 20 and max(big) > 2 ** 33     # more than 32 bits are used


def test_block_start_is_uniform():
    N, k, steps = 64 + 15, 16, 64000           # 64 possible starts
    starts = np.array([R.rb_start(77, 2, t, N, k) for t in range(steps)])
    counts = np.bincount(starts, minlength=N - k + 1)
    assert counts.size == N - k + 1
    chi2 = float(((counts - steps / 64) ** 2 / (steps / 64)).sum())
    assert chi2 < 63 + 6 * np.sqrt(2 * 63)
    other = np.array([R.rb_start(77, 3, t, N, k) for t in range(2000)])
    assert (other == starts[:2000]).mean() < 0.06


def test_quantiser_exact_data_conserves_the_gradient():
    """8-bit codes, every block holding an entry of magnitude 127 and integers otherwise: the quantiser is exact,
    so the decoded error is the dense error feedback recursion e+ = g + e - Delta (entries of size ~100 to 1e-4)."""
    rng = np.random.default_rng(1)
    N, k, bits, block = 640, 64, 8, 64
    codes, scales = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
    e = np.zeros(N)
    for t in range(5):
        start = R.rb_start(5, 0, t, N, k)
        # choose g so that g + e is an integer vector with max 127 in every block outside the kept block
        target = rng.integers(-100, 101, N).astype(np.float64)
        target[::block] = 127.0
        inside = np.zeros(N, bool)
        inside[start:start + k] = True
        g = (target - e).astype(np.float32)
        delta = R.rb_step_matrix(g.reshape(1, N), codes, scales, k, bits, block, 0.0, 5, 0, t)
        p = g.astype(np.float64) + e
        assert np.abs(delta.astype(np.float64) - p[start:start + k]).max() < 1e-4
        e_new = R.decode(codes, scales, N, bits, block).astype(np.float64)
        assert np.all(e_new[inside] == 0.0)
        # blocks the kept block cuts through lose their 127: restrict the exactness claim to untouched blocks
        blk = np.arange(N) // block
        touched = np.unique(blk[inside])
        clean = ~np.isin(blk, touched)
        assert np.abs(e_new[clean] - p[clean]).max() < 1e-4      # the decoded step 127 * fl32(1/127) is 1 up to 1e-7
        e = e_new


@pytest.mark.parametrize("beta", [0.0, 0.75])
def test_quantiser_argument_inside_and_outside_the_block(beta):
    rng = np.random.default_rng(2)
    N, k, bits, block = 4096, 512, 8, 128
    codes, scales = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
    for t in range(4):
        g = (rng.standard_normal(N) * 0.1).astype(np.float32)
        e = R.decode(codes, scales, N, bits, block).astype(np.float64)
        start = R.rb_start(8, 1, t, N, k)
        delta = R.rb_step_matrix(g.reshape(1, N), codes, scales, k, bits, block, beta, 8, 1, t)
        p = g.astype(np.float64) + (1.0 - beta) * e
        assert np.abs(delta - p[start:start + k]).max() < 1e-7
        x = g.astype(np.float64) + e
        x[start:start + k] = beta * e[start:start + k]
        e_new = R.decode(codes, scales, N, bits, block).astype(np.float64)
        step = np.repeat(scales.astype(np.float64) / R.levels(bits), block)[:N]
        assert np.all(np.abs(e_new - x) <= step * (1 + 1e-4) + 1e-7)
        if beta == 0.0:
            assert np.all(e_new[start:start + k] == 0.0)
        elif t > 1:
            assert np.abs(e_new[start:start + k]).max() > 0       # the kept-back share of the error stays


@pytest.mark.parametrize("beta", [0.0, 0.5])
def test_sketch_version_keeps_beta_s_plus_the_sketch_of_p_outside_the_block(beta):
    rng = np.random.default_rng(3)
    n, m, w, k = 30, 16, 7, 100
    b, s = R.cs_hash(21, 4, n, w)
    Pi = np.zeros((w, n))
    Pi[b, np.arange(n)] = s
    table = np.zeros((w, m), np.float32)
    S = np.zeros((w, m))
    for t in range(4):
        g = rng.integers(-20, 21, (n, m)).astype(np.float32)
        start = R.rb_start(21, 4, t, n * m, k)
        delta = R.cs_rb_step_matrix(g, table, k, beta, 21, 4, t)
        p = g.astype(np.float64) + (1.0 - beta) * (Pi.T @ S)
        flat = p.ravel().copy()
        assert np.abs(delta - flat[start:start + k]).max() < 1e-4
        flat[start:start + k] = 0.0
        S = beta * S + Pi @ flat.reshape(n, m)
        assert np.abs(table - S).max() < 1e-3 * max(1.0, np.abs(S).max())


def test_collision_free_sketch_conserves_the_gradient():
    rng = np.random.default_rng(4)
    n, m, w, k = 10, 12, 2048, 30
    seed = next(sd for sd in range(1, 10000) if np.unique(R.cs_hash(sd, 0, n, w)[0]).size == n)
    b, s = R.cs_hash(seed, 0, n, w)
    table = np.zeros((w, m), np.float32)
    for t in range(4):
        g = rng.integers(-50, 51, (n, m)).astype(np.float32)
        e = R.cs_decode(table, b, s, n).astype(np.float64)
        start = R.rb_start(seed, 0, t, n * m, k)
        delta = R.cs_rb_step_matrix(g, table, k, 0.0, seed, 0, t)
        full = np.zeros(n * m)
        full[start:start + k] = delta
        e_new = R.cs_decode(table, b, s, n).astype(np.float64)
        assert np.array_equal(g.astype(np.float64) + e, full.reshape(n, m) + e_new)       # integers: exact
