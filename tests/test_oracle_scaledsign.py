"""Pins of the scaled-sign oracle (oracle/randblock_ref.c, second part) against what Section 5.1 fixes:
Q(p) = ||p||_1 / d * sign(p) per matrix, inside Algorithm 2 / 4 with either error compressor.

  * the scale against numpy's l1 norm, the sign words against numpy's signbit (zero entries count as positive);
  * the compressor is the closed form: Delta = c * (+-1), so ||Delta||_1 = ||p||_1 and <Delta, p> = c ||p||_1,
    and it is contractive (Assumption 4): ||p - Delta||^2 = ||p||^2 - ||p||_1^2 / d < ||p||^2;
  * with an error compressor that is exact on the data (a collision-free sketch) the recursion is dense error
    feedback: g + e_t = Delta + e_{t+1};
  * quantiser: every decoded entry of the new state lies within one quantisation step of g + e - Delta;
  * sketch with collisions: the table is beta S + Pi (p - Delta) through the explicit sign matrix.
"""
import numpy as np
import pytest

from oracle import conef_ref as R


def unpack_signs(words, N):
    j = np.arange(N)
    return ((words[j // 32] >> (j % 32).astype(np.uint32)) & 1).astype(bool)


def test_scale_and_sign_words_against_numpy():
    rng = np.random.default_rng(1)
    N, bits, block = 1000, 8, 8
    g = (rng.standard_normal(N) * 0.3).astype(np.float32)
    g[5], g[6] = 0.0, -0.0
    codes, scales = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
    words, c = R.ss_step_matrix(g.reshape(1, N), codes, scales, bits, block, 0.0, 3, 0, 0)     # e = 0: p = g
    assert c == np.float32(np.abs(g.astype(np.float64)).sum() / N)
    neg = unpack_signs(words, N)
    want = np.signbit(g)
    want[6] = False                       # p = fma(0, 0, -0) = +0: a zero entry counts as positive whatever its sign in g
    assert np.array_equal(neg, want) and not neg[5]
    assert words.size == (N + 31) // 32 and (int(words[-1]) >> (N % 32)) == 0          # bits beyond N stay clear


def test_compressor_identities_and_contraction():
    rng = np.random.default_rng(2)
    N = 4096
    g = rng.standard_t(3.0, N).astype(np.float32)
    codes, scales = np.zeros(R.n_words(N, 8), np.uint32), np.zeros(R.n_blocks(N, 64), np.float32)
    words, c = R.ss_step_matrix(g.reshape(1, N), codes, scales, 8, 64, 0.0, 3, 0, 0)
    p = g.astype(np.float64)
    delta = np.where(unpack_signs(words, N), -float(c), float(c))
    l1 = np.abs(p).sum()
    assert abs(np.abs(delta).sum() - l1) < 1e-6 * l1
    assert abs(delta @ p - float(c) * l1) < 1e-6 * l1 * float(c)
    res = ((p - delta) ** 2).sum()
    assert abs(res - ((p ** 2).sum() - l1 ** 2 / N)) < 1e-5 * (p ** 2).sum()
    assert res < (p ** 2).sum()


@pytest.mark.parametrize("beta", [0.0, 0.75])
def test_quantiser_argument_is_g_plus_e_minus_delta(beta):
    rng = np.random.default_rng(3)
    N, bits, block = 4096, 8, 128
    codes, scales = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
    for t in range(4):
        g = (rng.standard_normal(N) * 0.1).astype(np.float32)
        e = R.decode(codes, scales, N, bits, block).astype(np.float64)
        words, c = R.ss_step_matrix(g.reshape(1, N), codes, scales, bits, block, beta, 8, 1, t)
        p = g.astype(np.float64) + (1.0 - beta) * e
        assert abs(float(c) - np.abs(p).mean()) < 1e-6 * np.abs(p).mean()
        near_zero = np.abs(p) < 1e-6
        assert np.array_equal(unpack_signs(words, N)[~near_zero], (p < 0)[~near_zero])
        delta = np.where(unpack_signs(words, N), -float(c), float(c))
        x = g.astype(np.float64) + e - delta
        e_new = R.decode(codes, scales, N, bits, block).astype(np.float64)
        step = np.repeat(scales.astype(np.float64) / R.levels(bits), block)[:N]
        assert np.all(np.abs(e_new - x) <= step * (1 + 1e-4) + 1e-7)


def test_collision_free_sketch_is_dense_error_feedback():
    rng = np.random.default_rng(4)
    n, m, w = 10, 12, 2048
    seed = next(sd for sd in range(1, 10000) if np.unique(R.cs_hash(sd, 0, n, w)[0]).size == n)
    b, s = R.cs_hash(seed, 0, n, w)
    table = np.zeros((w, m), np.float32)
    for t in range(4):
        g = (rng.standard_normal((n, m)) * 0.1).astype(np.float32)
        e = R.cs_decode(table, b, s, n).astype(np.float64)
        words, c = R.cs_ss_step_matrix(g, table, 0.0, seed, 0)
        delta = np.where(unpack_signs(words, n * m), -float(c), float(c)).reshape(n, m)
        e_new = R.cs_decode(table, b, s, n).astype(np.float64)
        assert np.abs(g.astype(np.float64) + e - delta - e_new).max() < 1e-6


def test_sketch_with_collisions_through_the_sign_matrix():
    rng = np.random.default_rng(5)
    n, m, w, beta = 30, 16, 7, 0.5
    b, s = R.cs_hash(21, 4, n, w)
    Pi = np.zeros((w, n))
    Pi[b, np.arange(n)] = s
    table = np.zeros((w, m), np.float32)
    S = np.zeros((w, m))
    for t in range(4):
        g = (rng.standard_normal((n, m)) * 0.1).astype(np.float32)
        words, c = R.cs_ss_step_matrix(g, table, beta, 21, 4)
        p = g.astype(np.float64) + (1.0 - beta) * (Pi.T @ S)
        assert abs(float(c) - np.abs(p).mean()) < 1e-5 * np.abs(p).mean()
        delta = np.where(unpack_signs(words, n * m), -float(c), float(c)).reshape(n, m)
        S = beta * S + Pi @ (p - delta)
        assert np.abs(table - S).max() < 2e-5 * max(1.0, np.abs(S).max())
