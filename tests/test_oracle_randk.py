"""Pins of the random-k oracle (oracle/randk_ref.c; stratified reading of the compressor of the paper's iConEF
experiment) against what the construction and Algorithms 2 - 4 fix:

  * one kept coordinate per stratum, inside its stratum (short last stratum included), the stated function of the
    pinned Philox; k = ceil(N / G);
  * the kept coordinate is uniform within its stratum (chi-square over steps), differs between matrices and steps,
    and neighbouring strata (which share a Philox call) are uncorrelated;
  * Delta is p = g + (1 - beta) e there, and the average of ||p - Delta||^2 over steps is (1 - 1/G) ||p||^2
    (the contraction of Assumption 4 with delta = 1 - k/N, as for a uniformly drawn k-subset);
  * beta = 0 with an exact error compressor: g + e_t = Delta + e_{t+1} entry by entry; the new error is zero on
    the kept coordinates;
  * beta > 0: beta e stays on the kept coordinates; every decoded entry within one quantisation step of its argument;
  * count sketch: the table is beta S + the sketch of p off the kept coordinates;
  * iConEF-v1 around it: from zero state the plain step; the pair within one second-level step of p - Delta.
"""
import numpy as np
import pytest

from oracle import conef_ref as R


def test_one_kept_coordinate_per_stratum_the_stated_function_of_the_generator():
    seed = 0x1234567ABCDEF
    for N, G in ((35, 10), (1000, 10), (64, 1), (100, 100), (101, 100), (7, 50), (4096, 3)):
        for mat, step in ((0, 0), (5, 2 ** 40 + 3)):
            idx = R.rk_indices(seed, mat, step, N, G)
            k = -(-N // G)
            assert idx.size == k == R.rk_count(N, G)
            for i in (0, 1, k // 2, k - 1):
                if i >= k:
                    continue
                out = R.philox4x32_10([i >> 2, mat + 0x40000000, step & 0xFFFFFFFF, step >> 32],
                                      [seed & 0xFFFFFFFF, seed >> 32])
                ln = min(G, N - i * G)
                assert idx[i] == i * G + ((int(out[i & 3]) * ln) >> 32)
            lo = np.arange(k) * G
            assert np.all(idx >= lo) and np.all(idx < np.minimum(lo + G, N))
    assert np.array_equal(R.rk_indices(3, 0, 0, 64, 1), np.arange(64))          # G = 1: everything is kept


def test_kept_coordinate_is_uniform_within_its_stratum_and_strata_are_uncorrelated():
    N, G, steps = 16 * 9 + 5, 16, 8000
    draws = np.stack([R.rk_indices(77, 2, t, N, G) for t in range(steps)])       # steps x 10
    off = draws - np.arange(draws.shape[1]) * G
    for i in (0, 1, 4, 8):
        counts = np.bincount(off[:, i], minlength=G)
        chi2 = float(((counts - steps / G) ** 2 / (steps / G)).sum())
        assert chi2 < (G - 1) + 6 * np.sqrt(2 * (G - 1)), (i, chi2)
    counts = np.bincount(off[:, 9], minlength=5)                                  # the short last stratum: 5 coordinates
    assert counts.size == 5
    assert float(((counts - steps / 5) ** 2 / (steps / 5)).sum()) < 4 + 6 * np.sqrt(8)
    for a, b in ((0, 1), (1, 2), (3, 4), (4, 5)):                                 # same and different Philox calls
        c = np.corrcoef(off[:, a], off[:, b])[0, 1]
        assert abs(c) < 5 / np.sqrt(steps)
    other = np.stack([R.rk_indices(77, 3, t, N, G) for t in range(500)])
    assert (other == draws[:500]).mean() < 2.0 / G + 0.05


def test_delta_is_p_on_the_kept_coordinates_and_the_contraction_holds_on_average():
    rng = np.random.default_rng(1)
    N, G, bits, block = 2000, 10, 8, 100
    g = rng.standard_normal(N).astype(np.float32)
    ratios = []
    for t in range(400):
        codes, scales = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
        delta = R.rk_step_matrix(g.reshape(1, N), codes, scales, G, bits, block, 0.0, 9, 0, t)
        idx = R.rk_indices(9, 0, t, N, G)
        assert np.array_equal(delta, g[idx])                                      # zero state: p = g
        rest = g.astype(np.float64).copy()
        rest[idx] = 0
        ratios.append((rest ** 2).sum() / (g.astype(np.float64) ** 2).sum())
    assert abs(np.mean(ratios) - (1 - 1 / G)) < 0.005


def test_quantiser_exact_data_conserves_the_gradient():
    rng = np.random.default_rng(2)
    N, G, bits, block = 640, 8, 8, 64
    codes, scales = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
    e = np.zeros(N)
    for t in range(5):
        idx = R.rk_indices(5, 0, t, N, G)
        kept = np.zeros(N, bool)
        kept[idx] = True
        # g + e integer with two entries of magnitude 127 per block, at least one of which is not kept
        target = rng.integers(-100, 101, N).astype(np.float64)
        target[0::block] = 127.0
        target[1::block] = -127.0
        g = (target - e).astype(np.float32)
        delta = R.rk_step_matrix(g.reshape(1, N), codes, scales, G, bits, block, 0.0, 5, 0, t)
        p = g.astype(np.float64) + e
        assert np.abs(delta - p[idx]).max() < 1e-4
        e_new = R.decode(codes, scales, N, bits, block).astype(np.float64)
        assert np.all(e_new[kept] == 0.0)
        full = np.zeros(N)
        full[idx] = delta
        assert np.abs(p - full - e_new).max() < 1e-4          # g + e = Delta + e+
        e = e_new


@pytest.mark.parametrize("beta", [0.0, 0.75])
def test_quantiser_argument_on_and_off_the_kept_coordinates(beta):
    rng = np.random.default_rng(3)
    N, G, bits, block = 4096 + 50, 7, 8, 128
    codes, scales = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
    for t in range(4):
        g = (rng.standard_normal(N) * 0.1).astype(np.float32)
        e = R.decode(codes, scales, N, bits, block).astype(np.float64)
        idx = R.rk_indices(8, 1, t, N, G)
        delta = R.rk_step_matrix(g.reshape(1, N), codes, scales, G, bits, block, beta, 8, 1, t)
        p = g.astype(np.float64) + (1.0 - beta) * e
        assert np.abs(delta - p[idx]).max() < 1e-7
        x = g.astype(np.float64) + e
        x[idx] = beta * e[idx]
        e_new = R.decode(codes, scales, N, bits, block).astype(np.float64)
        step = np.repeat(scales.astype(np.float64) / R.levels(bits), block)[:N]
        assert np.all(np.abs(e_new - x) <= step * (1 + 1e-4) + 1e-7)
        if beta == 0.0:
            assert np.all(e_new[idx] == 0.0)
        elif t > 1:
            assert np.abs(e_new[idx]).max() > 0


@pytest.mark.parametrize("beta", [0.0, 0.5])
def test_sketch_version_keeps_beta_s_plus_the_sketch_of_p_off_the_kept_coordinates(beta):
    rng = np.random.default_rng(4)
    n, m, w, G = 30, 16, 7, 6
    b, s = R.cs_hash(21, 4, n, w)
    Pi = np.zeros((w, n))
    Pi[b, np.arange(n)] = s
    table = np.zeros((w, m), np.float32)
    S = np.zeros((w, m))
    for t in range(4):
        g = rng.integers(-20, 21, (n, m)).astype(np.float32)
        idx = R.rk_indices(21, 4, t, n * m, G)
        delta = R.cs_rk_step_matrix(g, table, G, beta, 21, 4, t)
        flat = (g.astype(np.float64) + (1.0 - beta) * (Pi.T @ S)).ravel()
        assert np.abs(delta - flat[idx]).max() < 1e-4
        flat[idx] = 0.0
        S = beta * S + Pi @ flat.reshape(n, m)
        assert np.abs(table - S).max() < 1e-3 * max(1.0, np.abs(S).max())


def test_iconef_around_it():
    rng = np.random.default_rng(5)
    N, G, bits, block, seed = 128 * 7 + 20, 10, 4, 64, 31
    s = R.levels(bits)
    c1, s1 = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
    c2, s2 = np.zeros_like(c1), np.zeros_like(s1)
    pc, ps = np.zeros_like(c1), np.zeros_like(s1)
    g = rng.standard_normal((1, N)).astype(np.float32)
    d_i = R.i_rk_step_matrix(g, c1, s1, c2, s2, G, bits, block, seed, 2, 0)
    d_p = R.rk_step_matrix(g, pc, ps, G, bits, block, 0.0, seed, 2, 0)
    assert np.array_equal(d_i, d_p) and np.array_equal(c1, pc) and np.array_equal(s1, ps)      # from zero state: the plain step
    for t in range(1, 4):
        g = rng.standard_normal((1, N)).astype(np.float32)
        p = R.i_form_p(g, c1, s1, c2, s2, bits, block).astype(np.float64)
        idx = R.rk_indices(seed, 2, t, N, G)
        delta = R.i_rk_step_matrix(g, c1, s1, c2, s2, G, bits, block, seed, 2, t)
        assert np.array_equal(delta, p[idx].astype(np.float32))
        x = p.copy()
        x[idx] = 0
        e = R.decode(c1, s1, N, bits, block).astype(np.float64) + R.decode(c2, s2, N, bits, block).astype(np.float64)
        step2 = (s2.astype(np.float64) / s)[np.arange(N) // block]
        assert np.all(np.abs(x - e) <= step2 * (1 + 1e-5) + 1e-7 * np.abs(x))
        assert np.all(e[idx] == 0)


# ---------------------------------------------------------------- the uniformly drawn k-subset (G < 0 in the oracle's routines)
def test_uniform_subset_is_a_bijection_with_its_inverse_and_exactly_k_kept():
    for N, k, seed, mat, step in [(37, 5, 1, 0, 0), (1000, 100, 9, 3, 7), (4097, 1, 2, 1, 2 ** 40 + 5), (64, 64, 3, 2, 1)]:
        images = [R.rku_perm(seed, mat, step, N, j) for j in range(N)]
        assert sorted(images) == list(range(N))
        assert all(R.rku_inverse(seed, mat, step, N, images[j]) == j for j in range(0, N, max(1, N // 97)))
        idx = R.rk_indices(seed, mat, step, N, -k)
        assert idx.size == k == R.rk_count(N, -k) and len(set(idx.tolist())) == k
        assert [images[int(j)] for j in idx] == list(range(k))          # slot i holds the coordinate that pi sends to i
    # another step, matrix or seed: another subset
    base = set(R.rk_indices(9, 3, 7, 1000, -100).tolist())
    for other in (R.rk_indices(9, 3, 8, 1000, -100), R.rk_indices(9, 4, 7, 1000, -100), R.rk_indices(10, 3, 7, 1000, -100)):
        assert len(base & set(other.tolist())) < 40


def test_uniform_subset_is_the_stated_function_of_the_generator():
    """pi recomputed here with Python integers from the pinned Philox: six alternating rounds on Z_a x Z_b."""
    def mix(u):
        u = (u * 0x9E3779B1) & 0xFFFFFFFF; u ^= u >> 15; u = (u * 0x85EBCA77) & 0xFFFFFFFF; u ^= u >> 13
        return u
    seed, mat, step, N = 0x1234_5678_9ABC_DEF0, 2, 2 ** 33 + 1, 5000
    key = np.array([seed & 0xFFFFFFFF, seed >> 32], np.uint32)
    o0 = R.philox4x32_10(np.array([mat, 0xFFFFFFFD, step & 0xFFFFFFFF, step >> 32], np.uint32), key)
    o1 = R.philox4x32_10(np.array([mat, 0xFFFFFFFC, step & 0xFFFFFFFF, step >> 32], np.uint32), key)
    keys = [int(o0[0]), int(o0[1]), int(o0[2]), int(o0[3]), int(o1[0]), int(o1[1])]
    a = 71                                             # ceil(sqrt(5000)): 70^2 = 4900 < 5000 <= 71^2
    b = -(-N // a)
    for j in (0, 1, 70, 71, 4999, 2500):
        x = j
        while True:
            L, Rr = divmod(x, b)
            for i in range(6):
                if i % 2 == 0:
                    L = (L + ((mix(Rr ^ keys[i]) * a) >> 32)) % a
                else:
                    Rr = (Rr + ((mix(L ^ keys[i]) * b) >> 32)) % b
            x = L * b + Rr
            if x < N:
                break
        assert R.rku_perm(seed, mat, step, N, j) == x


def test_uniform_subset_keeps_single_coordinates_and_pairs_at_the_uniform_rates():
    """Over many steps every coordinate is kept at the rate k / N and every pair, neighbours included, at
    k (k-1) / (N (N-1)): what distinguishes it from the stratified form, which never keeps two of one stratum."""
    N, k, T, seed = 37, 5, 40000, 77
    inc, pair = np.zeros(N), np.zeros((N, N))
    for t in range(T):
        kept = np.zeros(N)
        kept[R.rk_indices(seed, 0, t, N, -k)] = 1.0
        inc += kept
        pair += np.outer(kept, kept)
    p1, p2 = k / N, k * (k - 1) / (N * (N - 1))
    z1 = (inc / T - p1) / np.sqrt(p1 * (1 - p1) / T)
    assert np.abs(z1).max() < 4.5
    z2 = (pair / T - p2) / np.sqrt(p2 * (1 - p2) / T)
    np.fill_diagonal(z2, 0.0)
    assert np.abs(z2).max() < 5.0 and (z2 ** 2).sum() / (N * (N - 1)) < 1.25
    # the stratified form with the same rate fails this by far: neighbours of one stratum are never kept together
    G = 8
    pair_s = np.zeros((N, N))
    for t in range(4000):
        kept = np.zeros(N)
        kept[R.rk_indices(seed, 0, t, N, G)] = 1.0
        pair_s += np.outer(kept, kept)
    assert pair_s[0, 1] == 0


def test_uniform_subset_step_is_the_stratified_step_with_other_coordinates():
    """Delta = p on the kept coordinates (in slot order), the error compressor gets p - Delta with beta e kept on them:
    checked against the stated construction with the pinned quantiser, and the contraction on average."""
    rng = np.random.default_rng(3)
    N, k, bits, block, seed, mat = 1024, 100, 4, 64, 5, 1
    codes, scales = np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32)
    ratio = []
    for t in range(5):
        g = rng.standard_normal((1, N)).astype(np.float32)
        p = R.form_p(g, codes, scales, bits, block).ravel()
        e = R.decode(codes, scales, N, bits, block)
        idx = R.rk_indices(seed, mat, t, N, -k)
        d = R.rk_step_matrix(g, codes, scales, -k, bits, block, 0.0, seed, mat, t)
        assert np.array_equal(d, p[idx])
        x = p.copy()
        x[idx] = 0.0 * e[idx]
        wc, ws = R.quantise(x, bits, block, seed, mat, t)
        assert np.array_equal(codes, wc) and np.array_equal(scales, ws)
        ratio.append(((p ** 2).sum() - (d ** 2).sum()) / (p ** 2).sum())
    assert abs(np.mean(ratio) - (1 - k / N)) < 0.05
    # around it: the two-vector forms take the same subset
    c1, s1, c2, s2 = codes.copy(), scales.copy(), np.zeros_like(codes), np.zeros_like(scales)
    g = rng.standard_normal((1, N)).astype(np.float32)
    d = R.i_rk_step_matrix(g, c1, s1, c2, s2, -k, bits, block, seed, mat, 9)
    assert np.array_equal(d, R.form_p(g, codes, scales, bits, block).ravel()[R.rk_indices(seed, mat, 9, N, -k)])
