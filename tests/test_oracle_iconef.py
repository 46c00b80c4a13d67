"""Pins of the iConEF-v1 oracle (oracle/iconef_ref.c) against what Algorithm 3 (Section 3.2) fixes:

  * from zero state the first compressed vector and Delta are those of the plain ConEF step (pinned elsewhere):
    Algorithm 3 with q = 0 accumulates and compresses as Algorithm 2 does;
  * the accumulation adds BOTH stored vectors: with known codes and scales in each, the kept values are
    g + d1 q1 + d2 q2 to fp32 rounding, both terms large;
  * p - Delta = e~+ + q+ + r, entry by entry, with |r| at most one step of the second quantiser, and the second
    quantiser's block maximum is at most one step of the first: the stored pair is about s times closer to
    p - Delta than the first vector alone (the reason for the second buffer);
  * data the first quantiser holds exactly leaves the second vector empty;
  * the second vector is the (pinned) quantiser applied to x - decode(e~+), drawing the random numbers of matrix
    word l + 2^31: recomputed here from the first vector with the quantiser called directly;
  * both quantisations are unbiased: the mean of e~+ + q+ over seeds approaches p - Delta;
  * scaled sign: c and the sign words are those of numpy on p = g + e~ + q; the argument is p - c sign(p).
"""
import numpy as np
import pytest

from oracle import conef_ref as R


def fresh(N, bits, block):
    return (np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32),
            np.zeros(R.n_words(N, bits), np.uint32), np.zeros(R.n_blocks(N, block), np.float32))


@pytest.mark.parametrize("bits,block", [(4, 64), (8, 128), (2, 32)])
def test_first_step_from_zero_state_is_the_plain_step(bits, block):
    rng = np.random.default_rng(2)
    N, k, seed = 1000, 90, 77
    g = rng.standard_normal((1, N)).astype(np.float32)
    c1, s1, c2, s2 = fresh(N, bits, block)
    pc, ps = np.zeros_like(c1), np.zeros_like(s1)
    d_i = R.i_rb_step_matrix(g, c1, s1, c2, s2, k, bits, block, seed, 3, 11)
    d_p = R.rb_step_matrix(g, pc, ps, k, bits, block, 0.0, seed, 3, 11)
    assert np.array_equal(d_i, d_p) and np.array_equal(c1, pc) and np.array_equal(s1, ps)
    assert s2.max() > 0 and np.any(c2 != 0)                      # and something is left for the second vector
    c1, s1, c2, s2 = fresh(N, bits, block)
    pc, ps = np.zeros_like(c1), np.zeros_like(s1)
    w_i, c_i = R.i_ss_step_matrix(g, c1, s1, c2, s2, bits, block, seed, 3, 11)
    w_p, c_p = R.ss_step_matrix(g, pc, ps, bits, block, 0.0, seed, 3, 11)
    assert c_i == c_p and np.array_equal(w_i, w_p) and np.array_equal(c1, pc) and np.array_equal(s1, ps)


def put_codes(q, bits):
    """Packs signed integer codes (two's complement fields, first element in the low bits)."""
    W = 32 // bits
    f = (q.astype(np.int64) & ((1 << bits) - 1)).reshape(-1, W)
    return (f << (bits * np.arange(W))).sum(axis=1).astype(np.uint32)


def test_accumulation_adds_both_vectors_exactly_on_dyadic_data():
    """Known codes in both vectors, step sizes near 2 and 0.25 (the step is scale * fl32(1/s), taken from that
    product): the expected p is g + d1 q1 + d2 q2 in fp64."""
    rng = np.random.default_rng(3)
    N, bits, block = 512, 8, 64
    s = R.levels(bits)
    q1 = rng.integers(-s, s + 1, N)
    q2 = rng.integers(-s, s + 1, N)
    c1, c2 = put_codes(q1, bits), put_codes(q2, bits)
    assert np.array_equal(R.unpack_codes(c1, N, bits), q1)
    s1 = np.full(N // block, 2.0 * s, np.float32)
    s2 = np.full(N // block, 0.25 * s, np.float32)
    d1 = float(np.float32(s1[0]) * np.float32(1.0 / s))
    d2 = float(np.float32(s2[0]) * np.float32(1.0 / s))
    g = rng.integers(-50, 51, N).astype(np.float32).reshape(1, N)
    p = R.i_form_p(g, c1, s1, c2, s2, bits, block).astype(np.float64)
    want = g.ravel().astype(np.float64) + d1 * q1 + d2 * q2
    assert np.abs(p - want).max() <= 2 ** -20 * np.abs(want).max()          # two fp32 roundings
    assert np.abs(d1 * q1).max() > 100 and np.abs(d2 * q2).max() > 10        # both terms matter
    # and the kept block carries exactly these values
    k = 100
    delta = R.i_rb_step_matrix(g, c1.copy(), s1.copy(), c2.copy(), s2.copy(), k, bits, block, 5, 0, 0)
    start = R.rb_start(5, 0, 0, N, k)
    assert np.array_equal(delta, p[start:start + k].astype(np.float32))


@pytest.mark.parametrize("bits,block", [(4, 128), (8, 64)])
def test_pair_is_within_one_second_level_step_of_the_argument(bits, block):
    rng = np.random.default_rng(4)
    N, k, seed = 128 * 9 + 40, 200, 99
    s = R.levels(bits)
    c1, s1, c2, s2 = fresh(N, bits, block)
    for t in range(4):
        g = (rng.standard_normal((1, N)) * 10.0 ** rng.integers(-3, 2)).astype(np.float32)
        p = R.i_form_p(g, c1, s1, c2, s2, bits, block).astype(np.float64)
        start = R.rb_start(seed, 1, t, N, k)
        delta = R.i_rb_step_matrix(g, c1, s1, c2, s2, k, bits, block, seed, 1, t)
        assert np.array_equal(delta, p[start:start + k].astype(np.float32))
        x = p.copy()
        x[start:start + k] = 0.0
        e1 = R.decode(c1, s1, N, bits, block).astype(np.float64)
        e2 = R.decode(c2, s2, N, bits, block).astype(np.float64)
        blk = np.arange(N) // block
        step1 = (s1.astype(np.float64) / s)[blk]
        step2 = (s2.astype(np.float64) / s)[blk]
        assert np.all(np.abs(x - e1) <= step1 * (1 + 1e-6))                     # first quantiser: one step
        assert np.all(s2.astype(np.float64)[blk] <= step1 * (1 + 1e-6))         # so the second block maximum is at most that
        r = x - e1 - e2
        assert np.all(np.abs(r) <= step2 * (1 + 1e-5) + 1e-7 * np.abs(x))       # pair: one second-level step
        # the point of the second buffer: the stored pair is far closer than the first vector alone
        assert np.linalg.norm(r) < np.linalg.norm(x - e1) * (3.0 / s)
        assert np.all(e1[start:start + k] == 0) and np.all(e2[start:start + k] == 0)


def test_exactly_held_data_leaves_the_second_vector_empty():
    rng = np.random.default_rng(5)
    N, k, bits, block = 640, 64, 8, 64
    c1, s1, c2, s2 = fresh(N, bits, block)
    x = rng.integers(-100, 101, N).astype(np.float32)
    x[::block] = 127.0
    R.i_rb_step_matrix(x.reshape(1, N), c1, s1, c2, s2, k, bits, block, 5, 0, 0)
    start = R.rb_start(5, 0, 0, N, k)
    want = x.copy()
    want[start:start + k] = 0
    # a block that lost its 127 to the kept range need not be exact; compare the others
    blocks = [b for b in range(N // block) if (b + 1) * block <= start or b * block >= start + k]
    assert len(blocks) >= N // block - 2
    e1 = R.decode(c1, s1, N, bits, block)
    for b in blocks:
        sl = slice(b * block, (b + 1) * block)
        assert np.abs(e1[sl] - want[sl]).max() <= 1e-4
        # what is left is rounding of the decode (127 * fl32(1/127) is not 1): at most a few 1e-6
        assert s2[b] <= 2e-5


def test_second_vector_is_the_quantiser_applied_to_the_first_rounding_error_with_its_own_draws():
    rng = np.random.default_rng(6)
    N, bits, block, seed, mat, step = 777, 4, 32, 0xABCDEF0123, 6, 2 ** 33 + 1
    g = rng.standard_normal((1, N)).astype(np.float32)
    c1, s1, c2, s2 = fresh(N, bits, block)
    _, c = R.i_ss_step_matrix(g, c1, s1, c2, s2, bits, block, seed, mat, step)
    p = g.ravel()                                                             # zero state: p = g
    x = (p - np.where(np.signbit(p), -c, c).astype(np.float32)).astype(np.float32)
    e1 = R.decode(c1, s1, N, bits, block)
    y = (x - e1).astype(np.float32)
    k2, sc2 = R.quantise(y, bits, block, seed, mat | 0x80000000, step)
    assert np.array_equal(k2, c2) and np.array_equal(sc2, s2)
    # with the first quantiser's draws it would have come out differently
    k_same, _ = R.quantise(y, bits, block, seed, mat, step)
    assert not np.array_equal(k_same, c2)
    # planted mistakes: the second quantiser fed x, or x + e1, instead of x - e1
    assert not np.array_equal(R.quantise(x, bits, block, seed, mat | 0x80000000, step)[1], s2)
    assert not np.array_equal(R.quantise((x + e1).astype(np.float32), bits, block, seed, mat | 0x80000000, step)[1], s2)


def test_pair_is_unbiased():
    rng = np.random.default_rng(7)
    N, bits, block, k = 256, 2, 64, 32
    g = rng.standard_normal((1, N)).astype(np.float32)
    acc1, acc = np.zeros(N), np.zeros(N)
    seeds = 3000
    start = R.rb_start(0, 0, 0, N, k)
    for sd in range(seeds):
        c1, s1, c2, s2 = fresh(N, bits, block)
        # same block every time (the start depends on the seed): use the step's draw but rebuild x per seed
        R.i_rb_step_matrix(g, c1, s1, c2, s2, k, bits, block, sd, 0, 0)
        st = R.rb_start(sd, 0, 0, N, k)
        x = g.ravel().astype(np.float64).copy()
        x[st:st + k] = 0
        e1 = R.decode(c1, s1, N, bits, block).astype(np.float64)
        e2 = R.decode(c2, s2, N, bits, block).astype(np.float64)
        acc1 += e1 - x
        acc += e1 + e2 - x
    # 2-bit codes have one level: a single vector errs by up to the block maximum per draw; the mean must vanish
    sigma = np.abs(g).max() / np.sqrt(seeds)
    assert np.abs(acc1 / seeds).max() < 5 * sigma
    assert np.abs(acc / seeds).max() < 5 * sigma
    assert start >= 0


def test_scaled_sign_uses_the_sum_of_both_vectors():
    rng = np.random.default_rng(8)
    N, bits, block, seed = 1024 + 32, 4, 32, 42
    c1, s1, c2, s2 = fresh(N, bits, block)
    for t in range(3):
        g = rng.standard_normal((1, N)).astype(np.float32)
        p = R.i_form_p(g, c1, s1, c2, s2, bits, block)
        words, c = R.i_ss_step_matrix(g, c1, s1, c2, s2, bits, block, seed, 0, t)
        assert abs(float(c) - np.abs(p.astype(np.float64)).sum() / N) <= 1e-7 * float(c)
        bits_ = (words[np.arange(N) // 32] >> (np.arange(N) % 32).astype(np.uint32)) & 1
        assert np.array_equal(bits_.astype(bool), np.signbit(p))
        x = p.astype(np.float64) - np.where(np.signbit(p), -float(c), float(c))
        e = R.decode(c1, s1, N, bits, block).astype(np.float64) + R.decode(c2, s2, N, bits, block).astype(np.float64)
        step2 = (s2.astype(np.float64) / R.levels(bits))[np.arange(N) // block]
        assert np.all(np.abs(x - e) <= step2 * (1 + 1e-5) + 1e-6 * np.abs(x).max())
        if t > 0:
            assert np.any(c2 != 0)          # the second vector is live state that the next accumulation used


# ---------------------------------------------------------------- around the rank-r compressor
def test_rank_r_first_step_from_zero_state_is_the_plain_step():
    rng = np.random.default_rng(20)
    n, m, rank, bits, block, seed = 48, 96, 4, 4, 32, 55
    g = rng.standard_normal((n, m)).astype(np.float32)
    Q0 = rng.standard_normal((m, rank)).astype(np.float32)
    c1, s1, c2, s2 = fresh(n * m, bits, block)
    Ph, Qn = R.i_step_matrix(g, c1, s1, c2, s2, Q0, rank, bits, block, seed, 2, 9)
    st = R.MatState.fresh(n, m, bits, block, Q0)
    Ph0, Qn0 = R.step_matrix(g, st, rank, bits, block, seed, 2, 9)
    assert np.array_equal(Ph, Ph0) and np.array_equal(Qn, Qn0)
    assert np.array_equal(c1, st.codes) and np.array_equal(s1, st.scales)
    assert np.any(c2 != 0)


def test_rank_r_factors_come_from_the_sum_of_both_vectors_and_the_pair_holds_the_residual():
    rng = np.random.default_rng(21)
    n, m, rank, bits, block, seed = 40, 64, 2, 8, 64, 56
    s = R.levels(bits)
    c1, s1, c2, s2 = fresh(n * m, bits, block)
    Q = rng.standard_normal((m, rank)).astype(np.float32)
    for t in range(4):
        g = rng.standard_normal((n, m)).astype(np.float32)
        p = R.i_form_p(g, c1, s1, c2, s2, bits, block).astype(np.float64).reshape(n, m)
        e_first = R.decode(c1, s1, n * m, bits, block).astype(np.float64).reshape(n, m)
        Ph, Qn = R.i_step_matrix(g, c1, s1, c2, s2, Q, rank, bits, block, seed, 0, t)
        Ph64, Qn64 = Ph.astype(np.float64), Qn.astype(np.float64)
        # P^ is an orthonormal basis of the columns of p Q, and Q+ = p^T P^, with the p that holds BOTH vectors
        assert np.abs(Ph64.T @ Ph64 - np.eye(rank)).max() < 1e-5
        raw = p @ Q.astype(np.float64)
        assert np.abs(raw - Ph64 @ (Ph64.T @ raw)).max() < 1e-4 * np.abs(raw).max()
        assert np.abs(Qn64 - p.T @ Ph64).max() < 1e-5 * np.abs(Qn64).max()
        if t > 1:       # with the second vector left out of p, Q+ would be visibly different
            p_wrong = g.astype(np.float64) + e_first
            assert np.abs(Qn64 - p_wrong.T @ Ph64).max() > 1e-4 * np.abs(Qn64).max()
        x = (p - Ph64 @ Qn64.T).ravel()
        e = R.decode(c1, s1, n * m, bits, block).astype(np.float64) + R.decode(c2, s2, n * m, bits, block).astype(np.float64)
        step2 = (s2.astype(np.float64) / s)[np.arange(n * m) // block]
        assert np.all(np.abs(x - e) <= step2 * (1 + 1e-4) + 1e-5 * np.abs(x).max())
        Q = Qn


def test_rank_r_error_steps_are_the_pinned_ones_on_the_residual():
    rng = np.random.default_rng(22)
    n, m, rank, bits, block, seed = 33, 50, 3, 4, 25 * 4, 57
    g = rng.standard_normal((n, m)).astype(np.float32)
    Q = rng.standard_normal((m, rank)).astype(np.float32)
    c1, s1, c2, s2 = fresh(n * m, bits, block)
    R.i_step_matrix(g, c1, s1, c2, s2, Q, rank, bits, block, seed, 1, 0)           # some state in both vectors
    a = [v.copy() for v in (c1, s1, c2, s2)]
    g = rng.standard_normal((n, m)).astype(np.float32)
    p = R.i_form_p(g, *a, bits, block).reshape(n, m)
    Ph, Qn = R.i_step_matrix(g, c1, s1, c2, s2, Q, rank, bits, block, seed, 1, 1)
    x = R.residual(p, Ph, Qn)
    R.i_error(x, *a, bits, block, seed, 1, 1)
    for got, want in zip((c1, s1, c2, s2), a):
        assert np.array_equal(got, want)
