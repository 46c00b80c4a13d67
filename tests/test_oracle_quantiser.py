"""Pins for the oracle's error compressor: eq. (3) of Section 4.2.1 with the per-block
max-norm (Section 5.1), Assumption 3 (unbiased, relative variance theta), and the packed
two's-complement code format."""
import numpy as np
import pytest

BITS_BLOCK = [(8, 64), (4, 128), (2, 256)]


def _rand_x(rng, n, kind="normal"):
    if kind == "normal":
        return rng.standard_normal(n).astype(np.float32)
    if kind == "laplace":
        return rng.laplace(0, 1e-3, n).astype(np.float32)
    if kind == "t3":
        return (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    raise ValueError(kind)


def _frac_parts(x, a, s):
    """fp32 re-derivation of the 16.16 fixed-point value U = floor(|x| * (s/a) * 2^16):
    returns (l, f) = (U >> 16, (U mod 2^16) / 2^16), the level below and the up-probability."""
    inv16 = np.float32(np.float32(s) / np.float32(a)) * np.float32(65536.0)
    prod = (np.abs(x).astype(np.float32) * inv16).astype(np.float32)
    U = np.floor(prod.astype(np.float64)).astype(np.int64)
    return U >> 16, (U & 0xFFFF).astype(np.float64) / 65536.0


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_exact_expectation_by_enumerating_all_draws(ref, bits):
    """Every element sees all 65536 draws: the number of 'up' roundings must be exactly
    f * 2^16 with f the fraction of |x|/a*s truncated to 16 bits -- the probability rule of
    eq. (3) on the grid of the draw -- and the mean decoded value must equal x up to that
    2^-16 granularity."""
    W = 32 // bits
    B = W                                   # one word per block: smallest legal block
    s = ref.levels(bits)
    rng = np.random.default_rng(bits)
    x = rng.standard_normal(B).astype(np.float32)
    x[1] = 0.0
    x[2] = -x[2] if x[2] > 0 else x[2]       # make sure a negative value is present
    a = np.abs(x).max()
    reps = 65536
    big = np.tile(x, reps)
    draw = np.repeat(np.arange(reps, dtype=np.uint16), B)
    codes, scales = ref.quantise(big, bits, B, draw=draw)
    assert np.all(scales == a)
    q = ref.unpack_codes(codes[:0], 0, bits)   # smoke the empty case
    assert q.size == 0
    # decode every copy
    dec = ref.decode(codes, scales, big.size, bits, B).reshape(reps, B).astype(np.float64)
    l, f = _frac_parts(x, a, s)
    words = codes.reshape(reps, -1)
    fields = np.stack([(words[:, e // W] >> (bits * (e % W))) & ((1 << bits) - 1) for e in range(B)], 1)
    qs = np.where(fields >= (1 << (bits - 1)), fields.astype(np.int64) - (1 << bits), fields.astype(np.int64))
    mags = np.abs(qs)
    for e in range(B):
        ups = int((mags[:, e] == l[e] + 1).sum())
        downs = int((mags[:, e] == l[e]).sum())
        assert ups + downs == reps
        assert ups == int(round(f[e] * 65536.0))                  # P(up) = f, on the 2^-16 grid
        if x[e] != 0:
            assert np.all(np.sign(qs[mags[:, e] > 0, e]) == np.sign(x[e]))
    mean = dec.mean(0)
    step = float(a) / s
    assert np.all(np.abs(mean - x.astype(np.float64)) <= step * (2.0 ** -16) + 1e-6 * step)


@pytest.mark.parametrize("bits,block", BITS_BLOCK)
def test_grid_points_are_reproduced_exactly(ref, bits, block):
    """x already on the grid {a*q/s}: every draw returns q itself (f = 0 never rounds up)."""
    s = ref.levels(bits)
    rng = np.random.default_rng(7)
    for a in [np.float32(1.0), np.float32(0.37), np.float32(1e-3 * s), np.float32(3.1e4)]:
        q = rng.integers(-s, s + 1, block)
        q[0] = s                                      # the max-norm element
        x = (np.float32(a) * q.astype(np.float32) / np.float32(s)).astype(np.float32)
        # the grid is only exact when x/a*s rounds back to the integer; use a = s*2^k scaled values
        a2 = np.float32(s) * np.float32(2.0 ** -5)
        x2 = (q.astype(np.float32) * np.float32(2.0 ** -5)).astype(np.float32)
        for draw_val in [0, 1, 65535]:
            codes, scales = ref.quantise(x2, bits, block, draw=np.full(block, draw_val, np.uint16))
            assert scales[0] == a2
            assert np.array_equal(ref.unpack_codes(codes, block, bits), q)
            back = ref.decode(codes, scales, block, bits, block)
            assert np.allclose(back, x2, rtol=2e-7, atol=0)
        # general a: |x|/a*s lands within a few ulps of the integer, so a mid-range draw returns q
        codes, scales = ref.quantise(x, bits, block, draw=np.full(block, 32768, np.uint16))
        assert np.array_equal(ref.unpack_codes(codes, block, bits), q)
        back = ref.decode(codes, scales, block, bits, block)
        assert np.max(np.abs(back - x)) <= 1e-5 * float(scales[0])


@pytest.mark.parametrize("bits,block", BITS_BLOCK)
@pytest.mark.parametrize("kind", ["normal", "laplace", "t3"])
def test_sure_error_bound_and_absmax(ref, bits, block, kind):
    """|C(x)_j - x_j| < a/s for every draw; the max-norm element gets |q| = s (in at least 99 % of the blocks;
    never less than s - 1: fl(s / a) * a can land one fixed-point unit under s * 2^16, and then a small draw
    leaves it one level below); codes stay within [-s, s]; the stored scale is the block max-norm."""
    s = ref.levels(bits)
    rng = np.random.default_rng(11)
    N = block * 37 + block // 2                      # ragged last block
    x = _rand_x(rng, N, kind)
    top_hits = top_total = 0
    for seed in range(3):
        codes, scales = ref.quantise(x, bits, block, seed=seed, mat=1, step=seed)
        q = ref.unpack_codes(codes, N, bits)
        assert q.min() >= -s and q.max() <= s
        dec = ref.decode(codes, scales, N, bits, block)
        for b in range(ref.n_blocks(N, block)):
            sl = slice(b * block, min(N, (b + 1) * block))
            a = np.abs(x[sl]).max()
            assert scales[b] == a
            assert np.all(np.abs(dec[sl].astype(np.float64) - x[sl]) < float(a) / s * (1 + 1e-6))
            jmax = np.argmax(np.abs(x[sl]))
            # the max-norm element sits at the top level (one below only if its fixed-point
            # value lands one unit under s*2^16 and the draw is 0)
            assert abs(q[sl][jmax]) >= s - 1
            top_hits += int(abs(q[sl][jmax]) == s)
            top_total += 1
    assert top_hits >= 0.99 * top_total


def test_packing_is_lsb_first_twos_complement(ref):
    """Field j%W of word j/W sits at bits [b*(j%W), b*(j%W)+b); negative codes are two's complement."""
    for bits in (8, 4, 2):
        W = 32 // bits
        s = ref.levels(bits)
        B = 2 * W
        q = np.array([(-s + (3 * j) % (2 * s + 1)) for j in range(B)], np.int64)
        q[0] = s
        x = (q * 2.0 ** -3).astype(np.float32)
        codes, scales = ref.quantise(x, bits, B, draw=np.zeros(B, np.uint16))
        assert scales[0] == np.float32(s * 2.0 ** -3)
        want = np.zeros(2, np.uint64)
        for j in range(B):
            want[j // W] |= np.uint64((int(q[j]) & ((1 << bits) - 1)) << (bits * (j % W)))
        assert np.array_equal(codes.astype(np.uint64), want)


def test_zero_state_and_zero_block(ref):
    for bits, block in BITS_BLOCK:
        N = 3 * block
        e = ref.decode(np.zeros(ref.n_words(N, bits), np.uint32), np.zeros(3, np.float32), N, bits, block)
        assert np.all(e == 0)                         # e_0 = 0 (Algorithm 2, line 1) is the all-zero state
        x = np.zeros(N, np.float32)
        x[block + 3] = -2.5
        codes, scales = ref.quantise(x, bits, block, seed=5)
        assert scales[0] == 0 and scales[2] == 0 and scales[1] == 2.5
        q = ref.unpack_codes(codes, N, bits)
        assert q[block + 3] == -ref.levels(bits) and np.count_nonzero(q) == 1


@pytest.mark.parametrize("bits,block", BITS_BLOCK)
def test_unbiased_over_seeds(ref, bits, block):
    """Assumption 3 / Proposition 1(i): the mean of C(x) over many seeds is x.  Per-element
    tolerance 5 standard errors of a Bernoulli with the eq. (3) probability."""
    s = ref.levels(bits)
    rng = np.random.default_rng(3)
    N = 4 * block
    x = _rand_x(rng, N, "normal")
    S = 1500
    acc = np.zeros(N)
    for seed in range(S):
        codes, scales = ref.quantise(x, bits, block, seed=1000 + seed, mat=2, step=9)
        acc += ref.decode(codes, scales, N, bits, block)
    mean = acc / S
    a = np.repeat(np.abs(x).reshape(-1, block).max(1), block).astype(np.float64)
    _, f = [np.concatenate(t) for t in zip(*[_frac_parts(x[i * block:(i + 1) * block],
                                                          np.abs(x[i * block:(i + 1) * block]).max(), s)
                                             for i in range(4)])]
    tol = 5 * (a / s) * np.sqrt(np.maximum(f * (1 - f), 1e-4) / S) + a / s * 2.0 ** -15
    assert np.all(np.abs(mean - x) <= tol)
    # and no systematic shrink or growth overall
    assert abs((mean - x).sum()) <= 5 * np.sqrt(((a / s) ** 2 * f * (1 - f) / S).sum()) + 1e-12


@pytest.mark.parametrize("bits,block,kind,theta_max", [
    (8, 64, "normal", 2e-4), (4, 128, "normal", 0.05), (4, 128, "laplace", 0.09), (4, 128, "t3", 0.25)])
def test_variance_closed_form_and_contraction(ref, bits, block, kind, theta_max):
    """E||C(x)-x||^2 = sum_blocks (a/s)^2 sum_j f_j(1-f_j) (Bernoulli variance of the eq. (3)
    rule), which is at most B/(4 s^2) ||x||^2 because a <= ||x_block||; for the 8- and 4-bit
    settings this is a relative variance theta < 1 (Assumption 3)."""
    s = ref.levels(bits)
    rng = np.random.default_rng(5)
    nb = 64
    N = nb * block
    x = _rand_x(rng, N, kind)
    xb = x.reshape(nb, block)
    closed = 0.0
    for b in range(nb):
        a = np.abs(xb[b]).max()
        _, f = _frac_parts(xb[b], a, s)
        f = f.astype(np.float64)
        closed += (float(a) / s) ** 2 * (f * (1 - f)).sum()
    S = 300
    emp = 0.0
    for seed in range(S):
        codes, scales = ref.quantise(x, bits, block, seed=seed, mat=0, step=1)
        d = ref.decode(codes, scales, N, bits, block).astype(np.float64) - x
        emp += (d * d).sum()
    emp /= S
    nx2 = float((x.astype(np.float64) ** 2).sum())
    assert abs(emp - closed) <= 0.03 * closed
    assert closed <= block / (4.0 * s * s) * nx2
    theta = emp / nx2
    assert theta < theta_max < 1.0


def test_two_bit_is_the_ternary_scheme(ref):
    """b = 2 gives s = 1: codes in {-1, 0, +1} with P(q != 0) = |x|/a (the {+-1, 0} quantisation
    the paper names as a special case); at block 256 on Gaussian input its relative variance is
    above 1: unbiased, but not a contraction."""
    rng = np.random.default_rng(8)
    block, nb = 256, 16
    N = block * nb
    x = _rand_x(rng, N, "normal")
    S = 400
    nz = np.zeros(N)
    err = 0.0
    for seed in range(S):
        codes, scales = ref.quantise(x, 2, block, seed=seed)
        q = ref.unpack_codes(codes, N, 2)
        assert set(np.unique(q)) <= {-1, 0, 1}
        nz += (q != 0)
        d = ref.decode(codes, scales, N, 2, block).astype(np.float64) - x
        err += (d * d).sum()
    a = np.repeat(np.abs(x).reshape(nb, block).max(1), block)
    prob = np.abs(x) / a
    assert np.all(np.abs(nz / S - prob) <= 5 * np.sqrt(np.maximum(prob * (1 - prob), 1e-3) / S) + 1e-4)
    theta = err / S / float((x.astype(np.float64) ** 2).sum())
    assert 1.0 < theta < 64.0                        # 64 = B/(4 s^2)


def test_memory_saving_closed_form(ref):
    """Bytes kept per element against an fp32 error vector: 1 - (b + 32/B)/32, inside or near the
    80-90 % band the paper reports for its memory saving."""
    for bits, block, want in [(8, 64, 0.734), (4, 128, 0.867), (2, 256, 0.934)]:
        N = block * 1000
        kept = 4 * ref.n_words(N, bits) + 4 * ref.n_blocks(N, block)
        assert abs(1 - kept / (4 * N) - want) < 1e-3
        assert abs((1 - kept / (4 * N)) - (1 - (bits + 32 / block) / 32)) < 1e-12
