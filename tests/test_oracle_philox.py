"""Pins for the oracle's random source: Philox4x32-10 and the 16-bit draw layout."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(t, 16) for t in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def py_philox(ctr, key, rounds=10):
    """Philox4x32 written with Python integers (independent of the C oracle)."""
    c = list(ctr)
    k = list(key)
    for _ in range(rounds):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF,
             ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_known_answers(ref):
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert [int(v) for v in ref.philox4x32_10(ctr, key)] == want
        assert py_philox(ctr, key) == want          # the test's own copy is pinned too


def test_random_inputs_agree_with_python_integers(ref):
    rng = np.random.default_rng(1)
    for _ in range(50):
        ctr = [int(v) for v in rng.integers(0, 2**32, 4)]
        key = [int(v) for v in rng.integers(0, 2**32, 2)]
        assert [int(v) for v in ref.philox4x32_10(ctr, key)] == py_philox(ctr, key)


def test_rand16_layout(ref):
    """Element j uses counter (j>>3, mat, lo(step), hi(step)), key (lo(seed), hi(seed)), and
    takes half (j&1) of word (j&7)>>1, low half first."""
    seed, mat, step = 0x0123456789ABCDEF, 7, (5 << 32) | 11
    for j in [0, 1, 2, 7, 8, 9, 15, 1000003, (1 << 33) + 5]:
        out = py_philox([(j >> 3) & 0xFFFFFFFF, mat, step & 0xFFFFFFFF, step >> 32],
                        [seed & 0xFFFFFFFF, seed >> 32])
        w = out[(j & 7) >> 1]
        want = (w >> 16) if (j & 1) else (w & 0xFFFF)
        assert ref.rand16(seed, mat, step, j) == want


def test_rand16_depends_on_every_argument(ref):
    base = ref.rand16(1, 2, 3, 4)
    eight = [ref.rand16(1, 2, 3, j) for j in range(8)]
    assert len(set(eight)) == 8                      # 8 distinct halves of one call
    diffs = [ref.rand16(2, 2, 3, 4), ref.rand16(1, 3, 3, 4), ref.rand16(1, 2, 4, 4),
             ref.rand16(1, 2, 3 + (1 << 32), 4), ref.rand16(1 + (1 << 32), 2, 3, 4)]
    assert all(d != base for d in diffs)


def test_rand16_is_uniform(ref):
    n = 40000
    v = np.array([ref.rand16(99, 0, 0, j) for j in range(n)])
    assert v.min() >= 0 and v.max() <= 65535
    assert abs(v.mean() - 32767.5) < 4 * 65536 / np.sqrt(12 * n)
    hist = np.bincount(v >> 12, minlength=16)
    chi2 = ((hist - n / 16) ** 2 / (n / 16)).sum()
    assert chi2 < 45.0                               # 15 dof, p ~ 1e-4
