"""Pins for the oracle's Philox generator and its uniform / Gumbel maps."""
import os

import numpy as np
from scipy import stats

from oracle import philox

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat_rows():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([int(t, 16) for t in line.split()])
    return rows


def test_known_answer_vectors():
    rows = _kat_rows()
    assert len(rows) == 3
    for r in rows:
        out = philox.philox4x32_10(*r[:6])
        assert [int(x) for x in out] == r[6:]


def test_vectorised_equals_scalar_calls():
    rng = np.random.default_rng(1)
    c = rng.integers(0, 2 ** 32, size=(6, 50), dtype=np.uint64)
    vec = philox.philox4x32_10(*c)
    for i in range(50):
        one = philox.philox4x32_10(*[int(c[j, i]) for j in range(6)])
        assert [int(v[i]) for v in vec] == [int(x) for x in one]


def test_counter_layout():
    # entry x of a row is output word (x & 3) of the block with counter word 0 = x >> 2,
    # word 1 = node row, word 2 = sequence, word 3 = tag | step << 4; key = seed halves.
    seed, step, tag, seq, node = 0x0123456789ABCDEF, 5, 2, 77, 9
    w = philox.words(seed, step, tag, seq, node, np.arange(16))
    for x in range(16):
        blk = philox.philox4x32_10(x >> 2, node, seq, tag | (step << 4),
                                   seed & 0xFFFFFFFF, seed >> 32)
        assert int(w[x]) == int(blk[x & 3])
    # changing any coordinate changes the stream
    base = philox.words(seed, step, tag, seq, node, np.arange(64))
    for kw in (dict(seed=seed + 1), dict(step=step + 1), dict(tag=tag + 1),
               dict(seq=seq + 1), dict(node=node + 1)):
        a = dict(seed=seed, step=step, tag=tag, seq=seq, node=node)
        a.update(kw)
        other = philox.words(a["seed"], a["step"], a["tag"], a["seq"], a["node"], np.arange(64))
        assert np.mean(other == base) < 0.1


def test_uniform_grid_is_open_and_fp32_exact():
    w = np.array([0, 1, 511, 512, 2 ** 32 - 1, 2 ** 31], dtype=np.uint64)
    u = philox.uniform_from_word(w)
    assert u.min() == 2.0 ** -24 and u.max() == 1.0 - 2.0 ** -24
    assert np.all(u.astype(np.float32).astype(np.float64) == u)
    # odd multiples of 2^-24
    assert np.all((u * 2 ** 24) % 2 == 1)


def test_uniform_and_gumbel_moments():
    n = 1 << 20
    w = philox.words(42, 0, 0, 3, 1, np.arange(n))
    u = philox.uniform_from_word(w)
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    g = philox.gumbel_from_word(w)
    assert stats.kstest(g, "gumbel_r").pvalue > 1e-3
    assert abs(g.mean() - np.euler_gamma) < 5 * np.pi / np.sqrt(6 * n)
    assert abs(g.var() - np.pi ** 2 / 6) < 0.02
    # upper clip of the 24-bit grid
    assert g.max() <= -np.log(-np.log1p(-2.0 ** -24)) + 1e-12


def test_bits_are_balanced_and_rows_uncorrelated():
    n = 1 << 16
    a = philox.words(7, 0, 0, 0, 0, np.arange(n)).astype(np.uint64)
    b = philox.words(7, 0, 0, 0, 1, np.arange(n)).astype(np.uint64)
    for bit in range(32):
        frac = np.mean((a >> np.uint64(bit)) & np.uint64(1))
        assert abs(frac - 0.5) < 5 * 0.5 / np.sqrt(n)
    ua, ub = philox.uniform_from_word(a), philox.uniform_from_word(b)
    assert abs(np.corrcoef(ua, ub)[0, 1]) < 5 / np.sqrt(n)
    assert abs(np.corrcoef(ua[:-1], ua[1:])[0, 1]) < 5 / np.sqrt(n)


def test_accept_uniform_coordinates():
    u = philox.accept_uniform(11, 2, 5, 9)
    w = philox.philox4x32_10(0, 9, 5, 1 | (2 << 4), 11, 0)[0]
    assert u == (2 * (int(w) >> 9) + 1) * 2.0 ** -24
