"""Pins for the oracle's random draws and its Gumbel-max sampler (CPU only).

What fixes them: the generator's published known-answer vectors, the exact
dyadic form of the uniform mapping, and the Gumbel-max theorem (the argmax of
z_i + Gumbel noise is distributed as softmax(z))."""
import os

import numpy as np
import pytest
from scipy import stats

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        rows.append((w[:4], w[4:6], w[6:]))
    return rows


def test_philox_known_answers(orc):
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert [int(x) for x in orc.philox(ctr, key)] == want


def _philox_py(ctr, key):
    """The generator's definition with Python big integers (no shared code)."""
    c, k = list(ctr), list(key)
    for _ in range(10):
        p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_python_definition_agrees_on_kat_and_random_counters(orc):
    for ctr, key, want in _kat():
        assert _philox_py(ctr, key) == want
    rng = np.random.default_rng(5)
    for _ in range(200):
        ctr = [int(x) for x in rng.integers(0, 2**32, 4)]
        key = [int(x) for x in rng.integers(0, 2**32, 2)]
        assert [int(x) for x in orc.philox(ctr, key)] == _philox_py(ctr, key)


def test_draw_bits_counter_layout(orc):
    # entry i of (sequence n, step s): word i%4 of Philox((i//4, s, n, 0), (seed_lo, seed_hi))
    seed = 0x123456789ABCDEF
    for n, s, i in [(0, 0, 0), (3, 7, 5), (255, 1023, 151935), (1, 0, 2), (0, 1, 2)]:
        want = _philox_py([i // 4, s, n, 0], [seed & 0xFFFFFFFF, seed >> 32])[i % 4]
        assert orc.draw_bits(seed, n, s, i) == want
    # n and s must not be interchangeable, and the seed must matter
    assert orc.draw_bits(seed, 1, 0, 2) != orc.draw_bits(seed, 0, 1, 2)
    assert orc.draw_bits(seed, 1, 0, 2) != orc.draw_bits(seed + 1, 1, 0, 2)


def test_uniform_mapping_is_exact_and_open(orc):
    assert orc.uniform(0) == 2.0 ** -24
    assert orc.uniform(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert orc.uniform(0x1FF) == 2.0 ** -24            # low 9 bits are dropped
    assert orc.uniform(0x200) == 3.0 * 2.0 ** -24
    for bits in (0x80000000, 0x12345678, 0xDEADBEEF):
        assert orc.uniform(bits) == (2 * (bits >> 9) + 1) / 2.0 ** 24


def test_uniform_draws_are_uniform(orc):
    n = 1 << 16
    u = np.array([orc.uniform(orc.draw_bits(42, 3, 1, i)) for i in range(n)])
    assert abs(u.mean() - 0.5) < 4 * (1 / np.sqrt(12 * n))
    counts, _ = np.histogram(u, bins=64, range=(0, 1))
    assert stats.chisquare(counts).pvalue > 1e-3


def test_gumbel_closed_form(orc):
    for u in (2.0 ** -24, 0.1, 0.5, np.exp(-1.0), 0.9, 1 - 2.0 ** -24):
        u32 = float(np.float32(u))
        want = -np.log(-np.log(u32))
        assert orc.gumbel(u32) == pytest.approx(want, rel=2e-6, abs=2e-7)
    assert orc.gumbel(float(np.float32(np.exp(-1.0)))) == pytest.approx(0.0, abs=1e-6)
    assert np.isfinite(orc.gumbel(2.0 ** -24)) and np.isfinite(orc.gumbel(1 - 2.0 ** -24))


@pytest.mark.parametrize("temperature", [1.0, 0.7])
def test_gumbel_max_frequencies_match_softmax(orc, temperature):
    rng = np.random.default_rng(0)
    V = 16
    logits = rng.normal(0, 1.5, V)
    p = np.exp(logits / temperature - np.max(logits / temperature))
    p /= p.sum()
    draws = 40000
    counts = np.zeros(V)
    for j in range(draws):
        tok, lp, _ = orc.sample(logits, temperature, seed=99, n=j % 64, s=j // 64)
        counts[tok] += 1
        if j < 50:
            assert lp == pytest.approx(np.log(p[tok]), abs=1e-6)
    assert stats.chisquare(counts, p * draws).pvalue > 1e-3


def test_sampler_limits_ties_and_gap(orc):
    logits = np.array([0.0, 3.0, 1.0, 2.9])
    # a very low temperature turns sampling into argmax
    for s in range(50):
        assert orc.sample(logits, 1e-3, 7, 0, s)[0] == 1
    # same (seed, n, s) -> same draw; another seed, n or s changes some draws
    flat = np.zeros(64)
    a = [orc.sample(flat, 1.0, 1, 0, s)[0] for s in range(40)]
    assert a == [orc.sample(flat, 1.0, 1, 0, s)[0] for s in range(40)]
    assert a != [orc.sample(flat, 1.0, 2, 0, s)[0] for s in range(40)]
    assert a != [orc.sample(flat, 1.0, 1, 1, s)[0] for s in range(40)]
    # with flat logits the winner is the entry with the largest Gumbel variate,
    # i.e. the largest uniform; equal uniforms resolve to the lowest index
    for s in range(20):
        bits = np.array([orc.draw_bits(1, 0, s, i) >> 9 for i in range(64)])
        tok, lp, gap = orc.sample(flat, 1.0, 1, 0, s)
        assert tok == int(np.argmax(bits))           # argmax returns the first maximum
        assert lp == pytest.approx(-np.log(64.0), abs=1e-6)
        g = np.sort([orc.gumbel(orc.uniform(orc.draw_bits(1, 0, s, i))) for i in range(64)])
        assert gap == pytest.approx(g[-1] - g[-2], abs=1e-6)


def test_sampler_exact_ties_go_to_the_lowest_index(orc):
    # two entries so large that the fp32 sum z + g absorbs the noise: an exact tie
    z = np.zeros(32)
    z[[9, 20]] = 1e9
    for s in range(30):
        tok, lp, gap = orc.sample(z, 1.0, 5, 0, s)
        assert tok == 9 and gap == 0.0
        assert lp == pytest.approx(-np.log(2.0), abs=1e-6)


def test_sampler_decides_in_fp32_in_both_builds(orc, orc32):
    rng = np.random.default_rng(3)
    logits = rng.normal(0, 1, 512).astype(np.float32).astype(np.float64)
    for s in range(100):
        t64 = orc.sample(logits, 1.0, 11, 2, s)
        t32 = orc32.sample(logits, 1.0, 11, 2, s)
        assert t64[0] == t32[0] and t64[2] == t32[2]
        assert t64[1] == pytest.approx(t32[1], abs=5e-5)
