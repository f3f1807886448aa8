"""Pins for the oracle's nucleus (top-p) sampler (CPU only).

What fixes it: top_p = 1 is the plain sampler; distributions whose kept set can be read off by hand
(dyadic uniform, a four-token table); the kept set is the shortest prefix of the descending order
reaching top_p, by brute force over all prefixes on small inputs; and sampling from the kept set in
proportion to p, by the frequencies of many draws (Gumbel-max theorem on the kept set)."""
import numpy as np
import pytest
from scipy import stats


def test_top_p_one_is_the_plain_sampler(orc):
    rng = np.random.default_rng(1)
    z = rng.normal(0, 2, 300)
    for s in range(40):
        tok, lp, gap, kept, margin = orc.sample_top_p(z, 0.8, 1.0, 5, 3, s)
        assert (tok, lp, gap) == orc.sample(z, 0.8, 5, 3, s)
        assert kept == 300


def test_uniform_dyadic_distribution_keeps_the_lowest_indices(orc):
    # 128 equal logits: p_i = 2^-7 exactly, every cumulative sum is exact; top_p = 1/4 keeps exactly 32 tokens,
    # the lower index first among equals, and every kept token has renormalised probability 1/32
    z = np.full(128, 0.37)
    seen = set()
    for s in range(400):
        tok, lp, gap, kept, margin = orc.sample_top_p(z, 1.0, 0.25, 9, 0, s)
        assert kept == 32 and 0 <= tok < 32
        assert lp == pytest.approx(-np.log(32.0), abs=1e-12)
        assert margin == pytest.approx(0.0, abs=1e-15)      # the cut sits exactly on top_p
        seen.add(tok)
    assert len(seen) == 32
    # with flat logits the winner is the kept index with the largest uniform draw
    for s in range(20):
        bits = np.array([orc.draw_bits(9, 0, s, i) >> 9 for i in range(32)])
        assert orc.sample_top_p(z, 1.0, 0.25, 9, 0, s)[0] == int(np.argmax(bits))
    # just above 1/4 one more token is needed
    assert orc.sample_top_p(z, 1.0, 0.2500001, 9, 0, 0)[3] == 33


@pytest.mark.parametrize("top_p,kept_set", [(0.4, [2]), (0.5, [2]), (0.51, [2, 0]), (0.79, [2, 0]), (0.81, [2, 0, 3]),
                                            (0.96, [2, 0, 3, 1])])
def test_four_token_table(orc, top_p, kept_set):
    p = np.array([0.3, 0.05, 0.5, 0.15])      # descending order: 2, 0, 3, 1
    z = np.log(p) + 1.7                        # softmax is shift invariant
    q = p[kept_set] / p[kept_set].sum()
    counts = dict.fromkeys(kept_set, 0)
    draws = 4000
    for s in range(draws):
        tok, lp, gap, kept, margin = orc.sample_top_p(z, 1.0, top_p, 3, 1, s)
        assert kept == len(kept_set) and tok in counts
        assert lp == pytest.approx(np.log(p[tok] / p[kept_set].sum()), abs=1e-9)
        counts[tok] += 1
    if len(kept_set) > 1:
        assert stats.chisquare([counts[t] for t in kept_set], q * draws).pvalue > 1e-3


def test_kept_set_is_the_shortest_prefix_reaching_top_p(orc):
    rng = np.random.default_rng(4)
    for trial in range(60):
        V = int(rng.integers(2, 40))
        z = rng.normal(0, 2.0, V)
        if trial % 3 == 0:
            z[rng.integers(0, V, 3)] = z[0]            # exact ties
        T = float(np.float32(rng.choice([1.0, 0.6, 1.5])))         # the C interface takes both as float
        top_p = float(np.float32(rng.uniform(0.05, 0.999)))
        p = np.exp(z / T - (z / T).max())
        p /= p.sum()
        order = sorted(range(V), key=lambda i: (-p[i], i))
        cum = np.cumsum(p[order])
        k = int(np.argmax(cum >= top_p)) + 1 if (cum >= top_p).any() else V
        lo = top_p - (cum[k - 2] if k > 1 else 0.0)
        hi = cum[k - 1] - top_p
        if min(lo, hi) < 1e-9:
            continue                                    # a cut that rounding could move
        toks = set()
        for s in range(30):
            tok, lp, gap, kept, margin = orc.sample_top_p(z, T, top_p, 11, trial, s)
            assert kept == k
            assert tok in order[:k]
            assert lp == pytest.approx(np.log(p[tok] / cum[k - 1]), abs=1e-9)
            assert margin == pytest.approx(min(lo, hi) if k < V else lo, abs=1e-9)   # nothing lies beyond the last token
            toks.add(tok)
        # the sampler's noise is tied to the vocabulary index: a kept token's draw does not depend on what else is kept,
        # so whenever the plain sampler's token is in the kept set, the nucleus sampler returns the same token
        for s in range(30):
            plain = orc.sample(z, T, 11, trial, s)[0]
            if plain in order[:k]:
                assert orc.sample_top_p(z, T, top_p, 11, trial, s)[0] == plain


def test_rollout_with_top_p(orc):
    from oracle import oracle as oracle_mod
    from paper_2602_02192_amd import synth
    shape = synth.TINY
    blob = synth.widen_to_f32(synth.make_weights(shape, 0))
    d = oracle_mod.desc_from_shape(shape)
    prompts, lens = synth.make_prompts(shape.vocab, 2, 6, seed=1)
    full = orc.rollout(d, blob, prompts, lens, 2, 5, 1.0, 3, want_logits=True)
    one = orc.rollout(d, blob, prompts, lens, 2, 5, 1.0, 3, top_p=1.0)
    assert np.array_equal(full["tokens"], one["tokens"]) and np.array_equal(full["logprobs"], one["logprobs"])
    # teacher-forced on the plain rollout's tokens the logits are the same, so every step can be checked on its own
    nuc = orc.rollout(d, blob, prompts, lens, 2, 5, 1.0, 3, top_p=0.5, forced=full["tokens"], want_logits=True)
    assert np.allclose(nuc["logits"], full["logits"])
    for n in range(4):
        for s in range(5):
            tok, lp, gap, kept, margin = orc.sample_top_p(full["logits"][n, s], 1.0, 0.5, 3, n, s)
            assert nuc["tokens"][n, s] == tok and nuc["logprobs"][n, s] == pytest.approx(lp, abs=1e-12)
            assert nuc["margins"][n, s] == pytest.approx(margin, abs=1e-12)
            assert kept < shape.vocab and nuc["logprobs"][n, s] > np.log(1.0 / kept) - 5.0
