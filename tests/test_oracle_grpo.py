"""Pins for the oracle's learner-side tensors (CPU only): the turn-aware response mask and the group-wise
normalised advantages of the paper's appendix.  What fixes them: token strings whose turn structure is written
out by hand, closed-form means and sample standard deviations, and the invariances of a standardisation."""
import numpy as np
import pytest

TAU = 7


def test_response_mask_on_hand_written_turns(orc):
    #            sys      user        assistant      user     assistant
    s = [TAU, 1, 2,   TAU, 3,      TAU, 4, 5, 6,   TAU, 8,   TAU, 9, 9]
    want = [0, 0, 0,   0, 0,        1, 1, 1, 1,     0, 0,     1, 1, 1]
    toks = np.array([s + [TAU, TAU],            # padding beyond the length is masked out whatever it holds
                     [1, 2, 3] + s[:13]])       # tokens before the first turn start belong to turn 0
    lens = np.array([len(s), 16], np.int32)
    mask, adv, adv_tok = orc.grpo_tensors(toks, lens, 2, TAU, [1.0, 3.0])
    assert mask[0].tolist() == want + [0, 0]
    assert mask[1].tolist() == [0, 0, 0] + want[:13]
    # turn index: cumulative count of turn starts, the start token itself already belongs to the new turn
    c = np.cumsum(np.array(s) == TAU)
    assert mask[0, :len(s)].tolist() == ((c > 1) & (c % 2 == 1)).astype(int).tolist()
    # per-token advantages: the sequence's advantage on the response tokens, zero elsewhere
    assert np.array_equal(adv_tok[0] != 0, mask[0] == 1)
    assert np.allclose(adv_tok[0][mask[0] == 1], adv[0]) and np.allclose(adv_tok[1][mask[1] == 1], adv[1])


def test_no_turn_start_or_a_single_turn_selects_nothing(orc):
    toks = np.array([[1, 2, 3, 4], [TAU, 2, 3, 4]])
    mask, _, _ = orc.grpo_tensors(toks, [4, 4], 2, TAU, [0.0, 1.0])
    assert not mask.any()


def test_advantages_closed_form(orc):
    toks = np.zeros((8, 1), np.int32)
    r = [1.0, 2.0, 3.0, 4.0, 10.0, 10.0, 10.0, 10.0]
    _, adv, _ = orc.grpo_tensors(toks, np.ones(8, np.int32), 4, TAU, r, eps=1e-6)
    sd = np.sqrt(5.0 / 3.0)                     # sample standard deviation of 1, 2, 3, 4 (divisor n - 1)
    assert adv[:4] == pytest.approx(np.array([-1.5, -0.5, 0.5, 1.5]) / (sd + 1e-6), abs=1e-14)
    assert (adv[4:] == 0).all()                 # a group of equal returns: 0 / (0 + eps)
    # two returns a, b: mean (a+b)/2, sample std |a-b|/sqrt 2, so the advantages are -+ 1/sqrt 2 (up to eps)
    _, adv, _ = orc.grpo_tensors(toks[:2], [1, 1], 2, TAU, [-3.0, 5.0], eps=0.0)
    assert adv == pytest.approx([-1 / np.sqrt(2), 1 / np.sqrt(2)], abs=1e-15)


def test_advantages_are_a_standardisation(orc):
    rng = np.random.default_rng(0)
    G, groups = 16, 5
    r = rng.normal(3.0, 40.0, G * groups)
    toks = np.zeros((G * groups, 1), np.int32)
    ones = np.ones(G * groups, np.int32)
    _, adv, _ = orc.grpo_tensors(toks, ones, G, TAU, r, eps=0.0)
    a = adv.reshape(groups, G)
    assert np.abs(a.mean(axis=1)).max() < 1e-13
    assert a.std(axis=1, ddof=1) == pytest.approx(np.ones(groups), abs=1e-12)
    # shift and positive scale of a group's returns change nothing (eps = 0); groups do not see each other
    r2 = r.copy()
    r2[:G] = 7.5 * r[:G] - 100.0
    r2[G:2 * G] = rng.normal(0, 1, G)
    _, adv2, _ = orc.grpo_tensors(toks, ones, G, TAU, r2, eps=0.0)
    assert adv2[:G] == pytest.approx(adv[:G], abs=1e-12)
    assert np.array_equal(adv2[2 * G:], adv[2 * G:])
    # eps only damps: same signs, smaller magnitudes
    _, adv3, _ = orc.grpo_tensors(toks, ones, G, TAU, r, eps=5.0)
    assert (np.sign(adv3) == np.sign(adv)).all() and (np.abs(adv3) < np.abs(adv)).all()
    with pytest.raises(ValueError):
        orc.grpo_tensors(toks[:3], ones[:3], 1, TAU, r[:3])      # one sample has no standard deviation
    with pytest.raises(ValueError):
        orc.grpo_tensors(toks[:5], ones[:5], 2, TAU, r[:5])      # not whole groups
