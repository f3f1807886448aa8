"""Pins for the oracle's primitives (CPU only): closed forms, invariants and
special cases that reduce to textbook identities."""
import numpy as np
import pytest
from scipy.special import log_softmax, softmax


def test_rmsnorm_unit_rms_scale_invariance_and_gain(orc):
    rng = np.random.default_rng(0)
    x = rng.normal(0, 3, 64)
    y = orc.rmsnorm(x, np.ones(64), 0.0)
    assert np.sqrt(np.mean(y * y)) == pytest.approx(1.0, abs=1e-12)
    assert np.allclose(orc.rmsnorm(7.5 * x, np.ones(64), 0.0), y, atol=1e-12)
    g = rng.normal(1, 0.3, 64).astype(np.float32)
    assert np.allclose(orc.rmsnorm(x, g, 0.0), y * g, atol=1e-12)      # gain is elementwise
    # eps sits inside the square root, added to the mean square
    x2 = np.array([3.0, 4.0])
    assert np.allclose(orc.rmsnorm(x2, np.ones(2), 0.5), x2 / np.sqrt(12.5 + np.float32(0.5)), atol=1e-12)
    # a hand value: (2,0,0,0) has mean square 1
    assert np.allclose(orc.rmsnorm(np.array([2.0, 0, 0, 0]), np.ones(4), 0.0), [2, 0, 0, 0])


def test_rope_identity_pairing_direction_and_frequencies(orc):
    rng = np.random.default_rng(1)
    x = rng.normal(0, 1, 8)
    assert np.array_equal(orc.rope(x, 0, 1e4), x)                       # position 0 is the identity
    # half-split pairing (i, i+hd/2), angle pos * base^(-2i/hd), counter-clockwise
    e0 = np.array([1.0, 0, 0, 0])
    assert np.allclose(orc.rope(e0, 1, 1e4), [np.cos(1.0), 0, np.sin(1.0), 0], atol=1e-15)
    e1 = np.array([0.0, 1.0, 0, 0])
    th1 = 1e4 ** (-2.0 / 4.0)
    assert np.allclose(orc.rope(e1, 3, 1e4), [0, np.cos(3 * th1), 0, np.sin(3 * th1)], atol=1e-15)
    e2 = np.array([0.0, 0, 1.0, 0])
    assert np.allclose(orc.rope(e2, 2, 1e4), [-np.sin(2.0), 0, np.cos(2.0), 0], atol=1e-15)
    # norm preserving; composition of rotations adds positions
    for pos in (1, 17, 4095):
        assert np.linalg.norm(orc.rope(x, pos, 1e4)) == pytest.approx(np.linalg.norm(x), rel=1e-12)


def test_rope_inner_product_depends_on_relative_position_only(orc):
    rng = np.random.default_rng(2)
    q, k = rng.normal(0, 1, 64), rng.normal(0, 1, 64)
    ref = orc.rope(q, 9, 1e4) @ orc.rope(k, 4, 1e4)
    for shift in (1, 100, 3000):
        assert orc.rope(q, 9 + shift, 1e4) @ orc.rope(k, 4 + shift, 1e4) == pytest.approx(ref, abs=1e-9)
    assert orc.rope(q, 9, 1e4) @ orc.rope(k, 5, 1e4) != pytest.approx(ref, abs=1e-6)


def test_silu_closed_forms(orc):
    assert orc.silu(0.0) == 0.0
    assert orc.silu(1.0) == pytest.approx(0.7310585786300049, abs=1e-15)
    for x in (0.3, 2.0, 11.0):
        assert orc.silu(x) - orc.silu(-x) == pytest.approx(x, abs=1e-12)
    assert orc.silu(-40.0) == pytest.approx(0.0, abs=1e-15)
    assert orc.silu(40.0) == pytest.approx(40.0, abs=1e-12)


def test_attention_special_cases(orc):
    rng = np.random.default_rng(3)
    hd = 16
    q = rng.normal(0, 1, hd)
    k = rng.normal(0, 1, (5, hd))
    v = rng.normal(0, 1, (5, hd))
    assert np.array_equal(orc.attend(q, k[:1], v[:1]), v[0])            # one key -> its value
    assert np.allclose(orc.attend(np.zeros(hd), k, v), v.mean(0), atol=1e-14)   # equal scores -> mean
    w = softmax(k @ q / np.sqrt(hd))                                    # library softmax, 1/sqrt(hd) scale
    assert np.allclose(orc.attend(q, k, v), w @ v, atol=1e-13)
    # huge scores do not overflow (max is subtracted) and select the best key
    big = orc.attend(300.0 * k[2], k, v)
    assert np.all(np.isfinite(big))
    # permuting the keys together with the values changes nothing
    perm = rng.permutation(5)
    assert np.allclose(orc.attend(q, k[perm], v[perm]), orc.attend(q, k, v), atol=1e-14)


def test_log_softmax_rows_sum_to_one_shift_and_temperature(orc):
    rng = np.random.default_rng(4)
    z = rng.normal(0, 2, 1000)
    ls = orc.log_softmax(z)
    assert np.exp(ls).sum() == pytest.approx(1.0, abs=1e-12)
    assert np.all(ls <= 0)
    assert np.allclose(orc.log_softmax(z + 123.0), ls, atol=1e-10)
    assert np.allclose(ls, log_softmax(z), atol=1e-12)
    assert np.allclose(orc.log_softmax(z, 0.5), log_softmax(z / 0.5), atol=1e-12)
    assert np.all(np.isfinite(orc.log_softmax(np.array([1e4, 0.0, -1e4]))))


def test_fp32_build_agrees_with_fp64_build(orc, orc32):
    rng = np.random.default_rng(5)
    x = rng.normal(0, 1, 128)
    assert np.allclose(orc32.rmsnorm(x, np.ones(128), 1e-6), orc.rmsnorm(x, np.ones(128), 1e-6), atol=1e-6)
    assert np.allclose(orc32.rope(x, 77, 1e4), orc.rope(x, 77, 1e4), atol=1e-6)
    assert np.allclose(orc32.log_softmax(x), orc.log_softmax(x), atol=1e-5)
