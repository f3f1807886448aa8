"""GPU parity of the learner-side tensors (turn-aware response mask, group-normalised advantages, per-token
advantages) against the oracle: masks bit for bit, advantages to f32 rounding of the f64 result."""
import numpy as np
import pytest

from paper_2602_02192_amd import synth

from gpu_util import make_ctx

pytestmark = pytest.mark.gpu

TAU = 11
SMALL = synth.ModelShape(2, 512, 8, 2, 128, 1024, 2048, dtype="bf16")   # its context stages 256 KB at 8 sequences
ADV_TOL = 1e-7      # sums in f64 on both sides; what is left is the f32 rounding of the result (2^-24 relative)


def check(ctx, orc, toks, lens, G, rewards, eps=1e-6, per_token=True):
    mask, adv, adv_tok = ctx.grpo_tensors(toks, lens, G, TAU, rewards, eps, per_token=per_token)
    rmask, radv, radv_tok = orc.grpo_tensors(toks, lens, G, TAU, rewards.astype(np.float64), float(np.float32(eps)))
    assert np.array_equal(mask, rmask)
    np.testing.assert_allclose(adv, radv, rtol=ADV_TOL, atol=1e-30, equal_nan=True)   # 0/0 of an all-equal group at eps = 0
    if per_token:
        assert np.array_equal(adv_tok != 0, (rmask == 1) & (adv[:, None] != 0))
        assert np.array_equal(adv_tok, np.where(rmask == 1, adv[:, None], np.float32(0)), equal_nan=True)   # exactly the sequence's value
    else:
        assert adv_tok is None
    return mask, adv


@pytest.mark.parametrize("N,G,stride,binary", [(48, 16, 5000, True), (6, 3, 1027, False), (64, 2, 1000, True),
                                              (2, 2, 1, True), (4, 4, 3, False), (130, 65, 4096, False), (8, 4, 12290, True)])
def test_learner_tensors_match_the_oracle(orc, N, G, stride, binary):
    ctx = make_ctx(synth.TINY, 8, 64)       # no policy: the call needs none
    toks, lens, rewards = synth.make_turn_records(N, stride, 1024, TAU, seed=N + stride, binary_rewards=binary)
    mask, adv = check(ctx, orc, toks, lens, G, rewards)
    if stride >= 1000:
        assert 0.05 < mask.mean() < 0.6                       # the recipe does produce response tokens
        check(ctx, orc, toks, lens, G, rewards, eps=0.0, per_token=False)
    ctx.close()


def test_small_staging_buffer_takes_several_passes_and_refuses_an_oversized_group(orc):
    from paper_2602_02192_amd import echo
    ctx = make_ctx(SMALL, 8, 64)
    toks, lens, rewards = synth.make_turn_records(96, 2000, 2048, TAU, seed=5)     # 1.7 MB of staging in all
    check(ctx, orc, toks, lens, 2, rewards)
    check(ctx, orc, toks, lens, 8, rewards)
    with pytest.raises(echo.EchoError) as e:                                       # one group of 16 x 9216 tokens: 1.3 MB
        ctx.grpo_tensors(np.zeros((16, 9216), np.int32), np.zeros(16, np.int32), 16, TAU, np.zeros(16, np.float32))
    assert e.value.code == echo.ECHO_ENOMEM
    for bad in (lambda: ctx.grpo_tensors(toks[:4], lens[:4], 1, TAU, rewards[:4]),
                lambda: ctx.grpo_tensors(toks[:5], lens[:5], 2, TAU, rewards[:5]),
                lambda: ctx.grpo_tensors(toks[:4], lens[:4] * 0 + 2001, 2, TAU, rewards[:4]),
                lambda: ctx.grpo_tensors(toks[:4], lens[:4], 2, TAU, rewards[:4], eps=-1.0)):
        with pytest.raises(echo.EchoError) as e:
            bad()
        assert e.value.code == echo.ECHO_EINVAL
    ctx.close()


def test_learner_tensors_at_the_paper_batch_shape(orc):
    """32 prompts x 16 samples of up to 1024 + 8192 tokens (Sec. 5.1's sampling setting) through the 4B-class
    context the benchmark uses (no policy needed), whose staging buffer takes the batch in several passes."""
    ctx = make_ctx(synth.DENSE_4B, 64, 512 + 1024)
    toks, lens, rewards = synth.make_turn_records(512, 9216, synth.DENSE_4B.vocab, 151644, seed=3)
    global TAU
    keep, TAU = TAU, 151644
    try:
        mask, adv = check(ctx, orc, toks, lens, 16, rewards)
    finally:
        TAU = keep
    assert mask.any() and (adv != 0).any()
    ctx.close()
