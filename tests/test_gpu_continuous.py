"""Continuous rollouts: more prompts than the cache holds, groups admitted as others finish.  Every sequence is
still the oracle's sequence n (its draws keyed by its own index and step), whatever shared the batch with it."""
import threading
import time

import numpy as np
import pytest

from paper_2602_02192_amd import synth

from gpu_util import (BF16_LOGPROB_TOL, F32_LOGPROB_TOL, check_tokens_fp32_sampler, make_ctx, oracle_rollout, valid_mask)

pytestmark = pytest.mark.gpu

MID = synth.ModelShape(2, 512, 8, 2, 128, 1024, 2048, dtype="bf16")


# the last two cases leave more than 32 rows in flight when the prompts run out, so the draining batch is compacted
@pytest.mark.parametrize("P,G,max_seqs,no_graph", [(7, 2, 4, False), (5, 3, 8, True), (3, 4, 4, False), (2, 2, 16, False),
                                                   (30, 2, 40, False), (12, 5, 70, True), (6, 1, 4, False)])
def test_fp32_free_running_matches_the_oracle_sequence_by_sequence(P, G, max_seqs, no_graph):
    shape = synth.TINY
    blob = synth.make_weights(shape, 0)
    blob32 = synth.widen_to_f32(blob)
    prompts, lens = synth.make_prompts(shape.vocab, P, 40, seed=P, ragged=True)
    lens[0] = 1                                            # a prompt of one token: nothing to prefill
    prompts[0, 1:] = -1
    lens[P - 1] = 33                                       # all but the last token fill exactly one key tile
    prompts[P - 1, :33] = np.arange(33) % shape.vocab
    max_new = 14
    stop = synth.make_stop_lens(P * G, 1, max_new, seed=3)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=1.0, seed=2, stop_lens=stop)
    ctx = make_ctx(shape, max_seqs, 64, blob)
    out = ctx.rollout(prompts, lens, G, max_new, 1.0, 2, stop_lens=stop, continuous=True, no_graph=no_graph)
    assert np.array_equal(out["lens"], ref["lens"]) and np.array_equal(out["lens"], stop)
    m = valid_mask(ref["lens"], max_new)
    if check_tokens_fp32_sampler(out["tokens"], ref) == 0:
        assert np.abs(out["logprobs"] - ref["logprobs"])[m].max() < F32_LOGPROB_TOL
    assert (out["tokens"][~m] == -1).all() and (out["logprobs"][~m] == 0).all()
    assert (out["versions"][m] == 0).all() and (out["versions"][~m] == -1).all()
    # teacher forced on the oracle's tokens every log-prob is comparable
    tf = ctx.rollout(prompts, lens, G, max_new, 1.0, 2, stop_lens=stop, continuous=True, forced=ref["tokens"].clip(0))
    check_tokens_fp32_sampler(tf["tokens"], ref)
    same = (tf["tokens"] == ref["tokens"]) & m
    assert np.abs(tf["logprobs"] - ref["logprobs"])[same].max() < F32_LOGPROB_TOL
    # nucleus sampling and an end-of-sequence token keep the same per-sequence meaning
    eos = int(ref["tokens"][1, 0])
    ref_e = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=0.8, seed=5, eos_id=eos, top_p=0.9)
    out_e = ctx.rollout(prompts, lens, G, max_new, 0.8, 5, eos_id=eos, top_p=0.9, continuous=True)
    clear = valid_mask(np.minimum(out_e["lens"], ref_e["lens"]), max_new) & (ref_e["margins"] > 1e-4)
    bad = (out_e["tokens"] != ref_e["tokens"]) & clear & (ref_e["gaps"] >= 1e-4)
    # a sequence that took another branch at a near-tie is only comparable up to there
    first_diff = np.where((out_e["tokens"] != ref_e["tokens"]).any(1), (out_e["tokens"] != ref_e["tokens"]).argmax(1), max_new)
    bad &= np.arange(max_new)[None, :] <= first_diff[:, None]
    assert not bad.any()
    ctx.close()


@pytest.mark.parametrize("P,max_seqs", [(9, 12), (20, 48)], ids=["three-groups", "compacted-while-draining"])
def test_bf16_path_against_the_oracle_and_against_rollouts_that_fit(P, max_seqs):
    shape = MID
    blob = synth.make_weights(shape, 0)
    blob32 = synth.widen_to_f32(blob)
    G, max_new = 4, 10
    prompts, lens = synth.make_prompts(shape.vocab, P, 70, seed=4, ragged=True)
    lens[2] = 65                                           # two whole shared key tiles, then the decode input
    prompts[2, :65] = (np.arange(65) * 7) % shape.vocab
    stop = synth.make_stop_lens(P * G, 2, max_new, seed=6)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=1.0, seed=2, stop_lens=stop)
    forced = ref["tokens"].clip(0)
    ctx = make_ctx(shape, max_seqs, 96, blob)
    out = ctx.rollout(prompts, lens, G, max_new, 1.0, 2, stop_lens=stop, continuous=True, forced=forced)
    m = valid_mask(stop, max_new)
    assert np.array_equal(out["lens"], stop)
    same = (out["tokens"] == ref["tokens"]) & m
    assert same[m].mean() > 0.9
    assert np.abs(out["logprobs"] - ref["logprobs"])[same].max() < BF16_LOGPROB_TOL
    # the first prompt alone through the ordinary rollout (which prefills the whole prompt and samples the first token
    # from that pass; its rows are streams 0..G-1 there as well): same tokens, log-probs within the two paths' tolerance
    one = ctx.rollout(prompts[:1], lens[:1], G, max_new, 1.0, 2, stop_lens=stop[:G], forced=forced[:G])
    agree = (one["tokens"] == out["tokens"][:G]) & m[:G]
    assert agree[m[:G]].mean() > 0.9
    assert np.abs(one["logprobs"] - out["logprobs"][:G])[agree].max() < 2 * BF16_LOGPROB_TOL
    ctx.close()


def test_shared_prompt_tiles_do_not_change_a_continuous_rollout():
    shape = MID
    blob = synth.make_weights(shape, 0)
    P, G, max_new = 6, 4, 8
    prompts, lens = synth.make_prompts(shape.vocab, P, 100, seed=8)
    lens[:] = [40, 100, 64, 65, 97, 33]                    # whole and cut key tiles before the decode input
    stop = synth.make_stop_lens(P * G, 1, max_new, seed=9)
    ctx = make_ctx(shape, 8, 128, blob)
    a = ctx.rollout(prompts, lens, G, max_new, 1.0, 3, stop_lens=stop, continuous=True)
    b = ctx.rollout(prompts, lens, G, max_new, 1.0, 3, stop_lens=stop, continuous=True, own_prompt_copy=True)
    for k in ("tokens", "logprobs", "lens"):
        assert np.array_equal(a[k], b[k]), k
    # what shares the batch with a sequence does not change its record beyond rounding (another batch size splits the
    # keys and the GEMMs differently): capacity for all groups at once, fed a's tokens, reproduces a
    ctx.close()
    big = make_ctx(shape, 24, 128, blob)
    c = big.rollout(prompts, lens, G, max_new, 1.0, 3, stop_lens=stop, continuous=True, forced=a["tokens"].clip(0))
    m = valid_mask(stop, max_new)
    same = (a["tokens"] == c["tokens"]) & m
    assert np.array_equal(a["lens"], c["lens"]) and same[m].mean() > 0.97
    assert np.abs(a["logprobs"] - c["logprobs"])[same].max() < 2 * BF16_LOGPROB_TOL
    big.close()


def test_a_staged_snapshot_is_switched_in_between_steps_and_errors():
    from paper_2602_02192_amd import echo
    shape = synth.TINY
    A, B = synth.make_weights(shape, 0), synth.make_weights(shape, 10)
    P, G, max_new = 40, 2, 24
    prompts, lens = synth.make_prompts(shape.vocab, P, 16, seed=1)
    ctx = make_ctx(shape, 4, 48, A, version=3, slots=2)
    box = {}
    t = threading.Thread(target=lambda: box.update(out=ctx.rollout(prompts, lens, G, max_new, 1.0, 2, continuous=True)))
    t.start()
    for _ in range(2000):
        if ctx.stats().rollout_running:
            break
        time.sleep(0.002)
    assert ctx.stats().rollout_running
    ctx.load_policy(8, B)
    t.join(120)
    assert not t.is_alive() and "out" in box
    v = box["out"]["versions"]
    assert set(np.unique(v)) <= {3, 8} and (v[-1] == 8).all()          # the last prompt ran wholly under the new snapshot
    assert (np.diff(v, axis=1) >= 0).all()                                # within a sequence versions only advance
    assert ctx.stats().active_version == 8
    # what a continuous rollout refuses
    for bad, code in ((lambda: ctx.rollout(prompts, lens, 5, 4, 1.0, 2, continuous=True), echo.ECHO_ENOMEM),   # G > max_seqs
                      (lambda: ctx.rollout(prompts, lens, G, 40, 1.0, 2, continuous=True), echo.ECHO_ENOMEM),  # context
                      (lambda: ctx.rollout(prompts, lens, G, 4, 1.0, 2, continuous=True, swap_at_step=[2]), echo.ECHO_EINVAL),
                      (lambda: ctx.rollout(prompts[:1], lens[:1], G, 4, 1.0, 2, continuous=True, want_logits=True), echo.ECHO_EINVAL),
                      (lambda: ctx.rollout(prompts, lens * 0, G, 4, 1.0, 2, continuous=True), echo.ECHO_EINVAL)):
        with pytest.raises(echo.EchoError) as e:
            bad()
        assert e.value.code == code
    ctx.close()


@pytest.mark.parametrize("prefix_kernel", [2, 3], ids=["once-per-group-kernel", "several-rows-per-decode-workgroup"])
def test_refill_and_compaction_with_the_groups_prompts_attended_once_per_group(prefix_kernel):
    """Enough rows that a row's keys stay in one workgroup, so the shared prompt tiles can go through the prefix kernel
    (forced on: at this size it would not pay): its job list is rebuilt as groups are admitted, finish and are
    compacted.  The same with decode workgroups that take eight neighbouring rows -- rows at different positions, of
    different groups once rows have moved, idle rows between them -- and the prompt tiles that neighbours of one group have
    in common once.  Teacher-forced against the oracle."""
    shape = MID
    blob = synth.make_weights(shape, 0)
    blob32 = synth.widen_to_f32(blob)
    P, G, max_new = 30, 8, 12
    prompts, lens = synth.make_prompts(shape.vocab, P, 100, seed=12)
    lens[:] = np.resize(np.array([33, 64, 100, 65, 97, 40, 32], np.int32), P)     # 32: one whole tile minus the decode input
    stop = synth.make_stop_lens(P * G, 1, max_new, seed=13)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=1.0, seed=2, stop_lens=stop)
    ctx = make_ctx(shape, 168, 128, blob)
    out = ctx.rollout(prompts, lens, G, max_new, 1.0, 2, stop_lens=stop, continuous=True, forced=ref["tokens"].clip(0), prefix_kernel=prefix_kernel)
    m = valid_mask(stop, max_new)
    assert np.array_equal(out["lens"], stop)
    same = (out["tokens"] == ref["tokens"]) & m
    assert same[m].mean() > 0.9
    assert np.abs(out["logprobs"] - ref["logprobs"])[same].max() < BF16_LOGPROB_TOL
    ctx.close()
