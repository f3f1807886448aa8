"""GPU parity tests: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

from paper_2602_02192_amd import synth

from gpu_util import (BF16_LOGIT_TOL, BF16_LOGPROB_TOL, F32_LOGIT_TOL, F32_LOGPROB_TOL,
                      check_argmax, check_tokens_fp32_sampler, make_ctx, oracle_rollout, valid_mask)

pytestmark = pytest.mark.gpu


def test_generator_bits_match_definition(orc):
    ctx = make_ctx(synth.TINY, 8, 64)
    for seed, n, s, i0, cnt in [(0, 0, 0, 0, 4096), (0xDEADBEEF12345678, 255, 4095, 151000, 936), (2, 7, 31, 5, 1003)]:
        got = ctx.draw_bits(seed, n, s, i0, cnt)
        want = np.array([orc.draw_bits(seed, n, s, i0 + j) for j in range(cnt)], np.uint32)
        assert np.array_equal(got, want)
    ctx.close()


def _tiny_inputs(shape, P=4, plen=16, seed_w=0):
    blob = synth.make_weights(shape, seed_w)
    prompts, lens = synth.make_prompts(shape.vocab, P, plen, seed=1)
    return blob, synth.widen_to_f32(blob), prompts, lens


def test_tiny_fp32_rollout_matches_oracle():
    """Workload 1: 2-layer fp32 decoder, 4 prompts x G=2, prompt 16, 32 new tokens, T=1."""
    shape = synth.TINY
    blob, blob32, prompts, lens = _tiny_inputs(shape)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=2, max_new=32, temperature=1.0, seed=2, want_logits=True)
    ctx = make_ctx(shape, 8, 64, blob)
    # free running: the fp32 path draws the oracle's tokens (near-ties aside)
    out = ctx.rollout(prompts, lens, 2, 32, 1.0, 2)
    assert (out["lens"] == 32).all()
    n_flip = check_tokens_fp32_sampler(out["tokens"], ref)
    if n_flip == 0:
        assert np.abs(out["logprobs"] - ref["logprobs"]).max() < F32_LOGPROB_TOL
    # teacher forced on the oracle's stream: logits, log-probs and tokens
    tf = ctx.rollout(prompts, lens, 2, 32, 1.0, 2, forced=ref["tokens"], want_logits=True)
    assert np.abs(tf["logits"] - ref["logits"]).max() < F32_LOGIT_TOL
    check_tokens_fp32_sampler(tf["tokens"], ref)
    same = tf["tokens"] == ref["tokens"]
    assert np.abs(tf["logprobs"] - ref["logprobs"])[same].max() < F32_LOGPROB_TOL
    assert (tf["versions"] == 0).all()
    # graph replay and kernel-by-kernel launches give identical results
    ng = ctx.rollout(prompts, lens, 2, 32, 1.0, 2, no_graph=True)
    assert np.array_equal(ng["tokens"], out["tokens"]) and np.array_equal(ng["logprobs"], out["logprobs"])
    # per-step timing marks change nothing and return one duration per decode step
    ts = ctx.rollout(prompts, lens, 2, 32, 1.0, 2, time_steps=True)
    assert np.array_equal(ts["tokens"], out["tokens"]) and np.array_equal(ts["logprobs"], out["logprobs"])
    ms = ctx.step_times()
    assert ms.shape == (31,) and (ms > 0).all() and ms.sum() <= ctx.stats().decode_ms * 1.05 + 0.5
    ctx.close()


@pytest.mark.parametrize("debug_naive", [True, False])
def test_tiny_bf16_teacher_forced_matches_oracle(debug_naive):
    shape = synth.TINY.replace(dtype="bf16")
    blob, blob32, prompts, lens = _tiny_inputs(shape)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=2, max_new=32, temperature=1.0, seed=2, want_logits=True)
    ctx = make_ctx(shape, 8, 64, blob, debug_naive=debug_naive)
    tf = ctx.rollout(prompts, lens, 2, 32, 1.0, 2, forced=ref["tokens"], want_logits=True)
    tol = F32_LOGIT_TOL if debug_naive else BF16_LOGIT_TOL
    err = np.abs(tf["logits"] - ref["logits"]).max()
    assert err < tol, err
    m = valid_mask(ref["lens"], 32)
    check_argmax(tf["logits"], ref["logits"], m, tol, "tiny-bf16")
    same = tf["tokens"] == ref["tokens"]
    assert same.mean() > 0.9
    lp_tol = F32_LOGPROB_TOL if debug_naive else BF16_LOGPROB_TOL
    assert np.abs(tf["logprobs"] - ref["logprobs"])[same].max() < lp_tol
    # fused sampler == unfused fp32 sampler on the same logits, bit for bit
    if not debug_naive:
        fused = ctx.rollout(prompts, lens, 2, 32, 1.0, 2, forced=ref["tokens"])
        unf = ctx.rollout(prompts, lens, 2, 32, 1.0, 2, forced=ref["tokens"], unfused_sampler=True)
        assert np.array_equal(fused["tokens"], unf["tokens"])
        assert np.array_equal(fused["tokens"], tf["tokens"])
        assert np.abs(fused["logprobs"] - unf["logprobs"]).max() < 1e-5
    ctx.close()


MID = synth.ModelShape(2, 512, 8, 2, 128, 1024, 2048, dtype="bf16")


def test_mid_bf16_ragged_long_context_splitk_vs_oracle_and_simple():
    """head_dim 128, 4 query heads per KV head, ragged prompts that span several 256-key chunks and a
    ragged tail tile; the split-K MFMA attention against the oracle and against the plain kernel."""
    shape = MID
    blob = synth.make_weights(shape, 3)
    blob32 = synth.widen_to_f32(blob)
    prompts, lens = synth.make_prompts(shape.vocab, 3, 333, seed=4, ragged=True)
    lens[0] = 333                       # one prompt at full length: 2 chunks, last tile of 13 keys
    prompts[0] = synth.make_prompts(shape.vocab, 1, 333, seed=5)[0][0]
    stop = np.array([8, 3, 8, 5, 1, 8], np.int32)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=2, max_new=8, temperature=1.0, seed=7, stop_lens=stop,
                         want_logits=True)
    ctx = make_ctx(shape, 6, 352, blob)
    tf = ctx.rollout(prompts, lens, 2, 8, 1.0, 7, stop_lens=stop, forced=np.maximum(ref["tokens"], 0), want_logits=True)
    assert np.array_equal(tf["lens"], ref["lens"])
    m = valid_mask(ref["lens"], 8)
    err = np.abs(tf["logits"] - ref["logits"])[m].max()
    assert err < BF16_LOGIT_TOL, err
    assert (tf["tokens"][~m] == -1).all() and (tf["logprobs"][~m] == 0).all() and (tf["versions"][~m] == -1).all()
    same = (tf["tokens"] == ref["tokens"]) & m
    assert same[m].mean() > 0.9
    assert np.abs(tf["logprobs"] - ref["logprobs"])[same].max() < BF16_LOGPROB_TOL
    simple = ctx.rollout(prompts, lens, 2, 8, 1.0, 7, stop_lens=stop, forced=np.maximum(ref["tokens"], 0), want_logits=True,
                         attn_plain=True)
    assert np.abs(simple["logits"] - ref["logits"])[m].max() < BF16_LOGIT_TOL
    assert np.abs(simple["logits"] - tf["logits"])[m].max() < BF16_LOGIT_TOL
    ctx.close()


def test_the_c_client_runs_a_rollout_without_python():
    """csrc/echo_client.cpp through the C ABI alone (hipMalloc arena, the library's own streams): exit status 0 and a
    finite mean log-prob of a near-uniform policy over 1024 tokens."""
    import os
    import re
    import subprocess
    client = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2602_02192_amd", "echo_client")
    assert os.path.exists(client), "run `python -m paper_2602_02192_amd.build` first"
    r = subprocess.run([client, "tiny", "8", "16", "16"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr[-2000:]
    m = re.search(r"(\d+) tokens generated .* mean log-prob (-?[0-9.]+)", r.stdout)
    assert m, r.stdout
    assert int(m.group(1)) == 8 * 16
    lp = float(m.group(2))
    assert np.isfinite(lp) and -8.0 < lp < -6.0          # ln 1024 = 6.93
