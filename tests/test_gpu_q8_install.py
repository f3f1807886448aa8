"""GPU parity of the quantised snapshot install: echo_load_policy_q8 must leave, bit for bit, the snapshot that
echo_load_policy leaves for the bf16 blob the oracle (oracle/quant.py) dequantises from the same bytes."""
import numpy as np
import pytest
import torch

from oracle import quant
from paper_2602_02192_amd import synth

from gpu_util import make_ctx

pytestmark = pytest.mark.gpu

MID = synth.ModelShape(2, 512, 8, 2, 128, 1024, 2048, dtype="bf16")
ODD = synth.ModelShape(2, 272, 4, 2, 64, 720, 1000, dtype="bf16")     # row and column counts that no tile of 32 x 128 divides
BIGV = synth.ModelShape(2, 1024, 8, 2, 128, 2048, 60000, dtype="bf16")  # embedding and lm_head go through the staging buffer in six batches of rows each


def tensors_of(s):
    return quant.tensor_list(s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn, s.vocab, s.qk_norm, s.tie_embeddings)


def roll(ctx, shape, seed=3):
    prompts, lens = synth.make_prompts(shape.vocab, 3, 20, seed=seed, ragged=True)
    prompts = np.maximum(prompts, 0)
    rng = np.random.default_rng(seed)
    forced = rng.integers(0, shape.vocab, size=(6, 5)).astype(np.int32)
    return ctx.rollout(prompts, lens, 2, 5, 1.0, 7, forced=forced, want_logits=True)


@pytest.mark.parametrize("shape", [MID, MID.replace(qk_norm=True, tie_embeddings=True), ODD, BIGV],
                         ids=["mid", "mid-qknorm-tied", "odd-sizes", "matrices-larger-than-the-staging-buffer"])
def test_q8_install_equals_the_install_of_the_dequantised_blob(shape):
    from paper_2602_02192_amd import echo
    q8 = synth.make_q8_weights(shape, 11)
    bits = quant.dequantize_q8(tensors_of(shape), q8)
    bf16 = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    a = make_ctx(shape, 6, 32, bf16)
    ref = roll(a, shape)
    a.close()
    b = make_ctx(shape, 6, 32)
    assert echo.q8_blob_bytes(b.desc) == q8.size == quant.q8_blob_bytes(tensors_of(shape))
    assert q8.size < 0.52 * echo.blob_bytes(b.desc)
    b.load_policy_q8(0, q8)
    got = roll(b, shape)
    assert np.isfinite(got["logits"]).all() and np.abs(got["logits"]).max() > 0.05
    assert np.array_equal(got["logits"], ref["logits"])
    assert np.array_equal(got["tokens"], ref["tokens"]) and np.array_equal(got["logprobs"], ref["logprobs"])
    # a second quantised snapshot over the first (one weight slot: in place), and back to a bf16 one
    q8b = synth.make_q8_weights(shape, 12)
    b.load_policy_q8(1, q8b)
    bits_b = quant.dequantize_q8(tensors_of(shape), q8b)
    got_b = roll(b, shape)
    assert not np.array_equal(got_b["logits"], ref["logits"])
    b.load_policy(2, bf16)
    assert np.array_equal(roll(b, shape)["logits"], ref["logits"])
    c = make_ctx(shape, 6, 32, torch.from_numpy(bits_b.view(np.int16).copy()).view(torch.bfloat16))
    assert np.array_equal(roll(c, shape)["logits"], got_b["logits"])
    c.close()
    # what it refuses: a wrong size, a version that does not advance
    with pytest.raises(echo.EchoError) as e:
        b.load_policy_q8(3, q8[:-1])
    assert e.value.code == echo.ECHO_EINVAL
    with pytest.raises(echo.EchoError) as e:
        b.load_policy_q8(2, q8)
    assert e.value.code == echo.ECHO_ESTATE
    b.load_policy_q8(3, q8)                       # and the context is still usable
    assert np.array_equal(roll(b, shape)["logits"], ref["logits"])
    b.close()


@pytest.mark.parametrize("shape", [MID.replace(qk_norm=True), ODD, BIGV], ids=["mid-qknorm", "odd-sizes", "matrices-larger-than-the-staging-buffer"])
def test_q8_blob_in_pieces_equals_the_one_call_install(shape):
    """The quantised blob through echo_load_policy_q8_begin / _chunk / _commit with cuts inside scales, inside rows of
    codes, inside gains and across several tensors: the same logits, bit for bit, as the one-call install; an aborted load
    leaves the old snapshot in place (two weight slots) and its version can be offered again."""
    from paper_2602_02192_amd import echo
    q8 = synth.make_q8_weights(shape, 21)
    a = make_ctx(shape, 6, 32)
    a.load_policy_q8(0, q8)
    ref = roll(a, shape)
    a.close()
    b = make_ctx(shape, 6, 32, slots=2)
    for v, cuts in enumerate(([1, 2, 3, 997, 40001, 5, 262147], [q8.size // 3 + 1], [7], [1 << 20])):
        if cuts == [7] and q8.size > 4e6:
            continue                                  # seven-byte pieces of the large blob would take minutes
        b.load_policy_q8_chunked(v, q8, cuts)
        assert np.array_equal(roll(b, shape)["logits"], ref["logits"]), cuts
    other = synth.make_q8_weights(shape, 22)
    b.load_policy_begin(10, echo.blob_bytes(b.desc))   # a bf16 load opened and dropped, then a quantised one dropped half-way
    b.load_policy_abort()
    assert echo.lib.echo_load_policy_q8_begin(b.h, 10, other.size) == 0
    assert echo.lib.echo_load_policy_chunk(b.h, other.ctypes.data, other.size // 2) == 0
    assert echo.lib.echo_load_policy_commit(b.h) == echo.ECHO_ESTATE          # not all bytes are in
    assert echo.lib.echo_load_policy_abort(b.h) == 0
    assert np.array_equal(roll(b, shape)["logits"], ref["logits"])
    b.load_policy_q8_chunked(10, other, [123457])
    assert not np.array_equal(roll(b, shape)["logits"], ref["logits"])
    b.close()


def test_q8_install_during_a_rollout_is_staged_and_switched_in():
    """Two weight slots: the quantised snapshot is installed from another thread while the rollout runs and is switched in
    at the pinned step; the tokens after the switch carry its version."""
    import threading
    import time
    shape = MID
    q8 = synth.make_q8_weights(shape, 5)
    ctx = make_ctx(shape, 8, 96, synth.make_weights(shape, 1), slots=2)
    prompts, lens = synth.make_prompts(shape.vocab, 2, 16, seed=2)
    box = {}
    t = threading.Thread(target=lambda: box.update(out=ctx.rollout(prompts, lens, 4, 60, 1.0, 3, swap_at_step=[30], swap_timeout_ms=20000)))
    t.start()
    for _ in range(2000):
        if ctx.stats().rollout_running:
            break
        time.sleep(0.002)
    ctx.load_policy_q8(9, q8)
    t.join(60)
    assert not t.is_alive() and "out" in box
    v = box["out"]["versions"]
    assert (v[:, :30] == 0).all() and (v[:, 30:] == 9).all()
    assert ctx.stats().active_version == 9
    ctx.close()


def test_q8_needs_a_bf16_model_on_the_mfma_path():
    from paper_2602_02192_amd import echo
    ctx = make_ctx(synth.TINY, 4, 32)
    assert echo.q8_blob_bytes(ctx.desc) == 0
    with pytest.raises(echo.EchoError) as e:
        ctx.load_policy_q8(0, np.zeros(16, np.uint8))
    assert e.value.code == echo.ECHO_EINVAL
    ctx.close()
    ctx = make_ctx(MID, 4, 32, debug_naive=True)
    with pytest.raises(echo.EchoError) as e:
        ctx.load_policy_q8(0, synth.make_q8_weights(MID, 1))
    assert e.value.code == echo.ECHO_EINVAL
    ctx.close()
