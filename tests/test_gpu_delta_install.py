"""Delta install: a snapshot given as byte ranges over the newest installed one must leave exactly what a full install
of the patched blob leaves (the blob is patched on the CPU; the oracle rolls the patched model out), with one weight
slot (patched in place) and with two (the other slot becomes a copy of the base first), also while a rollout decodes."""
import threading
import time

import numpy as np
import pytest

from paper_2602_02192_amd import synth

from gpu_util import BF16_LOGIT_TOL, F32_LOGIT_TOL, make_ctx, oracle_rollout

pytestmark = pytest.mark.gpu

MID = synth.ModelShape(2, 512, 8, 2, 128, 1024, 2048, dtype="bf16")


def as_bytes(blob):
    import torch
    return blob.contiguous().view(torch.uint8).numpy()


def make_delta(shape, base, other, seed, n_ranges=9):
    """Ranges of odd sizes scattered over the blob (inside elements' rows, across tensor borders, one inside a norm gain,
    one whole matrix), filled from `other`; returns (offsets, sizes, data, patched blob)."""
    import torch
    elt = 4 if shape.dtype == "fp32" else 2
    a, b = as_bytes(base), as_bytes(other)
    rng = np.random.default_rng(seed)
    offs_tab = synth.blob_offsets(shape)
    spans = []
    o, shp = offs_tab["layers.0.wq"]
    spans.append((o * elt + 3 * elt, 5 * elt))                                   # five values inside one row
    spans.append(((o + shp[1] - 2) * elt, 7 * elt))                              # across a row border
    o2, shp2 = offs_tab["layers.1.w_gate"]
    spans.append((o2 * elt, int(np.prod(shp2)) * elt))                           # a whole matrix
    o3, shp3 = offs_tab["layers.1.w_up"]
    spans.append(((o3 + 11) * elt, (3 * shp3[1] + 5) * elt))                     # three rows and a bit, unaligned start
    o4, _ = offs_tab["layers.0.ffn_norm"]
    spans.append(((o4 - 9) * elt, 40 * elt))                                     # end of a matrix, a gain, start of the next
    o5, _ = offs_tab["final_norm"]
    spans.append(((o5 - 1000) * elt, 3000 * elt))                                # last matrix, final gain, lm_head (or the blob's end)
    o6, shp6 = offs_tab["embed"]
    spans.append((17 * shp6[1] * elt + elt, 2 * shp6[1] * elt))                  # embedding rows (also the lm_head when tied)
    total = a.size
    for _ in range(n_ranges - len(spans)):
        off = int(rng.integers(0, total // elt - 5000)) * elt
        spans.append((off, int(rng.integers(1, 4000)) * elt))
    spans = sorted((min(o, total - elt), s) for o, s in spans)
    merged = []
    for o, s in spans:                                                             # ascending, non-overlapping
        s = min(s, total - o)
        if merged and o < merged[-1][0] + merged[-1][1]:
            continue
        merged.append((o, s))
    patched = a.copy()
    data = []
    for o, s in merged:
        patched[o:o + s] = b[o:o + s]
        data.append(b[o:o + s])
    pt = torch.from_numpy(patched.copy()).view(base.dtype)
    return np.array([m[0] for m in merged], np.uint64), np.array([m[1] for m in merged], np.uint64), np.concatenate(data), pt


@pytest.mark.parametrize("shape,slots", [(synth.TINY, 1), (synth.TINY.replace(dtype="bf16"), 2), (MID.replace(qk_norm=True), 1),
                                         (MID.replace(tie_embeddings=True), 2), (MID, 2)],
                         ids=["tiny-fp32-inplace", "tiny-bf16-2slots", "mid-qknorm-inplace", "mid-tied-2slots", "mid-2slots"])
def test_delta_leaves_the_snapshot_of_the_patched_blob(shape, slots):
    base, other = synth.make_weights(shape, 4, gain_jitter=0.1), synth.make_weights(shape, 14, gain_jitter=0.1)
    offsets, sizes, data, patched = make_delta(shape, base, other, seed=1)
    assert len(offsets) >= 7 and not np.array_equal(as_bytes(patched), as_bytes(base))
    prompts, lens = synth.make_prompts(shape.vocab, 3, 20, seed=1)
    whole = make_ctx(shape, 8, 64, patched, version=7)
    want = whole.rollout(prompts, lens, 2, 10, 1.0, 5, want_logits=True)
    whole.close()
    ctx = make_ctx(shape, 8, 64, base, version=3, slots=slots)
    before = ctx.rollout(prompts, lens, 2, 10, 1.0, 5, want_logits=True)
    assert not np.array_equal(before["logits"], want["logits"])
    ctx.load_policy_delta(3, 7, offsets, sizes, data)
    st = ctx.stats()
    assert st.active_version == 7 and st.staged_version == -1
    got = ctx.rollout(prompts, lens, 2, 10, 1.0, 5, want_logits=True)
    for k in ("tokens", "logprobs", "logits", "lens", "versions"):
        assert np.array_equal(got[k], want[k]), k
    # and the oracle on the patched blob
    ref = oracle_rollout(shape, synth.widen_to_f32(patched), prompts, lens, G=2, max_new=10, temperature=1.0, seed=5,
                         forced=got["tokens"], want_logits=True)
    assert np.abs(got["logits"] - ref["logits"]).max() < (F32_LOGIT_TOL if shape.dtype == "fp32" else BF16_LOGIT_TOL)
    # a second delta on top of the first (back to the base's bytes in the same ranges), and an empty one
    ctx.load_policy_delta(7, 8, offsets, sizes, np.concatenate([as_bytes(base)[int(o):int(o + s)] for o, s in zip(offsets, sizes)]))
    again = ctx.rollout(prompts, lens, 2, 10, 1.0, 5, want_logits=True)
    assert np.array_equal(again["logits"], before["logits"]) and (again["versions"] == 8).all()
    ctx.load_policy_delta(8, 9, [], [], np.zeros(0, np.uint8))
    assert np.array_equal(ctx.rollout(prompts, lens, 2, 10, 1.0, 5, want_logits=True)["logits"], before["logits"])
    ctx.close()


def test_delta_states_and_argument_errors():
    from paper_2602_02192_amd import echo
    shape = synth.TINY.replace(dtype="bf16")
    base = synth.make_weights(shape, 0)
    nbytes = as_bytes(base).size
    ctx = make_ctx(shape, 8, 64)
    two = np.zeros(2, np.uint8)

    def err(fn, code):
        with pytest.raises(echo.EchoError) as e:
            fn()
        assert e.value.code == code, e.value

    err(lambda: ctx.load_policy_delta(0, 1, [0], [2], two), echo.ECHO_ESTATE)            # nothing installed yet
    ctx.load_policy(5, base)
    err(lambda: ctx.load_policy_delta(4, 6, [0], [2], two), echo.ECHO_ESTATE)            # not against the newest snapshot
    err(lambda: ctx.load_policy_delta(5, 5, [0], [2], two), echo.ECHO_ESTATE)            # version does not advance
    err(lambda: ctx.load_policy_delta(5, 6, [1], [2], two), echo.ECHO_EINVAL)            # inside an element
    err(lambda: ctx.load_policy_delta(5, 6, [0], [3], np.zeros(3, np.uint8)), echo.ECHO_EINVAL)
    err(lambda: ctx.load_policy_delta(5, 6, [nbytes - 2], [4], np.zeros(4, np.uint8)), echo.ECHO_EINVAL)   # past the end
    err(lambda: ctx.load_policy_delta(5, 6, [8, 4], [2, 2], np.zeros(4, np.uint8)), echo.ECHO_EINVAL)      # out of order
    err(lambda: ctx.load_policy_delta(5, 6, [4, 4], [4, 2], np.zeros(6, np.uint8)), echo.ECHO_EINVAL)      # overlapping
    ctx.load_policy_begin(6, nbytes)
    err(lambda: ctx.load_policy_delta(5, 7, [0], [2], two), echo.ECHO_ESTATE)            # another load is open
    ctx.load_policy_abort()
    assert ctx.stats().active_version == -1 or ctx.stats().active_version == 5
    ctx.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_delta_arrives_while_a_rollout_decodes(dtype):
    """Two slots: the delta is applied to a copy of the running snapshot while the rollout decodes and is switched in at
    the pinned step; steps before it are the base's, steps from it on the patched model's (oracle with both blobs)."""
    shape = synth.TINY.replace(dtype=dtype)
    base, other = synth.make_weights(shape, 0), synth.make_weights(shape, 10)
    offsets, sizes, data, patched = make_delta(shape, base, other, seed=2, n_ranges=40)
    prompts, lens = synth.make_prompts(shape.vocab, 4, 16, seed=1)
    k, max_new = 5, 12
    ref = oracle_rollout(shape, [synth.widen_to_f32(base), synth.widen_to_f32(patched)], prompts, lens, G=2, max_new=max_new,
                         temperature=1.0, seed=2, versions=[3, 8], swap_at_step=[k], want_logits=True)
    ctx = make_ctx(shape, 8, 32, base, version=3, slots=2)
    box = {}

    def run():
        box["out"] = ctx.rollout(prompts, lens, 2, max_new, 1.0, 2, swap_at_step=[k], swap_timeout_ms=30000, forced=ref["tokens"],
                                 want_logits=True)

    t = threading.Thread(target=run)
    t.start()
    for _ in range(4000):
        if ctx.stats().rollout_running:
            break
        time.sleep(0.002)
    assert ctx.stats().rollout_running
    ctx.load_policy_delta(3, 8, offsets, sizes, data)
    t.join(60)
    assert not t.is_alive() and "out" in box
    out = box["out"]
    assert np.abs(out["logits"] - ref["logits"]).max() < (F32_LOGIT_TOL if dtype == "fp32" else BF16_LOGIT_TOL)
    assert np.array_equal(out["versions"], ref["versions"])
    assert np.abs(out["logits"][:, k:] - oracle_rollout(shape, synth.widen_to_f32(base), prompts, lens, G=2, max_new=max_new,
                                                         temperature=1.0, seed=2, forced=ref["tokens"], want_logits=True)["logits"][:, k:]).max() > 1e-3
    ctx.close()
