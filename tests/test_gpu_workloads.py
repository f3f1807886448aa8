"""GPU parity tests shaped like the larger workloads: wide batches (128 and 256 sequences) with ragged stop
lengths, a snapshot swap inside a rollout, teacher-forced scoring, edge cases, and the 4B-class shape in the
benchmark's launch configuration (sampled sequences against the oracle, the rest through properties)."""
import threading
import time

import numpy as np
import pytest

from oracle import oracle
from paper_2602_02192_amd import synth

from gpu_util import (BF16_LOGIT_TOL, BF16_LOGPROB_TOL, F32_LOGIT_TOL, F32_LOGPROB_TOL, NEAR_TIE_GAP,
                      check_argmax, check_tokens_fp32_sampler, make_ctx, oracle_rollout, valid_mask)

pytestmark = pytest.mark.gpu

MID = synth.ModelShape(2, 512, 8, 2, 128, 1024, 2048, dtype="bf16")


@pytest.mark.parametrize("n_prompts,G", [(16, 8), (32, 8), (5, 3), (40, 8)])
def test_wide_batches_with_ragged_stops_match_oracle(n_prompts, G):
    """128 and 256 sequences (the row counts of the 8B and the KV-heavy workloads), an odd 15 and 320: ragged
    prompts, per-sequence stop lengths, finished rows dropping out while the others go on.  With this shape's two KV
    heads the decode attention takes several rows per workgroup from 256 rows on: two at 256, and at 320 sets of two and
    three rows that straddle the groups of eight, re-dealt every step as sequences stop."""
    shape = MID
    N = n_prompts * G
    blob = synth.make_weights(shape, 3)
    blob32 = synth.widen_to_f32(blob)
    prompts, lens = synth.make_prompts(shape.vocab, n_prompts, 45, seed=6, ragged=True)
    prompts = np.maximum(prompts, 0)
    max_new = 10
    stop = synth.make_stop_lens(N, 1, max_new, seed=3)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=1.0, seed=5, stop_lens=stop,
                         want_logits=True)
    ctx = make_ctx(shape, N, 64, blob)
    tf = ctx.rollout(prompts, lens, G, max_new, 1.0, 5, stop_lens=stop, forced=np.maximum(ref["tokens"], 0), want_logits=True)
    assert np.array_equal(tf["lens"], ref["lens"]) and np.array_equal(tf["lens"], stop)
    m = valid_mask(ref["lens"], max_new)
    err = np.abs(tf["logits"] - ref["logits"])[m].max()
    assert err < BF16_LOGIT_TOL, err
    check_argmax(tf["logits"], ref["logits"], m, BF16_LOGIT_TOL, f"wide-{N}")
    same = (tf["tokens"] == ref["tokens"]) & m
    assert same[m].mean() > 0.9
    assert np.abs(tf["logprobs"] - ref["logprobs"])[same].max() < BF16_LOGPROB_TOL
    assert (tf["tokens"][~m] == -1).all() and (tf["logprobs"][~m] == 0).all()
    # the fused sampler agrees bit for bit with the fp32 sampler run on the same logits
    # (both with every row kept in place: moving the rows of the drained batch together changes the GEMM shapes, hence
    # the rounding of the logits)
    fused = ctx.rollout(prompts, lens, G, max_new, 1.0, 5, stop_lens=stop, forced=np.maximum(ref["tokens"], 0), no_compaction=True)
    assert np.array_equal(fused["tokens"], tf["tokens"])
    # the default: as sequences stop, the rows still generating are moved together (128 -> 64 -> 32 rows here) and the
    # step runs on the smaller batch; every sequence is still the oracle's
    comp = ctx.rollout(prompts, lens, G, max_new, 1.0, 5, stop_lens=stop, forced=np.maximum(ref["tokens"], 0))
    assert np.array_equal(comp["lens"], stop)
    same_c = (comp["tokens"] == ref["tokens"]) & m
    assert same_c[m].mean() > 0.9 and (comp["tokens"][~m] == -1).all()
    assert np.abs(comp["logprobs"] - ref["logprobs"])[same_c].max() < BF16_LOGPROB_TOL
    agree = (comp["tokens"] == fused["tokens"]) & m
    assert agree[m].mean() > 0.97 and np.abs(comp["logprobs"] - fused["logprobs"])[agree].max() < 2e-3
    if N > 32:
        assert ctx.rollout(prompts, lens, G, max_new, 1.0, 5, stop_lens=stop, eos_id=int(ref["tokens"][0, 0]))["lens"].max() <= max_new
    # free running: valid tokens, log-probs of a distribution, group members share the first step's distribution
    free = ctx.rollout(prompts, lens, G, max_new, 1.0, 5, stop_lens=stop)
    assert np.array_equal(free["lens"], stop)
    mm = valid_mask(free["lens"], max_new)
    assert ((free["tokens"][mm] >= 0) & (free["tokens"][mm] < shape.vocab)).all() and (free["logprobs"][mm] <= 0).all()
    assert np.array_equal(free["tokens"][:, 0], tf["tokens"][:, 0])
    ctx.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_snapshot_swap_inside_a_rollout(dtype):
    """A second snapshot is installed from another thread while the rollout runs and is switched in at a
    pinned step: earlier steps are those of A, later ones those of B on A's KV cache; versions are tagged."""
    shape = synth.TINY.replace(dtype=dtype)
    A, B = synth.make_weights(shape, 0), synth.make_weights(shape, 10)
    A32, B32 = synth.widen_to_f32(A), synth.widen_to_f32(B)
    prompts, lens = synth.make_prompts(shape.vocab, 4, 16, seed=1)
    k, max_new = 5, 12
    ref = oracle_rollout(shape, [A32, B32], prompts, lens, G=2, max_new=max_new, temperature=1.0, seed=2, versions=[3, 8],
                         swap_at_step=[k], want_logits=True)
    ctx = make_ctx(shape, 8, 32, A, version=3, slots=2)
    box = {}

    def run():
        box["out"] = ctx.rollout(prompts, lens, 2, max_new, 1.0, 2, swap_at_step=[k], swap_timeout_ms=20000, forced=ref["tokens"],
                                 want_logits=True)

    t = threading.Thread(target=run)
    t.start()
    for _ in range(2000):           # once the rollout is inside its loop a new snapshot is staged, not activated
        if ctx.stats().rollout_running:
            break
        time.sleep(0.005)
    assert ctx.stats().rollout_running
    ctx.load_policy(8, B)
    t.join(60)
    assert not t.is_alive() and "out" in box
    out = box["out"]
    tol = F32_LOGIT_TOL if dtype == "fp32" else BF16_LOGIT_TOL
    assert np.abs(out["logits"] - ref["logits"]).max() < tol
    assert (out["versions"][:, :k] == 3).all() and (out["versions"][:, k:] == 8).all()
    assert np.array_equal(out["versions"], ref["versions"])
    assert np.abs(out["logits"][:, k:] - oracle_rollout(shape, A32, prompts, lens, G=2, max_new=max_new, temperature=1.0, seed=2,
                                                         forced=ref["tokens"], want_logits=True)["logits"][:, k:]).max() > 1e-2
    if dtype == "fp32":
        check_tokens_fp32_sampler(out["tokens"], ref)
    st = ctx.stats()
    assert st.active_version == 8 and st.staged_version == -1
    # versions only advance; a rollout that pins a swap nobody stages gives up with a message
    from paper_2602_02192_amd import echo
    with pytest.raises(echo.EchoError) as e:
        ctx.load_policy(8, A)
    assert e.value.code == echo.ECHO_ESTATE
    with pytest.raises(echo.EchoError) as e:
        ctx.rollout(prompts, lens, 2, 4, 1.0, 2, swap_at_step=[2], swap_timeout_ms=50)
    assert e.value.code == echo.ECHO_ESTATE
    ctx.close()


@pytest.mark.parametrize("shape", [synth.TINY, MID], ids=["tiny-fp32", "mid-bf16"])
def test_teacher_forced_scoring_matches_oracle_and_the_rollout(shape):
    blob = synth.make_weights(shape, 0)
    blob32 = synth.widen_to_f32(blob)
    orc = oracle.load("f64")
    d = oracle.desc_from_shape(shape)
    prompts, lens = synth.make_prompts(shape.vocab, 3, 20, seed=1, ragged=True)
    prompts = np.maximum(prompts, 0)
    ctx = make_ctx(shape, 6, 64, blob)
    out = ctx.rollout(prompts, lens, 2, 9, 0.8, 4)
    # whole strings (prompt + generated), right padded
    T = 20 + 9
    toks = np.zeros((6, T), np.int32)
    tl = np.zeros(6, np.int32)
    for n in range(6):
        p = n // 2
        s = np.concatenate([prompts[p, :lens[p]], out["tokens"][n, :out["lens"][n]]])
        toks[n, :s.size] = s
        tl[n] = s.size
    got = ctx.logprobs(toks, tl, 0.8)
    tol = F32_LOGPROB_TOL if shape.dtype == "fp32" else BF16_LOGPROB_TOL
    for n in range(6):
        want = orc.logprobs(d, blob32, toks[n, :tl[n]], 0.8)
        assert np.abs(got[n, :tl[n]] - want).max() < tol
        assert got[n, 0] == 0 and (got[n, tl[n]:] == 0).all()
        # the sampler's own log-probs are the scores of its tokens (what the importance ratio divides by)
        p = n // 2
        assert np.abs(got[n, lens[p]:tl[n]] - out["logprobs"][n, :out["lens"][n]]).max() < tol
    ctx.close()


@pytest.mark.parametrize("heads", [(8, 1, 128), (8, 2, 128), (4, 4, 64), (4, 2, 64), (2, 2, 128)],
                         ids=lambda h: "Hq%d-Hkv%d-hd%d" % h)
def test_causal_block_attention_scores_every_position_like_the_oracle(heads):
    """Teacher-forced scoring of ragged strings that span several key tiles and several row blocks, with block
    boundaries that fall inside a pass of rows shared by consecutive strings: every position's log-prob is compared."""
    Hq, Hkv, hd = heads
    shape = synth.ModelShape(2, 256, Hq, Hkv, hd, 512, 1024, dtype="bf16", qk_norm=(hd == 64))
    blob = synth.make_weights(shape, 11)
    blob32 = synth.widen_to_f32(blob)
    orc = oracle.load("f64")
    d = oracle.desc_from_shape(shape)
    tl = np.array([1, 203, 2, 97, 33, 64, 131, 7], np.int32)
    rng = np.random.default_rng(5)
    toks = rng.integers(0, shape.vocab, size=(tl.size, int(tl.max()))).astype(np.int32)
    ctx = make_ctx(shape, 8, 224, blob)
    got = ctx.logprobs(toks, tl, 0.9)
    for n in range(tl.size):
        want = orc.logprobs(d, blob32, toks[n, :tl[n]], 0.9)
        assert np.abs(got[n, :tl[n]] - want).max() < BF16_LOGPROB_TOL, n
        assert (got[n, tl[n]:] == 0).all()
    ctx.close()


def test_full_4096_row_pass_with_wide_tiles_and_a_pass_boundary_matches_the_oracle():
    """Ten strings, 4306 rows: the first scoring pass is a full 4096 rows, which puts the QKV and gate/up projections
    on the 256 x 256-tile GEMM (256 and 128 tiles); one string straddles the pass boundary.  The short strings sit
    in different 256-row blocks of the pass and are compared with the oracle at every position."""
    shape = synth.ModelShape(2, 512, 16, 8, 128, 1024, 1024, dtype="bf16")
    blob = synth.make_weights(shape, 21)
    blob32 = synth.widen_to_f32(blob)
    orc = oracle.load("f64")
    d = oracle.desc_from_shape(shape)
    tl = np.array([128, 1000, 96, 1200, 64, 1300, 80, 178, 100, 160], np.int32)
    assert tl[:8].sum() == 4046 and tl.sum() == 4306
    rng = np.random.default_rng(9)
    toks = rng.integers(0, shape.vocab, size=(tl.size, int(tl.max()))).astype(np.int32)
    ctx = make_ctx(shape, tl.size, 1312, blob)
    got = ctx.logprobs(toks, tl, 1.0)
    assert np.isfinite(got).all()
    for n in (0, 2, 4, 6, 8, 9):
        want = orc.logprobs(d, blob32, toks[n, :tl[n]], 1.0)
        assert np.abs(got[n, :tl[n]] - want).max() < BF16_LOGPROB_TOL, n
    # the long strings: scoring twice in a different order (other row blocks, other passes) gives the same numbers
    order = np.array([5, 3, 1, 7, 0, 2, 4, 6, 9, 8])
    again = ctx.logprobs(toks[order], tl[order], 1.0)
    for i, n in enumerate(order):
        assert np.abs(again[i, :tl[n]] - got[n, :tl[n]]).max() < 2e-3, n
    ctx.close()


GRP8 = synth.ModelShape(2, 512, 16, 2, 64, 1024, 2048, dtype="bf16")
GRP1 = synth.ModelShape(2, 256, 4, 4, 64, 512, 1024, dtype="bf16")      # one query head per KV head
GRP2 = synth.ModelShape(2, 512, 4, 2, 128, 1024, 1024, dtype="bf16")


@pytest.mark.parametrize("shape,G,P", [(MID, 8, 21), (GRP8, 8, 21), (MID, 3, 54), (MID, 4, 5), (GRP1, 5, 13), (GRP2, 8, 9)],
                         ids=["grp4-G8", "grp8-G8", "grp4-G3", "grp4-G4-keys-split-over-workgroups", "grp1-G5", "grp2-G8"])
def test_group_shared_prompt_tiles(shape, G, P):
    """Decode attention reads the whole 32-key tiles of a prompt from the group's first cache slot (three cases with
    enough rows that every row's keys stay in one workgroup, one small batch whose keys are split over workgroups).  Prompt lengths below, at and between tile boundaries;
    sequences of a group stop at different lengths."""
    blob = synth.make_weights(shape, 5)
    prompts, lens = synth.make_prompts(shape.vocab, P, 100, seed=8)
    lens[:] = np.resize(np.array([31, 32, 33, 64, 100, 7, 96], np.int32), P)
    N, max_new = P * G, 40
    stop = np.resize(np.array([3, 40, 17, 29, 40, 1, 36, 22], np.int32), N)
    ctx = make_ctx(shape, N, 160, blob)
    # 1. every row reading the group's copy of the prompt tiles itself against every row reading its own replicated copy:
    # bit for bit (same kernel, same order of operations, other addresses)
    a = ctx.rollout(prompts, lens, G, max_new, 1.0, 11, stop_lens=stop, prefix_kernel=1)
    b = ctx.rollout(prompts, lens, G, max_new, 1.0, 11, stop_lens=stop, prefix_kernel=1, own_prompt_copy=True)
    assert np.array_equal(a["lens"], stop) and np.array_equal(b["lens"], stop)
    assert np.array_equal(a["tokens"], b["tokens"])
    assert np.array_equal(a["logprobs"], b["logprobs"])
    # 1b. the shared tiles attended once per group by the prefix kernel (the default where a row's keys stay in one
    # workgroup): the same sums in another order, so equal up to rounding -- fed the same tokens, the same tokens come out
    # (near-ties aside) with log-probs a rounding apart
    forced = np.maximum(a["tokens"], 0)
    af = ctx.rollout(prompts, lens, G, max_new, 1.0, 11, stop_lens=stop, forced=forced, prefix_kernel=1)
    pf = ctx.rollout(prompts, lens, G, max_new, 1.0, 11, stop_lens=stop, forced=forced, prefix_kernel=2)   # also for batches this small, where it does not pay
    m = valid_mask(stop, max_new)
    same = (pf["tokens"] == af["tokens"]) & m
    assert same[m].mean() > 0.995, same[m].mean()
    assert np.abs(pf["logprobs"] - af["logprobs"])[same].max() < 2e-3
    # 1c. decode workgroups that take several neighbouring rows and the prompt tiles those have in common once (the default
    # for batches that leave every compute unit a workgroup that way): groups of 3 straddle the workgroups' rows, a batch
    # that is no multiple of the rows per workgroup leaves the last one partly empty, and without compaction the
    # sequences that have stopped stay behind as idle rows between the others
    for nc in (False, True):
        rf = ctx.rollout(prompts, lens, G, max_new, 1.0, 11, stop_lens=stop, forced=forced, prefix_kernel=3, no_compaction=nc)
        assert np.array_equal(rf["lens"], stop)
        same = (rf["tokens"] == af["tokens"]) & m
        assert same[m].mean() > 0.995, same[m].mean()
        assert np.abs(rf["logprobs"] - af["logprobs"])[same].max() < 2e-3
    # 2. against the oracle, teacher-forced on the oracle's tokens, for three prompts spread over the batch
    blob32 = synth.widen_to_f32(blob)
    pick = [0, P // 2, P - 1]
    forced12 = np.zeros((N, 12), np.int32)
    refs = {}
    for p in pick:
        refs[p] = oracle_rollout(shape, blob32, prompts[p:p + 1], lens[p:p + 1], G=G, max_new=12, temperature=1.0, seed=11, want_logits=True)
        forced12[p * G:(p + 1) * G] = np.maximum(refs[p]["tokens"], 0)
    for pk in (2, 3):
        tf = ctx.rollout(prompts, lens, G, 12, 1.0, 11, forced=forced12, want_logits=True, prefix_kernel=pk)
        for p in pick:
            assert np.abs(tf["logits"][p * G:(p + 1) * G] - refs[p]["logits"]).max() < BF16_LOGIT_TOL, (pk, p)
    ctx.close()


@pytest.mark.parametrize("shape,top_p,temperature", [(synth.TINY, 0.9, 1.0), (synth.TINY, 0.3, 0.7), (MID, 0.95, 1.0)],
                         ids=["tiny-fp32-p0.9", "tiny-fp32-p0.3-T0.7", "mid-bf16-p0.95"])
def test_nucleus_sampling_matches_the_oracle(shape, top_p, temperature):
    """top_p < 1: teacher-forced on the oracle's own nucleus rollout, so every step's draw is compared on its own.
    Where the oracle's cut is not within rounding of top_p and its draw is no near-tie, the all-fp32 path returns the
    oracle's token; log-probs are those of the renormalised kept set.  The sampled token is always inside the kept set
    that the returned logits define, and its log-prob is its renormalised log-probability there."""
    blob = synth.make_weights(shape, 2)
    blob32 = synth.widen_to_f32(blob)
    P, G, max_new = 3, 4, 10
    prompts, lens = synth.make_prompts(shape.vocab, P, 24, seed=6, ragged=True)
    prompts = np.maximum(prompts, 0)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=temperature, seed=13, top_p=top_p,
                         want_logits=True)
    ctx = make_ctx(shape, P * G, 24 + max_new, blob)
    got = ctx.rollout(prompts, lens, G, max_new, temperature, 13, top_p=top_p, forced=ref["tokens"], want_logits=True)
    again = ctx.rollout(prompts, lens, G, max_new, temperature, 13, top_p=top_p, forced=ref["tokens"])
    assert np.array_equal(got["tokens"], again["tokens"]) and np.array_equal(got["logprobs"], again["logprobs"])
    fp32 = shape.dtype == "fp32"
    assert np.abs(got["logits"] - ref["logits"]).max() < (F32_LOGIT_TOL if fp32 else BF16_LOGIT_TOL)
    clear = (ref["margins"] > 1e-4) & (ref["gaps"] > NEAR_TIE_GAP)
    same = got["tokens"] == ref["tokens"]
    if fp32:
        assert clear.mean() > 0.5 and same[clear].all()      # near-uniform p over 1024 tokens: a fifth of the cuts sit within 1e-4
        assert np.abs(got["logprobs"] - ref["logprobs"])[same & clear].max() < F32_LOGPROB_TOL
    else:
        assert same.mean() > 0.8
        assert np.abs(got["logprobs"] - ref["logprobs"])[same].max() < BF16_LOGPROB_TOL
    # self-consistency on the GPU's own logits (fp64 arithmetic here): token inside the kept set, log-prob renormalised
    T32 = float(np.float32(temperature))
    for n in range(P * G):
        for s in range(max_new):
            z = got["logits"][n, s].astype(np.float64) / T32
            p = np.exp(z - z.max())
            p /= p.sum()
            order = np.lexsort((np.arange(p.size), -p))
            cum = np.cumsum(p[order])
            k = int(np.argmax(cum >= top_p)) + 1
            tok = int(got["tokens"][n, s])
            pos = int(np.nonzero(order == tok)[0][0])
            slack = 1e-4                                  # the kernel sums quantised fp32 masses: the cut may sit a hair off
            k_lo = int(np.argmax(cum >= top_p - slack)) + 1
            k_hi = int(np.argmax(cum >= min(top_p + slack, cum[-1]))) + 1
            assert pos < k_hi, (n, s)
            lo, hi = np.log(p[tok] / cum[k_hi - 1]), np.log(p[tok] / cum[k_lo - 1])
            assert lo - 2e-4 <= got["logprobs"][n, s] <= hi + 2e-4, (n, s, k, got["logprobs"][n, s], lo, hi)
    # top_p = 1 through the same unfused path is the plain sampler
    a = ctx.rollout(prompts, lens, G, max_new, temperature, 13, unfused_sampler=True)
    b = ctx.rollout(prompts, lens, G, max_new, temperature, 13)
    if fp32:
        assert np.array_equal(a["tokens"], b["tokens"])
    ctx.close()


@pytest.mark.parametrize("shape", [synth.TINY, MID], ids=["tiny-fp32-V1024", "mid-bf16-V2048"])
def test_nucleus_cut_inside_exact_ties(shape):
    """A zero lm_head makes every logit exactly 0: all V tokens tie, the kept set is the lowest ceil(top_p * V) indices
    (lower index first among equals), every kept token has probability 1/k, and the token is the kept index with the
    largest uniform draw -- the oracle and the GPU must agree on every token.  V = 1024 resolves the ties through the
    index list, V = 2048 through the scan over contiguous runs; the cut's last radix round takes its 1024 keys from the
    candidate list that the round before filled (exactly full), and with 2048 candidates walks the row instead."""
    blob = synth.make_weights(shape, 4)
    off, shp = synth.blob_offsets(shape)["lm_head"]
    blob[off:off + int(np.prod(shp))] = 0
    blob32 = synth.widen_to_f32(blob)
    prompts, lens = synth.make_prompts(shape.vocab, 2, 9, seed=3)
    top_p, G, max_new = 0.3, 3, 6
    k = int(np.ceil(np.float32(top_p) * shape.vocab))
    ref = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=1.0, seed=21, top_p=top_p)
    assert (ref["tokens"] < k).all() and np.allclose(ref["logprobs"], -np.log(k))
    ctx = make_ctx(shape, 2 * G, 9 + max_new, blob)
    got = ctx.rollout(prompts, lens, G, max_new, 1.0, 21, top_p=top_p)
    assert np.array_equal(got["tokens"], ref["tokens"])
    assert np.abs(got["logprobs"] + np.log(k)).max() < 1e-5
    ctx.close()


def test_edge_cases_and_errors():
    from paper_2602_02192_amd import echo
    shape = synth.TINY
    blob = synth.make_weights(shape, 0)
    blob32 = synth.widen_to_f32(blob)
    ctx = make_ctx(shape, 8, 64)
    prompts, lens = synth.make_prompts(shape.vocab, 1, 1, seed=1)
    with pytest.raises(echo.EchoError) as e:            # no snapshot yet
        ctx.rollout(prompts, lens, 1, 1, 1.0, 0)
    assert e.value.code == echo.ECHO_ESTATE
    ctx.load_policy(0, blob)
    # smallest rollout: one prompt of one token, one sample, one new token
    out = ctx.rollout(prompts, lens, 1, 1, 1.0, 0, want_logits=True)
    ref = oracle_rollout(shape, blob32, prompts, lens, G=1, max_new=1, temperature=1.0, seed=0, want_logits=True)
    assert np.abs(out["logits"] - ref["logits"]).max() < F32_LOGIT_TOL and out["lens"][0] == 1
    check_tokens_fp32_sampler(out["tokens"], ref)
    # capacity: exactly max_seqs sequences and prompt + max_new == max_ctx are accepted, one more is not
    prompts, lens = synth.make_prompts(shape.vocab, 4, 40, seed=2)
    full = ctx.rollout(prompts, lens, 2, 24, 1.0, 1)
    assert (full["lens"] == 24).all()
    for bad in (lambda: ctx.rollout(prompts, lens, 3, 24, 1.0, 1), lambda: ctx.rollout(prompts, lens, 2, 25, 1.0, 1)):
        with pytest.raises(echo.EchoError) as e:
            bad()
        assert e.value.code == echo.ECHO_ENOMEM
    # argument checks
    for bad in (lambda: ctx.rollout(prompts, lens, 2, 4, 0.0, 1), lambda: ctx.rollout(prompts, lens, 2, 4, 1.0, 1, top_p=0.0),
                lambda: ctx.rollout(prompts, lens, 2, 4, 1.0, 1, top_p=1.5),
                lambda: ctx.rollout(prompts + shape.vocab, lens, 2, 4, 1.0, 1), lambda: ctx.rollout(prompts, lens * 0, 2, 4, 1.0, 1)):
        with pytest.raises(echo.EchoError) as e:
            bad()
        assert e.value.code == echo.ECHO_EINVAL
    # EOS: a sequence ends with the EOS token it emitted; the oracle agrees on where
    eos = int(full["tokens"][0, 3])
    ref = oracle_rollout(shape, blob32, prompts, lens, G=2, max_new=24, temperature=1.0, seed=1, eos_id=eos)
    got = ctx.rollout(prompts, lens, 2, 24, 1.0, 1, eos_id=eos)
    if check_tokens_fp32_sampler(got["tokens"], ref, mask=valid_mask(np.minimum(got["lens"], ref["lens"]), 24)) == 0:
        assert np.array_equal(got["lens"], ref["lens"])
    assert got["lens"][0] <= 4 and got["tokens"][0, got["lens"][0] - 1] == eos
    # the low-temperature limit picks the arg-max token
    cold = ctx.rollout(prompts, lens, 2, 3, 1e-4, 1, want_logits=True)
    assert np.array_equal(cold["tokens"][:, 0], cold["logits"][:, 0].argmax(-1))
    # a different seed draws different tokens; the same seed repeats them
    assert not np.array_equal(ctx.rollout(prompts, lens, 2, 24, 1.0, 9)["tokens"], full["tokens"])
    assert np.array_equal(ctx.rollout(prompts, lens, 2, 24, 1.0, 1)["tokens"], full["tokens"])
    ctx.close()


def test_dense4b_shape_in_the_benchmark_launch_configuration():
    """The 4B-class decoder (36 layers, full width, vocabulary 151936), 8 prompts x G = 8 = 64 sequences as the
    benchmark launches it.  The oracle is affordable for two whole sequences with a short prompt; the long
    configuration (prompt 512 + 1024 new tokens) is checked through properties and self-consistency."""
    import torch
    shape = synth.DENSE_4B
    blob_dev = synth.make_weights(shape, 0, device="cuda")
    blob = torch.empty(blob_dev.shape, dtype=blob_dev.dtype, pin_memory=True)
    blob.copy_(blob_dev)
    del blob_dev
    torch.cuda.empty_cache()
    blob32 = synth.widen_to_f32(blob)
    P, G, N = 8, 8, 64
    ctx = make_ctx(shape, N, 512 + 1024, blob)

    # -- sampled sequences against the oracle: short prompts, 6 teacher-forced steps, sequences 0 and 63
    prompts, lens = synth.make_prompts(shape.vocab, P, 12, seed=1)
    max_new = 6
    refs = {}
    for p in (0, 7):
        refs[p] = oracle_rollout(shape, blob32, prompts[p:p + 1], lens[p:p + 1], G=1, max_new=max_new, temperature=1.0, seed=2,
                                 want_logits=True)
    forced = np.zeros((N, max_new), np.int32)
    rng = np.random.default_rng(0)
    forced[:] = rng.integers(0, shape.vocab, size=(N, max_new))
    forced[0], forced[63] = refs[0]["tokens"][0], refs[7]["tokens"][0]
    # the oracle's sequence n=0 of a one-prompt rollout uses stream id 0; sequence 63 of the batch uses 63, so only
    # logits (which do not depend on the stream) are compared for it, tokens and log-probs for sequence 0
    out = ctx.rollout(prompts, lens, G, max_new, 1.0, 2, forced=forced)
    d = ctx.desc
    unf = ctx.rollout(prompts, lens, G, max_new, 1.0, 2, forced=forced, unfused_sampler=True)
    assert np.array_equal(out["tokens"], unf["tokens"])                      # fused sampler == fp32 sampler on the same logits
    assert np.abs(out["logprobs"] - unf["logprobs"]).max() < 1e-4
    lg = ctx.rollout(prompts[[0, 7]], lens[[0, 7]], 1, max_new, 1.0, 2, forced=np.stack([forced[0], forced[63]]), want_logits=True)
    for i, p in enumerate((0, 7)):
        err = np.abs(lg["logits"][i] - refs[p]["logits"][0]).max()
        assert err < BF16_LOGIT_TOL, (p, err)
        check_argmax(lg["logits"][i:i + 1], refs[p]["logits"], np.ones((1, max_new), bool), BF16_LOGIT_TOL, f"dense4b-seq{p}")
    same = out["tokens"][0] == refs[0]["tokens"][0]
    assert same.mean() >= 0.8
    assert np.abs(out["logprobs"][0] - refs[0]["logprobs"][0])[same].max() < BF16_LOGPROB_TOL
    # rows of the 64-row batch against the same sequences run in a batch of two: other launch shapes (other K splits of the
    # projections), so other rounding -- two paths that each sit within the tolerance of the exact value (at 36 layers
    # either is about 0.002 rms away from it)
    dlp = np.abs(lg["logprobs"][0] - out["logprobs"][0])[lg["tokens"][0] == out["tokens"][0]]
    print(f"[dense4b, batch of 64 against batch of 2] |dlogprob| max {dlp.max():.4f} mean {dlp.mean():.4f}")
    assert dlp.max() < 2 * BF16_LOGPROB_TOL and dlp.mean() < 0.3 * BF16_LOGPROB_TOL, (dlp.max(), dlp.mean())

    # -- the continuous entry point on the same shape: 16 prompts through the 64 cache slots, so the second eight are
    # admitted as the first finish; sequence 0 against the oracle, the first 64 against the ordinary rollout above
    prompts16 = np.concatenate([prompts, synth.make_prompts(shape.vocab, P, 12, seed=5)[0]])
    lens16 = np.concatenate([lens, lens])
    forced16 = np.concatenate([forced, forced[::-1]])
    stop16 = synth.make_stop_lens(2 * N, 3, max_new, seed=7)
    stop16[0] = max_new
    cont = ctx.rollout(prompts16, lens16, G, max_new, 1.0, 2, forced=forced16, stop_lens=stop16, continuous=True)
    assert np.array_equal(cont["lens"], stop16)
    same = cont["tokens"][0] == refs[0]["tokens"][0]
    assert same.mean() >= 0.8 and np.abs(cont["logprobs"][0] - refs[0]["logprobs"][0])[same].max() < BF16_LOGPROB_TOL
    m64 = valid_mask(stop16[:N], max_new)
    agree = (cont["tokens"][:N] == out["tokens"]) & m64
    assert agree[m64].mean() > 0.97                                   # same streams, same forced inputs: near-ties aside
    assert np.abs(cont["logprobs"][:N] - out["logprobs"])[agree].max() < 2 * BF16_LOGPROB_TOL
    assert (cont["tokens"][N:][valid_mask(stop16[N:], max_new)] >= 0).all() and np.isfinite(cont["logprobs"]).all()

    # -- the benchmark's prompt length against the oracle, inside the 64-row batch: sequence 0 with its 512-token prompt
    # and 8 teacher-forced steps (the oracle's stream id 0 is the batch's, so tokens and log-probs compare too); once with
    # every row reading the group's 16 shared prompt tiles itself, once with the once-per-group kernel attending them, once
    # the way the benchmark runs (0: two neighbouring rows and their common prompt tiles per decode workgroup)
    prompts, lens = synth.make_prompts(shape.vocab, P, 512, seed=1)
    ref512 = oracle_rollout(shape, blob32, prompts[0:1], lens[0:1], G=1, max_new=8, temperature=1.0, seed=2, want_logits=True)
    forced8 = rng.integers(0, shape.vocab, size=(N, 8)).astype(np.int32)
    forced8[0] = ref512["tokens"][0]
    for pk in (0, 1, 2):
        tf = ctx.rollout(prompts, lens, G, 8, 1.0, 2, forced=forced8, want_logits=True, prefix_kernel=pk)
        err = float(np.abs(tf["logits"][0] - ref512["logits"][0]).max())
        print(f"[dense4b, 512-token prompt, prefix_kernel={pk}] max |dlogit| = {err:.4f}")
        assert err < BF16_LOGIT_TOL, (pk, err)
        check_argmax(tf["logits"][0:1], ref512["logits"], np.ones((1, 8), bool), BF16_LOGIT_TOL, f"dense4b-512-pk{pk}")
        del tf
        fused = ctx.rollout(prompts, lens, G, 8, 1.0, 2, forced=forced8, prefix_kernel=pk)     # graph replay, fused sampler
        same = fused["tokens"][0] == ref512["tokens"][0]
        assert same.mean() >= 0.75
        assert np.abs(fused["logprobs"][0] - ref512["logprobs"][0])[same].max() < BF16_LOGPROB_TOL
    del blob32

    # -- the benchmark's own configuration: prompt 512, 1024 new tokens, graph replay
    big = ctx.rollout(prompts, lens, G, 1024, 1.0, 2)
    assert (big["lens"] == 1024).all() and (big["versions"] == 0).all()
    assert ((big["tokens"] >= 0) & (big["tokens"] < shape.vocab)).all()
    lp = big["logprobs"]
    assert (lp <= 0).all() and np.isfinite(lp).all()
    # near-uniform policy on random weights: log-probs sit around -ln V - sigma^2/2 .. , far from 0 and from -inf
    assert -16.0 < lp.mean() < -9.0
    # the G samples of a prompt draw their first token from one distribution; later tokens differ
    first = big["tokens"][:, 0].reshape(P, G)
    assert (np.array([len(set(r)) for r in first]) >= G - 1).all()
    assert len({tuple(r) for r in big["tokens"][:, :8]}) == N
    # self-consistency over the full length: scoring a rollout's own tokens reproduces the sampler's log-probs
    for n in (0, 37):
        s = np.concatenate([prompts[n // G], big["tokens"][n]])[None, :]
        got = ctx.logprobs(s, np.array([s.shape[1]], np.int32), 1.0)[0, 512:]
        # two paths (decode kernels, causal block kernels) that each sit within the tolerance of the exact value
        assert np.abs(got - lp[n]).max() < 2 * BF16_LOGPROB_TOL
        assert np.abs(got - lp[n]).mean() < 0.3 * BF16_LOGPROB_TOL
    # the groups' 512-token prompts attended once per group by the prefix kernel (forced on; off by default at this size):
    # the same tokens fed in, the same tokens out (near-ties aside), log-probs a rounding apart
    px = ctx.rollout(prompts, lens, G, 64, 1.0, 2, forced=big["tokens"][:, :64], prefix_kernel=2)
    same = px["tokens"] == big["tokens"][:, :64]
    dlp = np.abs(px["logprobs"] - big["logprobs"][:, :64])[same]
    # two paths that each sit within the tolerance of the exact value (36 layers amplify the other summation order)
    assert same.mean() > 0.995 and dlp.max() < 2 * BF16_LOGPROB_TOL and dlp.mean() < 0.3 * BF16_LOGPROB_TOL, (dlp.max(), dlp.mean())
    # kernel-by-kernel launches reproduce the graph replay bit for bit (same kernels, same order)
    ng = ctx.rollout(prompts, lens, G, 64, 1.0, 2, no_graph=True)
    assert np.array_equal(ng["tokens"], big["tokens"][:, :64]) and np.array_equal(ng["logprobs"], big["logprobs"][:, :64])
    ctx.close()


@pytest.mark.parametrize("no_graph", [False, True])
def test_draining_batch_with_eos_and_stop_lengths_is_compacted_and_matches_the_oracle(no_graph):
    """40 sequences on the all-fp32 path, ended by stop lengths and by an end-of-sequence token: the batch drains below 32
    rows (the host learns of EOS endings every 16 steps), rows are moved together, and every sequence still draws the
    oracle's tokens (its draws are keyed by its sequence index wherever its row has moved)."""
    shape = synth.TINY
    blob = synth.make_weights(shape, 0)
    blob32 = synth.widen_to_f32(blob)
    P, G, max_new = 10, 4, 96
    prompts, lens = synth.make_prompts(shape.vocab, P, 12, seed=3)
    stop = synth.make_stop_lens(P * G, 1, max_new, seed=4)
    stop[:6] = max_new                                    # some run to the end
    probe = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=1.0, seed=9, stop_lens=stop)
    vals, counts = np.unique(probe["tokens"][probe["tokens"] >= 0], return_counts=True)
    eos = int(vals[counts.argmax()])                      # a token that does occur
    ref = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=1.0, seed=9, stop_lens=stop, eos_id=eos)
    assert (ref["lens"] < stop).any()                     # EOS does end sequences early
    ctx = make_ctx(shape, P * G, 12 + max_new, blob)
    got = ctx.rollout(prompts, lens, G, max_new, 1.0, 9, stop_lens=stop, eos_id=eos, no_graph=no_graph)
    keep = ctx.rollout(prompts, lens, G, max_new, 1.0, 9, stop_lens=stop, eos_id=eos, no_graph=no_graph, no_compaction=True)
    for k in ("tokens", "lens", "versions"):              # fp32 debug kernels: row position does not change a row's arithmetic
        assert np.array_equal(got[k], keep[k]), k
    assert np.array_equal(got["logprobs"], keep["logprobs"])
    m = valid_mask(np.minimum(got["lens"], ref["lens"]), max_new)
    if check_tokens_fp32_sampler(got["tokens"], ref, mask=m) == 0:
        assert np.array_equal(got["lens"], ref["lens"])
        assert np.abs(got["logprobs"] - ref["logprobs"])[m].max() < F32_LOGPROB_TOL
    mm = valid_mask(got["lens"], max_new)
    assert (got["tokens"][~mm] == -1).all() and (got["logprobs"][~mm] == 0).all() and (got["versions"][~mm] == -1).all()
    ctx.close()
