"""GPU parity tests at the widths and depths of the larger workloads, against the fp64 oracle.

The oracle cannot afford the 8B- and 32B-class models whole, so each is cut one way at a time: full width (hidden size,
head grouping, feed-forward width, vocabulary 151936) at two layers, and full depth (64 layers) on a narrow model with
the 32B-class head grouping (8 query heads per key/value head, head_dim 128) and the full vocabulary.  Every case runs
in the batch sizes of its workload (64 and 128 rows; the 32B width also at 32 rows, where the gate/up projection takes its
widest workgroups); the oracle computes the first and the last sequence of the batch.
Also here: tied embeddings and per-head q/k norm on the decode path, operands beyond the half-precision range, and
snapshots installed back to back while a rollout keeps switching."""
import functools
import threading
import time

import numpy as np
import pytest

from oracle import oracle
from paper_2602_02192_amd import synth

from gpu_util import (BF16_LOGIT_TOL, BF16_LOGPROB_TOL, F32_LOGIT_TOL, F32_LOGPROB_TOL, NEAR_TIE_GAP, check_argmax, make_ctx,
                      oracle_rollout, valid_mask)

pytestmark = pytest.mark.gpu

WIDE_8B = synth.DENSE_8B.replace(n_layers=2)      # hidden 4096, 32 / 8 heads x 128, ffn 12288, vocabulary 151936
WIDE_32B = synth.DENSE_32B.replace(n_layers=2)    # hidden 5120, 64 / 8 heads x 128, ffn 25600, vocabulary 151936
DEEP_64 = synth.ModelShape(64, 1024, 8, 1, 128, 4096, 151936)   # 64 layers, 8 query heads on one key/value head
PLEN, NEW = 40, 6   # one whole key tile and a cut one before the first generated token


def _pinned_blob(shape, seed):
    import torch
    dev = synth.make_weights(shape, seed, device="cuda")
    host = torch.empty(dev.shape, dtype=dev.dtype, pin_memory=True)
    host.copy_(dev)
    del dev
    torch.cuda.empty_cache()
    return host


@functools.lru_cache(maxsize=1)
def _case(name):
    """Weights, 16 prompts and the oracle's records of prompt 0 and prompt 15 (teacher-forced on its own tokens),
    computed once per shape and used by both batch sizes."""
    shape = {"8b": WIDE_8B, "32b": WIDE_32B, "deep": DEEP_64}[name]
    blob = _pinned_blob(shape, 0)
    blob32 = synth.widen_to_f32(blob)
    prompts, lens = synth.make_prompts(shape.vocab, 16, PLEN, seed=1)
    orc = oracle.load("f64")
    d = oracle.desc_from_shape(shape)
    refs, scores = {}, {}
    for p in (0, 15):
        refs[p] = orc.rollout(d, blob32, prompts[p:p + 1], lens[p:p + 1], G=1, max_new=NEW, temperature=1.0, seed=2, want_logits=True)
        s = np.concatenate([prompts[p], refs[p]["tokens"][0]])
        scores[p] = (s, orc.logprobs(d, blob32, s, 1.0))
    del blob32
    return shape, blob, prompts, lens, refs, scores


@pytest.mark.parametrize("name,rows", [("8b", 64), ("8b", 128), ("32b", 64), ("32b", 128), ("32b", 32), ("deep", 64)])
def test_decode_prefill_and_scoring_at_workload_width_and_depth(name, rows):
    shape, blob, prompts16, lens16, refs, scores = _case(name)
    G, P = 8, rows // 8
    pick = list(range(P - 1)) + [15]               # the batch's last prompt is the oracle's second one
    prompts, lens = prompts16[pick], lens16[pick]
    N = P * G
    forced = np.random.default_rng(3).integers(0, shape.vocab, size=(N, NEW)).astype(np.int32)
    forced[0], forced[N - 1] = refs[0]["tokens"][0], refs[15]["tokens"][0]
    ctx = make_ctx(shape, N, PLEN + NEW + 26, blob)
    # decode steps inside the full batch; step 0 is the prefill pass's last row
    tf = ctx.rollout(prompts, lens, G, NEW, 1.0, 2, forced=forced, want_logits=True)
    worst = 0.0
    for n, p in ((0, 0), (N - 1, 15)):
        err = float(np.abs(tf["logits"][n] - refs[p]["logits"][0]).max())
        worst = max(worst, err)
        assert err < BF16_LOGIT_TOL, (name, rows, n, err)
        check_argmax(tf["logits"][n:n + 1], refs[p]["logits"], np.ones((1, NEW), bool), BF16_LOGIT_TOL, f"{name}-{rows}-seq{n}")
    # the fused sampler in graph replay: sequence 0 has the oracle's stream id, so tokens and log-probs compare
    out = ctx.rollout(prompts, lens, G, NEW, 1.0, 2, forced=forced)
    assert np.array_equal(out["tokens"], tf["tokens"])
    same = out["tokens"][0] == refs[0]["tokens"][0]
    assert same.mean() >= 0.8
    lp_err = float(np.abs(out["logprobs"][0] - refs[0]["logprobs"][0])[same].max())
    assert lp_err < BF16_LOGPROB_TOL, lp_err
    # teacher-forced scoring of the two strings (causal block kernels, 256 x 256-tile or one-block GEMMs by row count)
    toks = np.stack([scores[0][0], scores[15][0]]).astype(np.int32)
    got = ctx.logprobs(toks, np.full(2, toks.shape[1], np.int32), 1.0)
    sc_err = max(float(np.abs(got[i] - scores[p][1]).max()) for i, p in enumerate((0, 15)))
    assert sc_err < BF16_LOGPROB_TOL, sc_err
    # the two GPU paths on the same tokens (what the learner's importance ratio sees)
    self_diff = float(np.abs(got[0, PLEN:][same] - out["logprobs"][0][same]).max())
    print(f"[{name} x {rows} rows] max |dlogit| {worst:.4f}, |dlogprob| decode {lp_err:.4f} scoring {sc_err:.4f}, decode vs scoring {self_diff:.4f}")
    assert self_diff < 2 * BF16_LOGPROB_TOL
    ctx.close()


# 10 weight blocks of 32 rows in the output and down projections, 74 in the gate/up projection, K = 320 and 1184 (padded to
# 384 and 1280): no tile of the 256-row GEMMs (four or eight blocks wide) and no padded k-range divides these evenly
RAGGED = synth.ModelShape(2, 320, 4, 2, 64, 1184, 1000)


def test_ragged_tile_edges_of_the_256_row_gemms():
    """Weight-block counts that are no multiple of the tile width and hidden / feed-forward widths that are no multiple of
    the k padding, at the two row counts that take the 256-row tiles: 4096 rows in a scoring pass (256 x 256 tiles on the
    gate/up projection, 256 x 128 on the others) and a 256-row decode step."""
    shape = RAGGED
    blob = _pinned_blob(shape, 5)
    blob32 = synth.widen_to_f32(blob)
    orc = oracle.load("f64")
    d = oracle.desc_from_shape(shape)
    # scoring: 8 strings of 512 tokens = one pass of 4096 rows; the oracle scores the first and the last
    toks = np.random.default_rng(11).integers(0, shape.vocab, size=(8, 512)).astype(np.int32)
    ctx = make_ctx(shape, 256, 512, blob)
    got = ctx.logprobs(toks, np.full(8, 512, np.int32), 1.0)
    for i in (0, 7):
        want = orc.logprobs(d, blob32, toks[i], 1.0)
        err = float(np.abs(got[i] - want).max())
        assert err < BF16_LOGPROB_TOL, (i, err)
    # decode: 32 prompts x 8 = 256 rows, teacher-forced; the oracle follows the first and the last sequence
    G, P, plen, new = 8, 32, 24, 5
    prompts, lens = synth.make_prompts(shape.vocab, P, plen, seed=6)
    forced = np.random.default_rng(7).integers(0, shape.vocab, size=(P * G, new)).astype(np.int32)
    tf = ctx.rollout(prompts, lens, G, new, 1.0, 2, forced=forced, want_logits=True)
    for n, pidx in ((0, 0), (P * G - 1, P - 1)):
        ref = orc.rollout(d, blob32, prompts[pidx:pidx + 1], lens[pidx:pidx + 1], G=1, max_new=new, temperature=1.0, seed=2,
                          want_logits=True, forced=forced[n:n + 1])
        err = float(np.abs(tf["logits"][n] - ref["logits"][0]).max())
        assert err < BF16_LOGIT_TOL, (n, err)
    ctx.close()


# 17 strips of 256 columns in the output and down projections with K = 6144: at 4096 rows that is 272 tiles of 256 x 256 on
# 256 compute units, the case in which the GEMM splits K in two runs and the reducing kernel sums two planes
KSPLIT = synth.ModelShape(1, 4352, 48, 12, 128, 6144, 2048)


def test_k_split_of_the_4096_row_gemm():
    shape = KSPLIT
    blob = _pinned_blob(shape, 8)
    blob32 = synth.widen_to_f32(blob)
    orc = oracle.load("f64")
    d = oracle.desc_from_shape(shape)
    toks = np.random.default_rng(12).integers(0, shape.vocab, size=(8, 512)).astype(np.int32)
    ctx = make_ctx(shape, 8, 512, blob)
    got = ctx.logprobs(toks, np.full(8, 512, np.int32), 1.0)
    want = orc.logprobs(d, blob32, toks[5], 1.0)
    err = float(np.abs(got[5] - want).max())
    assert err < BF16_LOGPROB_TOL, err
    ctx.close()


def test_k_split_of_the_256_row_gemm():
    """A 256-row decode step whose projections are few 256 x 128 tiles with K = 2048: the launch splits K in four runs and
    the reducing kernels sum four planes."""
    shape = synth.ModelShape(1, 2048, 16, 4, 128, 2048, 2048)
    blob = _pinned_blob(shape, 9)
    blob32 = synth.widen_to_f32(blob)
    orc = oracle.load("f64")
    d = oracle.desc_from_shape(shape)
    G, P, plen, new = 8, 32, 40, 4
    prompts, lens = synth.make_prompts(shape.vocab, P, plen, seed=10)
    forced = np.random.default_rng(13).integers(0, shape.vocab, size=(P * G, new)).astype(np.int32)
    ctx = make_ctx(shape, P * G, plen + new + 20, blob)
    tf = ctx.rollout(prompts, lens, G, new, 1.0, 2, forced=forced, want_logits=True)
    for n, pidx in ((0, 0), (P * G - 1, P - 1)):
        ref = orc.rollout(d, blob32, prompts[pidx:pidx + 1], lens[pidx:pidx + 1], G=1, max_new=new, temperature=1.0, seed=2,
                          want_logits=True, forced=forced[n:n + 1])
        err = float(np.abs(tf["logits"][n] - ref["logits"][0]).max())
        assert err < BF16_LOGIT_TOL, (n, err)
    ctx.close()


@pytest.mark.parametrize("hd", [64, 128])
def test_tied_embeddings_and_qk_norm_on_the_decode_path(hd):
    """Gains drawn away from 1 (a dropped or misplaced gain shows), lm_head = embedding table, per-head q/k norm; ragged
    prompts over several key tiles; teacher-forced decode logits against the oracle."""
    shape = synth.ModelShape(2, 512, 8, 2, hd, 1024, 2048, dtype="bf16", qk_norm=True, tie_embeddings=True)
    blob = synth.make_weights(shape, 7, gain_jitter=0.2)
    blob32 = synth.widen_to_f32(blob)
    prompts, lens = synth.make_prompts(shape.vocab, 5, 90, seed=4, ragged=True)
    prompts = np.maximum(prompts, 0)
    G, max_new = 4, 9
    ref = oracle_rollout(shape, blob32, prompts, lens, G=G, max_new=max_new, temperature=0.9, seed=5, want_logits=True)
    ctx = make_ctx(shape, 20, 128, blob)
    tf = ctx.rollout(prompts, lens, G, max_new, 0.9, 5, forced=ref["tokens"], want_logits=True)
    assert np.abs(tf["logits"] - ref["logits"]).max() < BF16_LOGIT_TOL
    check_argmax(tf["logits"], ref["logits"], np.ones((20, max_new), bool), BF16_LOGIT_TOL, f"tied-qknorm-hd{hd}")
    out = ctx.rollout(prompts, lens, G, max_new, 0.9, 5, forced=ref["tokens"])
    same = out["tokens"] == ref["tokens"]
    assert same.mean() > 0.9 and np.abs(out["logprobs"] - ref["logprobs"])[same].max() < BF16_LOGPROB_TOL
    # and through the continuous entry point (every token from a decode step)
    cont = ctx.rollout(prompts, lens, G, max_new, 0.9, 5, forced=ref["tokens"], continuous=True)
    same = cont["tokens"] == ref["tokens"]
    assert same.mean() > 0.9 and np.abs(cont["logprobs"] - ref["logprobs"])[same].max() < BF16_LOGPROB_TOL
    ctx.close()


def test_operands_beyond_the_half_range_saturate_to_finite_values():
    """gate and up weights of +-40 make silu(gate) * up of the order 1e5 .. 1e6, past the largest finite half (65504): the
    feed-forward operand saturates instead of turning into inf, and everything downstream stays finite."""
    shape = synth.ModelShape(2, 256, 4, 2, 64, 512, 1024, dtype="bf16")
    blob = synth.make_weights(shape, 1)
    offs = synth.blob_offsets(shape)
    import torch
    gen = torch.Generator().manual_seed(9)
    for name in ("layers.0.w_gate", "layers.0.w_up"):
        off, shp = offs[name]
        n = int(np.prod(shp))
        blob[off:off + n] = (40.0 * torch.sign(torch.randn(n, generator=gen))).to(blob.dtype)
    prompts, lens = synth.make_prompts(shape.vocab, 4, 20, seed=2)
    ctx = make_ctx(shape, 8, 40, blob)
    out = ctx.rollout(prompts, lens, 2, 12, 1.0, 3, want_logits=True)
    assert np.isfinite(out["logits"]).all() and np.isfinite(out["logprobs"]).all()
    assert ((out["tokens"] >= 0) & (out["tokens"] < shape.vocab)).all() and (out["logprobs"] <= 0).all()
    # the same weights with fp32 activations (debug kernels) do not saturate: the logits differ visibly, so the MFMA path
    # did clamp, and the oracle's operand at that place is indeed beyond the half range
    naive = make_ctx(shape, 8, 40, blob, debug_naive=True)
    ref = naive.rollout(prompts, lens, 2, 12, 1.0, 3, forced=np.maximum(out["tokens"], 0), want_logits=True)
    naive.close()
    assert np.isfinite(ref["logits"]).all() and np.abs(ref["logits"] - out["logits"]).max() > 10 * BF16_LOGIT_TOL
    lp = ctx.logprobs(np.concatenate([prompts, np.maximum(out["tokens"][::2], 0)], axis=1), np.full(4, 32, np.int32), 1.0)
    assert np.isfinite(lp).all()
    ctx.close()


def _versions_to_schedule(vers_row, ids):
    """Versions of one sequence's tokens -> (indices into ids of the snapshots used, first step of each later one)."""
    used, swaps = [ids.index(int(vers_row[0]))], []
    for s in range(1, len(vers_row)):
        j = ids.index(int(vers_row[s]))
        if j != used[-1]:
            used.append(j)
            swaps.append(s)
    return used, swaps


@pytest.mark.parametrize("dtype,mode", [("fp32", "pinned-logits"), ("fp32", "pinned"), ("bf16", "pinned"), ("fp32", "continuous"),
                                        ("bf16", "continuous")])
def test_snapshots_installed_back_to_back_while_the_rollout_switches(dtype, mode):
    """Three snapshots: B is staged while the rollout decodes under A; the moment the rollout has switched to B the next
    install starts into the slot A has just left, while decode steps of A may still be queued on the GPU.  Every step's
    result must be that of the snapshot its version tag names (oracle with the same switch steps).  "pinned": switches at
    fixed steps, graph replay, the host queues steps ahead of the GPU; "pinned-logits": the same step by step with the
    logits returned; "continuous": the rollout switches whenever a snapshot has been staged."""
    continuous = mode == "continuous"
    shape = synth.TINY.replace(dtype=dtype)
    blobs = [synth.make_weights(shape, sd) for sd in (0, 10, 20)]
    b32 = [synth.widen_to_f32(b) for b in blobs]
    ids = [3, 8, 9]
    prompts, lens = synth.make_prompts(shape.vocab, 4, 16, seed=1)
    G, max_new = 2, 300
    swaps = [60, 140]
    forced = np.random.default_rng(5).integers(0, shape.vocab, size=(8, max_new)).astype(np.int32)
    # A continuous rollout that finds B staged before its first step has built the prompts' K/V under A and draws the
    # first token under B, which the oracle's schedule cannot express: such a run is repeated, staging B a little later.
    for attempt in range(8):
        ctx = make_ctx(shape, 8, 16 + max_new, blobs[0], version=ids[0], slots=2)
        box = {}

        def run():
            kw = dict(forced=forced, continuous=True) if continuous else dict(forced=forced, swap_at_step=swaps, swap_timeout_ms=30000,
                                                                              want_logits=mode == "pinned-logits")
            box["out"] = ctx.rollout(prompts, lens, G, max_new, 1.0, 2, **kw)

        t = threading.Thread(target=run)
        t.start()
        while t.is_alive() and not ctx.stats().rollout_running:
            time.sleep(0.0005)
        time.sleep(0.0005 * attempt)
        for j in (1, 2):
            ctx.load_policy(ids[j], blobs[j])                   # staged (or active at once if the rollout has already ended)
            while t.is_alive() and ctx.stats().staged_version >= 0:   # until the rollout has switched to it
                time.sleep(0.0002)
        t.join(120)
        assert not t.is_alive() and "out" in box
        out = box["out"]
        st = ctx.stats()
        assert st.active_version == ids[2] and st.staged_version == -1
        ctx.close()
        assert (out["lens"] == max_new).all()
        used, sw = _versions_to_schedule(out["versions"][0], ids)
        assert (out["versions"] == out["versions"][0]).all()
        if used[0] == 0:
            break
    assert used[0] == 0, "the rollout never drew its first token under the first snapshot"
    print(f"[{dtype} {mode}] snapshots used {used}, switched at steps {sw} (attempt {attempt})")
    if not continuous:
        assert used == [0, 1, 2] and sw == swaps
    ref = oracle_rollout(shape, [b32[j] for j in used], prompts, lens, G=G, max_new=max_new, temperature=1.0, seed=2,
                         versions=[ids[j] for j in used], swap_at_step=sw, forced=forced, want_logits=mode == "pinned-logits")
    assert np.array_equal(out["versions"], ref["versions"])
    if mode == "pinned-logits":
        assert np.abs(out["logits"] - ref["logits"]).max() < (F32_LOGIT_TOL if dtype == "fp32" else BF16_LOGIT_TOL)
    same = out["tokens"] == ref["tokens"]
    if dtype == "fp32":
        assert ((~same) & (ref["gaps"] >= NEAR_TIE_GAP)).sum() == 0
    else:
        assert same.mean() > 0.9
    assert np.abs(out["logprobs"] - ref["logprobs"])[same].max() < (F32_LOGPROB_TOL if dtype == "fp32" else BF16_LOGPROB_TOL)
