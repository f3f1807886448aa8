"""Pins for the oracle's decoder and rollout loop (CPU only).

The paper prints no worked forward pass, so the worked examples here are built so
that every intermediate has a closed form (written out below); the remaining pins
are invariants of the definition: KV-cached decoding equals full recompute,
causality, grouped-query attention with one query per KV head equals multi-head
attention, a zero down-projection makes the feed-forward block the identity, and a
rollout's recorded log-probs equal teacher-forced scoring of its own tokens."""
import numpy as np
import pytest

from oracle import oracle
from paper_2602_02192_amd import synth


def _blob(shape, **tensors):
    """fp32 blob, zero everywhere except gains = 1 and the named tensors."""
    blob = np.zeros(synth.blob_numel(shape), np.float32)
    offs = synth.blob_offsets(shape)
    for name, sh, is_gain in synth.tensor_table(shape):
        if is_gain:
            off = offs[name][0]
            blob[off:off + int(np.prod(sh))] = 1.0
    for name, val in tensors.items():
        key = name.replace("__", ".")
        off, sh = offs[key]
        blob[off:off + int(np.prod(sh))] = np.asarray(val, np.float32).reshape(sh).ravel()
    return blob


def _rand_model(shape, seed, gain_jitter=0.1):
    return synth.widen_to_f32(synth.make_weights(shape, seed, gain_jitter=gain_jitter))


SMALL = synth.ModelShape(2, 32, 4, 2, 8, 48, 40, dtype="fp32")


def test_blob_layout_agrees_with_generator(orc):
    for shape in (SMALL, SMALL.replace(qk_norm=True), SMALL.replace(tie_embeddings=True), synth.TINY):
        assert orc.blob_numel(oracle.desc_from_shape(shape)) == synth.blob_numel(shape)


def test_worked_example_uniform_attention(orc):
    # d=4, one head of width 4, E = 2I, Wq = Wk = 0 (all scores 0 -> uniform attention),
    # Wv = Wo = I, Wd = 0, lm_head = I, eps = 0.
    sh = synth.ModelShape(1, 4, 1, 1, 4, 4, 4, rms_eps=0.0, dtype="fp32")
    I = np.eye(4)
    blob = _blob(sh, embed=2 * I, layers__0__wv=I, layers__0__wo=I, lm_head=I,
                 layers__0__w_gate=0.3 * np.ones((4, 4)), layers__0__w_up=np.ones((4, 4)))
    d = oracle.desc_from_shape(sh)
    lg = orc.forward_cached(d, blob, [0, 1])
    # position 0: h = 2e0, a = 2e0 (mean square 1), o = v0 = 2e0, h' = 4e0, final norm -> 2e0
    assert np.allclose(lg[0], [2, 0, 0, 0], atol=1e-12)
    assert orc.log_softmax(lg[0])[0] == pytest.approx(2 - np.log(np.e ** 2 + 3), abs=1e-12)
    # position 1: o = (2e0 + 2e1)/2, h' = 2e1 + e0 + e1 = (1,3,0,0), rms = sqrt(2.5)
    assert np.allclose(lg[1], np.array([1, 3, 0, 0]) / np.sqrt(2.5), atol=1e-12)
    assert orc.logprobs(d, blob, [0, 1])[1] == pytest.approx(-np.log(np.e ** 2 + 3), abs=1e-12)


def test_worked_example_nonsymmetric_weights_and_swiglu(orc):
    # Same skeleton with shift matrices (S e_i = e_{i+1 mod 4}) so that a transposed operand
    # changes the answer, and with a live feed-forward block.
    sh = synth.ModelShape(1, 4, 1, 1, 4, 4, 4, rms_eps=0.0, dtype="fp32")
    I = np.eye(4)
    S = np.roll(I, 1, axis=0)            # S @ e_i = e_{i+1}
    c = 0.5
    blob = _blob(sh, embed=2 * I, layers__0__wv=S, layers__0__wo=I, lm_head=S @ S,
                 layers__0__w_gate=c * I, layers__0__w_up=I, layers__0__w_down=S)
    lg = orc.forward_cached(oracle.desc_from_shape(sh), blob, [0])[0]
    # h = 2e0; a = 2e0; v = S a = 2e1; single key -> o = 2e1; h' = 2e0 + 2e1
    # b = rmsnorm(h') = h'/sqrt(2) = sqrt2 (e0+e1); f = silu(c b) * b; h'' = h' + S f
    b = np.sqrt(2.0)
    f = (c * b) / (1 + np.exp(-c * b)) * b
    h2 = np.array([2.0, 2.0 + f, f, 0.0])
    want = (S @ S) @ (h2 / np.sqrt(np.mean(h2 * h2)))
    assert np.allclose(lg, want, atol=1e-12)
    assert lg[1] == 0.0 and lg[0] > 0          # S^2 moves coordinate 3 (zero) to 1 and 2 to 0


def test_worked_example_rope_enters_scores_only(orc):
    # d = hd = 2 (a single rotary pair, theta_0 = 1), Wq = Wk = Wv = Wo = I, Wd = 0, lm_head = I.
    sh = synth.ModelShape(1, 2, 1, 1, 2, 2, 2, rms_eps=0.0, dtype="fp32")
    I = np.eye(2)
    blob = _blob(sh, embed=2 * I, layers__0__wq=I, layers__0__wk=I, layers__0__wv=I,
                 layers__0__wo=I, lm_head=I)
    lg = orc.forward_cached(oracle.desc_from_shape(sh), blob, [0, 1])[1]
    # a0 = sqrt2 e0, a1 = sqrt2 e1.  q1 = R(1) a1 = sqrt2(-sin1, cos1); k0 = a0; k1 = q1.
    # scores / sqrt(hd): s0 = -sqrt2 sin1, s1 = sqrt2; values are NOT rotated.
    s = np.array([-np.sqrt(2) * np.sin(1.0), np.sqrt(2)])
    w = np.exp(s - s.max())
    w /= w.sum()
    h = np.array([0.0, 2.0]) + np.sqrt(2) * w
    assert np.allclose(lg, h / np.sqrt(np.mean(h * h)), atol=1e-12)


@pytest.mark.parametrize("qk_norm", [False, True])
def test_cached_decode_equals_full_recompute(orc, orc32, qk_norm):
    sh = SMALL.replace(qk_norm=qk_norm)
    blob = _rand_model(sh, 1)
    # larger weights so that attention is far from uniform
    blob *= 6.0
    d = oracle.desc_from_shape(sh)
    toks = np.random.default_rng(0).integers(0, sh.vocab, 12).astype(np.int32)
    a, b = orc.forward_cached(d, blob, toks), orc.forward_full(d, blob, toks)
    assert np.abs(a).max() > 0.1
    assert np.allclose(a, b, rtol=1e-11, atol=1e-12)
    a32, b32 = orc32.forward_cached(d, blob, toks), orc32.forward_full(d, blob, toks)
    assert np.allclose(a32, b32, rtol=1e-5, atol=1e-5)
    assert np.allclose(a32, a, rtol=1e-4, atol=2e-4)            # the fp32 build tracks the fp64 build


def test_worked_example_qk_norm_per_head_before_rotation_with_its_own_gains(orc):
    # d = 2, two query heads over one key/value head, hd = 2 (a single rotary pair, theta_0 = 1), eps = 0, tokens [0, 1].
    # E = 2I, so a0 = sqrt2 e0 and a1 = sqrt2 e1 and a projection of a_t is sqrt2 times column t of its matrix.
    #   Wq columns:  head 0: (*, *), (3, 4);   head 1: (*, *), (0, 10)      (only position 1 queries are looked at)
    #   Wk columns:  (4, 3) for token 0, (-3, 4) for token 1;  Wv = 3I;  Wo = [I | I] (adds the two heads);  Wd = 0
    #   gains: q_norm = (2, 1/2), k_norm = (1/2, 3): unequal inside the pair, so norm-then-rotate != rotate-then-norm,
    #   and q and k gains differ, so swapping them shows; two heads of different length, so one norm over the whole
    #   q vector shows; values are three times too long for a norm applied to them to go unnoticed.
    sh = synth.ModelShape(1, 2, 2, 1, 2, 2, 2, rms_eps=0.0, dtype="fp32", qk_norm=True)
    I = np.eye(2)
    wq = np.array([[1.0, 3.0], [2.0, 4.0], [5.0, 0.0], [1.0, 10.0]])
    wk = np.array([[4.0, -3.0], [3.0, 4.0]])
    gq, gk = np.array([2.0, 0.5]), np.array([0.5, 3.0])
    blob = _blob(sh, embed=2 * I, layers__0__wq=wq, layers__0__wk=wk, layers__0__wv=3 * I, layers__0__wo=np.hstack([I, I]),
                 layers__0__q_norm=gq, layers__0__k_norm=gk, lm_head=I)
    lg = orc.forward_cached(oracle.desc_from_shape(sh), blob, [0, 1])[1]
    r2, c1, s1 = np.sqrt(2.0), np.cos(1.0), np.sin(1.0)
    rot = lambda v: np.array([v[0] * c1 - v[1] * s1, v[0] * s1 + v[1] * c1])
    # per-head unit-RMS vectors times the gain, written out: |(3,4)| = 5 -> rms 5/sqrt2 * sqrt2 ... = (0.6, 0.8) sqrt2
    q0 = rot(r2 * np.array([0.6, 0.8]) * gq)            # = rot(sqrt2 (1.2, 0.4))
    q1 = rot(r2 * np.array([0.0, 1.0]) * gq)            # = rot(sqrt2 (0, 0.5))
    k0 = r2 * np.array([0.8, 0.6]) * gk                  # position 0: no rotation; = sqrt2 (0.4, 1.8)
    k1 = rot(r2 * np.array([-0.6, 0.8]) * gk)           # = rot(sqrt2 (-0.3, 2.4))
    assert np.allclose(q0, rot(r2 * np.array([1.2, 0.4]))) and np.allclose(k0, r2 * np.array([0.4, 1.8]))
    v0, v1 = 3 * r2 * np.array([1.0, 0.0]), 3 * r2 * np.array([0.0, 1.0])
    h = np.array([0.0, 2.0])
    for q in (q0, q1):
        s = np.array([q @ k0, q @ k1]) / np.sqrt(2.0)
        w = np.exp(s - s.max())
        w /= w.sum()
        h = h + w[0] * v0 + w[1] * v1
    want = h / np.sqrt(np.mean(h * h))
    assert np.allclose(lg, want, atol=1e-12)
    # the plausible mistakes move the answer by far more than the tolerance above
    def variant(q_vecs, k_vecs):
        hh = np.array([0.0, 2.0])
        for q in q_vecs:
            s = np.array([q @ k_vecs[0], q @ k_vecs[1]]) / np.sqrt(2.0)
            w = np.exp(s - s.max())
            w /= w.sum()
            hh = hh + w[0] * v0 + w[1] * v1
        return hh / np.sqrt(np.mean(hh * hh))
    rotate_then_norm = variant([gq * rot(r2 * np.array([0.6, 0.8])), gq * rot(r2 * np.array([0.0, 1.0]))],
                               [k0, gk * rot(r2 * np.array([-0.6, 0.8]))])
    swapped_gains = variant([rot(r2 * np.array([0.6, 0.8]) * gk), rot(r2 * np.array([0.0, 1.0]) * gk)],
                            [r2 * np.array([0.8, 0.6]) * gq, rot(r2 * np.array([-0.6, 0.8]) * gq)])
    qall = np.array([3.0, 4.0, 0.0, 10.0])
    qall = qall / np.sqrt(np.mean(qall * qall))        # one norm over both heads
    whole_vector = variant([rot(qall[:2] * gq), rot(qall[2:] * gq)], [k0, k1])
    for wrong in (rotate_then_norm, swapped_gains, whole_vector):
        assert np.abs(wrong - want).max() > 1e-3


def test_qk_norm_changes_the_result_and_gains_matter(orc):
    d0, d1 = oracle.desc_from_shape(SMALL), oracle.desc_from_shape(SMALL.replace(qk_norm=True))
    toks = np.arange(6, dtype=np.int32)
    b1 = _rand_model(SMALL.replace(qk_norm=True), 2) * 6
    lg1 = orc.forward_cached(d1, b1, toks)
    # dropping the two gain vectors from the blob gives the plain model with the same matrices
    offs = synth.blob_offsets(SMALL.replace(qk_norm=True))
    keep = np.ones(b1.size, bool)
    for name, (off, shp) in offs.items():
        if name.endswith("q_norm") or name.endswith("k_norm"):
            keep[off:off + int(np.prod(shp))] = False
    lg0 = orc.forward_cached(d0, b1[keep], toks)
    assert np.abs(lg1[1:] - lg0[1:]).max() > 1e-3


def test_causality(orc):
    blob = _rand_model(SMALL, 3) * 6
    d = oracle.desc_from_shape(SMALL)
    t1 = np.array([5, 9, 2, 7, 1, 30], np.int32)
    t2 = t1.copy()
    t2[4:] = [11, 12]
    a, b = orc.forward_full(d, blob, t1), orc.forward_full(d, blob, t2)
    assert np.array_equal(a[:4], b[:4])
    assert np.abs(a[4:] - b[4:]).max() > 1e-3


def test_gqa_with_replicated_kv_heads_equals_mha(orc):
    gqa = SMALL                                   # 4 query heads on 2 KV heads
    mha = SMALL.replace(n_kv_heads=4)
    bg = _rand_model(gqa, 4) * 6
    og, om = synth.blob_offsets(gqa), synth.blob_offsets(mha)
    bm = np.zeros(synth.blob_numel(mha), np.float32)
    hd, H = gqa.head_dim, gqa.hidden
    for name, (off, shp) in om.items():
        n = int(np.prod(shp))
        src_off, src_shp = og[name]
        src = bg[src_off:src_off + int(np.prod(src_shp))].reshape(src_shp)
        if name.endswith(".wk") or name.endswith(".wv"):
            # query head j uses KV head j // 2: replicate each KV head's rows twice
            src = src.reshape(2, hd, H).repeat(2, axis=0).reshape(4 * hd, H)
        bm[off:off + n] = src.ravel()
    toks = np.array([3, 1, 4, 1, 5, 9, 2, 6], np.int32)
    a = orc.forward_cached(oracle.desc_from_shape(gqa), bg, toks)
    b = orc.forward_cached(oracle.desc_from_shape(mha), bm, toks)
    assert np.allclose(a, b, rtol=1e-12, atol=1e-13)


def test_zero_down_projection_makes_ffn_identity(orc):
    b1 = _rand_model(SMALL, 5) * 6
    b2 = b1.copy()
    offs = synth.blob_offsets(SMALL)
    for l in range(SMALL.n_layers):
        for nm in ("w_down",):
            off, shp = offs[f"layers.{l}.{nm}"]
            b1[off:off + int(np.prod(shp))] = 0
            b2[off:off + int(np.prod(shp))] = 0
        off, shp = offs[f"layers.{l}.w_gate"]           # with Wd = 0 the gate cannot matter
        b2[off:off + int(np.prod(shp))] *= -3.0
    d = oracle.desc_from_shape(SMALL)
    toks = np.array([1, 2, 3, 4], np.int32)
    assert np.array_equal(orc.forward_cached(d, b1, toks), orc.forward_cached(d, b2, toks))


def test_tied_embeddings_use_the_embedding_as_lm_head(orc):
    tied = SMALL.replace(tie_embeddings=True)
    bt = _rand_model(tied, 6) * 6
    untied = np.concatenate([bt, bt[:SMALL.vocab * SMALL.hidden]])
    toks = np.array([7, 8, 9], np.int32)
    a = orc.forward_cached(oracle.desc_from_shape(tied), bt, toks)
    b = orc.forward_cached(oracle.desc_from_shape(SMALL), untied, toks)
    assert np.array_equal(a, b)


# ---- rollout loop -------------------------------------------------------------------------

def _roll(orc, blob, **kw):
    d = oracle.desc_from_shape(SMALL)
    prompts, lens = synth.make_prompts(SMALL.vocab, 3, 5, seed=1)
    args = dict(G=2, max_new=6, temperature=1.0, seed=2)
    args.update(kw)
    return orc.rollout(d, blob, prompts, lens, **args), prompts, lens


def test_rollout_logprobs_equal_teacher_forced_scoring_of_own_tokens(orc):
    blob = _rand_model(SMALL, 7) * 6
    d = oracle.desc_from_shape(SMALL)
    r, prompts, lens = _roll(orc, blob, temperature=0.8, want_logits=True)
    assert (r["lens"] == 6).all() and (r["tokens"] >= 0).all()
    for n in range(6):
        seq = np.concatenate([prompts[n // 2, :lens[n // 2]], r["tokens"][n]]).astype(np.int32)
        lp = orc.logprobs(d, blob, seq, 0.8)
        assert np.allclose(lp[lens[n // 2]:], r["logprobs"][n], atol=1e-10)
        # and the logits it sampled from are the full-recompute logits of the same string
        full = orc.forward_full(d, blob, seq)
        assert np.allclose(full[lens[n // 2] - 1:-1], r["logits"][n], rtol=1e-10, atol=1e-11)
    assert (r["logprobs"] < 0).all()


def test_group_members_share_first_logits_then_differ(orc):
    blob = _rand_model(SMALL, 7) * 6
    r, _, _ = _roll(orc, blob, G=4, temperature=4.0, want_logits=True)
    lg = r["logits"].reshape(3, 4, 6, -1)
    assert np.array_equal(lg[:, 0, 0], lg[:, 1, 0]) and np.array_equal(lg[:, 0, 0], lg[:, 3, 0])
    assert len({tuple(r["tokens"][n]) for n in range(12)}) == 12


def test_rollout_is_independent_of_batch_composition(orc):
    blob = _rand_model(SMALL, 7) * 6
    d = oracle.desc_from_shape(SMALL)
    full, prompts, lens = _roll(orc, blob)
    solo = orc.rollout(d, blob, prompts[:1], lens[:1], G=2, max_new=6, temperature=1.0, seed=2)
    assert np.array_equal(solo["tokens"], full["tokens"][:2])
    assert np.array_equal(solo["logprobs"], full["logprobs"][:2])


def test_stop_lengths_eos_padding_and_forcing(orc):
    blob = _rand_model(SMALL, 7) * 6
    stop = np.array([1, 6, 3, 9, 2, 4], np.int32)
    r, _, _ = _roll(orc, blob, stop_lens=stop)
    assert list(r["lens"]) == [1, 6, 3, 6, 2, 4]
    free, _, _ = _roll(orc, blob)
    for n in range(6):
        L = r["lens"][n]
        assert np.array_equal(r["tokens"][n, :L], free["tokens"][n, :L])
        assert (r["tokens"][n, L:] == -1).all() and (r["logprobs"][n, L:] == 0).all()
        assert (r["versions"][n, :L] == 0).all() and (r["versions"][n, L:] == -1).all()
    # an EOS id ends the sequence after the EOS token itself
    eos = int(free["tokens"][0, 2])
    e, _, _ = _roll(orc, blob, eos_id=eos)
    first = int(np.argmax(free["tokens"][0] == eos))
    assert e["lens"][0] == first + 1 and e["tokens"][0, first] == eos
    # teacher forcing: what is recorded at step s is the draw from the forced prefix
    forced = np.random.default_rng(9).integers(0, SMALL.vocab, (6, 6)).astype(np.int32)
    f, prompts, lens = _roll(orc, blob, forced=forced, want_logits=True)
    d = oracle.desc_from_shape(SMALL)
    seq = np.concatenate([prompts[0, :lens[0]], forced[0]]).astype(np.int32)
    full = orc.forward_full(d, blob, seq)
    assert np.allclose(full[lens[0] - 1:-1], f["logits"][0], rtol=1e-10, atol=1e-11)
    assert f["tokens"][0, 0] == free["tokens"][0, 0]            # step 0 sees the prompt only


def test_version_swap_semantics(orc):
    A = _rand_model(SMALL, 7) * 6
    d = oracle.desc_from_shape(SMALL)
    base, prompts, lens = _roll(orc, A, want_logits=True)
    # swapping to an identical copy changes nothing except the version tags
    same = orc.rollout(d, [A, A.copy()], prompts, lens, G=2, max_new=6, temperature=1.0, seed=2,
                       versions=[10, 12], swap_at_step=[3])
    assert np.array_equal(same["tokens"], base["tokens"])
    assert np.array_equal(same["logprobs"], base["logprobs"])
    assert (same["versions"][:, :3] == 10).all() and (same["versions"][:, 3:] == 12).all()
    # a snapshot that differs only in final_norm / lm_head leaves the KV cache valid, so from the
    # swap step on the logits are exactly those of B on the same token string
    B = A.copy()
    off, shp = synth.blob_offsets(SMALL)["lm_head"]
    B[off:] = _rand_model(SMALL, 8)[off:] * 6
    forced = base["tokens"]
    sw = orc.rollout(d, [A, B], prompts, lens, G=2, max_new=6, temperature=1.0, seed=2,
                     swap_at_step=[2], forced=forced, want_logits=True)
    onlyB = orc.rollout(d, B, prompts, lens, G=2, max_new=6, temperature=1.0, seed=2,
                        forced=forced, want_logits=True)
    assert np.array_equal(sw["logits"][:, :2], base["logits"][:, :2])
    assert np.array_equal(sw["logits"][:, 2:], onlyB["logits"][:, 2:])
    assert np.abs(sw["logits"][:, 2:] - base["logits"][:, 2:]).max() > 1e-3
    # a snapshot that differs everywhere: steps before the swap are untouched, later ones move
    C = _rand_model(SMALL, 11) * 6
    sc = orc.rollout(d, [A, C], prompts, lens, G=2, max_new=6, temperature=1.0, seed=2,
                     swap_at_step=[4], forced=forced, want_logits=True)
    assert np.array_equal(sc["logits"][:, :4], base["logits"][:, :4])
    assert np.abs(sc["logits"][:, 4:] - base["logits"][:, 4:]).max() > 1e-3


def test_tiny_config_rollout_fp32_build_tracks_fp64(orc, orc32):
    sh = synth.TINY
    blob = synth.widen_to_f32(synth.make_weights(sh, 0))
    d = oracle.desc_from_shape(sh)
    prompts, lens = synth.make_prompts(sh.vocab, 2, 16, seed=1)
    a = orc.rollout(d, blob, prompts, lens, G=2, max_new=4, temperature=1.0, seed=2, want_logits=True)
    b = orc32.rollout(d, blob, prompts, lens, G=2, max_new=4, temperature=1.0, seed=2, forced=a["tokens"],
                      want_logits=True)
    assert np.abs(a["logits"] - b["logits"]).max() < 2e-5
    assert np.abs(a["logits"]).std() > 0.1                       # logits are O(0.02 sqrt(d)), not ~0
    ok = (a["tokens"] == b["tokens"]) | (a["gaps"] < 1e-4)
    assert ok.all()
