"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

This module holds none of the method's arithmetic: it only draws random weights,
prompts and stop lengths, and lays the weights out in the flat blob order that
both sides read.  The same bytes are handed to the oracle and to the GPU library.

Blob order (row-major [out, in], y = W x), all tensors of one dtype:
  embed[V,d];
  per layer: attn_norm[d], wq[Hq*hd,d], wk[Hkv*hd,d], wv[Hkv*hd,d],
             (q_norm[hd], k_norm[hd] when qk_norm), wo[d,Hq*hd],
             ffn_norm[d], w_gate[F,d], w_up[F,d], w_down[d,F];
  final_norm[d]; lm_head[V,d] (absent when tie_embeddings).

Matrices and embeddings are N(0, 0.02^2); every RMSNorm gain is 1 (gains drawn
from N(0,0.02) would collapse the logits to ~0).  bf16 models are the fp32 draw
rounded to nearest-even once, here; the oracle reads those bf16 values widened
to fp32, so weight rounding never counts as GPU error.
"""
from __future__ import annotations

import dataclasses
from typing import List, Tuple

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 1e4
    dtype: str = "bf16"          # "fp32" | "bf16"
    qk_norm: bool = False
    tie_embeddings: bool = False

    def replace(self, **kw) -> "ModelShape":
        return dataclasses.replace(self, **kw)


# The model families of the workloads (decoder shapes only; weights are random).
TINY = ModelShape(2, 256, 4, 2, 64, 704, 1024, dtype="fp32")
DENSE_4B = ModelShape(36, 2560, 32, 8, 128, 9728, 151936)
DENSE_8B = ModelShape(36, 4096, 32, 8, 128, 12288, 151936)
DENSE_32B = ModelShape(64, 5120, 64, 8, 128, 25600, 151936)


def tensor_table(s: ModelShape) -> List[Tuple[str, Tuple[int, ...], bool]]:
    """(name, shape, is_gain) for every tensor in blob order."""
    d, hd = s.hidden, s.head_dim
    t: List[Tuple[str, Tuple[int, ...], bool]] = [("embed", (s.vocab, d), False)]
    for l in range(s.n_layers):
        p = f"layers.{l}."
        t.append((p + "attn_norm", (d,), True))
        t.append((p + "wq", (s.n_q_heads * hd, d), False))
        t.append((p + "wk", (s.n_kv_heads * hd, d), False))
        t.append((p + "wv", (s.n_kv_heads * hd, d), False))
        if s.qk_norm:
            t.append((p + "q_norm", (hd,), True))
            t.append((p + "k_norm", (hd,), True))
        t.append((p + "wo", (d, s.n_q_heads * hd), False))
        t.append((p + "ffn_norm", (d,), True))
        t.append((p + "w_gate", (s.ffn, d), False))
        t.append((p + "w_up", (s.ffn, d), False))
        t.append((p + "w_down", (d, s.ffn), False))
    t.append(("final_norm", (d,), True))
    if not s.tie_embeddings:
        t.append(("lm_head", (s.vocab, d), False))
    return t


def blob_numel(s: ModelShape) -> int:
    return sum(int(np.prod(shape)) for _, shape, _ in tensor_table(s))


def blob_offsets(s: ModelShape) -> dict:
    """name -> (element offset, shape)."""
    off, out = 0, {}
    for name, shape, _ in tensor_table(s):
        out[name] = (off, shape)
        off += int(np.prod(shape))
    return out


def make_weights(s: ModelShape, seed: int, device: str = "cpu",
                 gain_jitter: float = 0.0) -> torch.Tensor:
    """Flat weight blob in the model's dtype (torch.float32 or torch.bfloat16).

    Drawn with torch's seeded generator on `device`, tensor by tensor in blob order.
    The bytes depend on (shape, seed, device type); a caller that needs the same
    model on both sides generates once and passes the same blob to both.
    `gain_jitter` > 0 draws the norm gains as 1 + N(0, jitter^2) instead of 1, for
    tests that must notice a dropped or misplaced gain.
    """
    dt = torch.float32 if s.dtype == "fp32" else torch.bfloat16
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    blob = torch.empty(blob_numel(s), dtype=dt, device=device)
    off = 0
    for _, shape, is_gain in tensor_table(s):
        n = int(np.prod(shape))
        if is_gain:
            if gain_jitter > 0.0:
                w = 1.0 + gain_jitter * torch.randn(n, generator=g, device=device,
                                                    dtype=torch.float32)
                blob[off:off + n] = w.to(dt)
            else:
                blob[off:off + n] = 1.0
        else:
            # chunked so that a 1.5 GB tensor never needs a second fp32 copy of itself
            step = 1 << 26
            for a in range(0, n, step):
                b = min(n, a + step)
                w = torch.randn(b - a, generator=g, device=device, dtype=torch.float32)
                blob[off + a:off + b] = (w * 0.02).to(dt)     # RNE for bf16
        off += n
    return blob


def widen_to_f32(blob: torch.Tensor) -> np.ndarray:
    """The blob's values as a host fp32 array (lossless for bf16 and fp32)."""
    return blob.detach().to("cpu", torch.float32).numpy()


def make_prompts(vocab: int, n_prompts: int, prompt_len: int, seed: int,
                 ragged: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """Token ids iid uniform over [0, vocab): int32 [P, prompt_len] and lengths [P].

    With `ragged`, lengths are uniform in [1, prompt_len] and the tail is padded
    with -1 (never read)."""
    rng = np.random.default_rng(seed)
    toks = rng.integers(0, vocab, size=(n_prompts, prompt_len), dtype=np.int64).astype(np.int32)
    lens = np.full(n_prompts, prompt_len, dtype=np.int32)
    if ragged:
        lens = rng.integers(1, prompt_len + 1, size=n_prompts).astype(np.int32)
        for p in range(n_prompts):
            toks[p, lens[p]:] = -1
    return toks, lens


def make_stop_lens(n_seqs: int, lo: int, hi: int, seed: int) -> np.ndarray:
    """Per-sequence stop lengths iid uniform over {lo..hi} (stand-in for EOS)."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=n_seqs).astype(np.int32)


def make_turn_records(n_seqs: int, stride: int, vocab: int, turn_start_id: int, seed: int,
                      max_turns: int = 9, binary_rewards: bool = True) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Finished multi-turn records for the learner-side tensors: tokens int32 [N, stride], lens [N], rewards f32 [N].

    Lengths are uniform in [0, stride]; tokens are iid uniform over the vocabulary without the turn-start id, which is
    then planted at the first position and at up to max_turns - 1 further uniform positions (about one record in
    eight gets no turn start at all, one in eight a single one).  The padding beyond a record's length holds random
    tokens, turn starts included, so that a reader that ignores the length is caught.  Rewards are 0/1 outcomes
    (about one group-sized run in ten all equal) or, with binary_rewards off, normal with mean 3 and deviation 40."""
    rng = np.random.default_rng(seed)
    toks = rng.integers(0, vocab - 1, size=(n_seqs, stride), dtype=np.int64)
    toks[toks >= turn_start_id] += 1
    lens = rng.integers(0, stride + 1, size=n_seqs).astype(np.int32)
    for n in range(n_seqs):
        kind = rng.integers(0, 8)
        if kind == 0 or lens[n] == 0:
            pass
        else:
            toks[n, 0] = turn_start_id
            if kind > 1:
                k = int(rng.integers(1, max_turns))
                toks[n, rng.integers(0, lens[n], size=k)] = turn_start_id
        pad = stride - lens[n]
        if pad:
            toks[n, lens[n]:] = rng.integers(0, vocab, size=pad)
            toks[n, lens[n]:][rng.random(pad) < 0.01] = turn_start_id
    if binary_rewards:
        rewards = (rng.random(n_seqs) < 0.4).astype(np.float32)
        for g0 in range(0, n_seqs, 16):
            if rng.random() < 0.1:
                rewards[g0:g0 + 16] = rewards[g0]
    else:
        rewards = rng.normal(3.0, 40.0, n_seqs).astype(np.float32)
    return toks.astype(np.int32), lens, rewards


def make_q8_weights(s: ModelShape, seed: int) -> np.ndarray:
    """A quantised snapshot blob (uint8) for a bf16 shape, in the layout of echo_load_policy_q8: tensors in blob order,
    gains as bf16 ones, every matrix [rows, K] as rows fp32 scales followed by rows * K int8 codes.  Codes are
    round(N(0, 42^2)) clipped to [-127, 127] and scales uniform in [0.5, 1.5] * 0.02 / 42, so the weights they stand for
    look like the N(0, 0.02^2) weights of the other generators.  Random bytes only: what the codes mean is the
    library's and the oracle's business."""
    assert s.dtype == "bf16"
    rng = np.random.default_rng(seed)
    parts = []
    for _, shape, is_gain in tensor_table(s):
        if len(shape) == 1:
            assert is_gain
            parts.append(np.full(shape[0], 0x3F80, "<u2").view(np.uint8))
            continue
        rows, k = shape
        parts.append(((0.5 + rng.random(rows)) * (0.02 / 42.0)).astype("<f4").view(np.uint8))
        step = max(1, (1 << 26) // k)
        for a in range(0, rows, step):
            b = min(rows, a + step)
            c = np.clip(np.rint(rng.standard_normal((b - a, k), np.float32) * 42.0), -127, 127).astype(np.int8)
            parts.append(c.reshape(-1).view(np.uint8))
    return np.concatenate(parts)
