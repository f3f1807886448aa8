"""Oracle of the quantised snapshot format (test infrastructure; never imported by the product package).

The paper names quantised updates only as future work for cutting snapshot traffic ("Limitations and Future
Work"), without a format; the format checked here is this build's reading: the blob lists the same tensors in the same
order as the bf16 blob (embed[V,d]; per layer attn_norm[d], wq, wk, wv, (q_norm, k_norm), wo, ffn_norm, w_gate, w_up,
w_down; final_norm[d]; lm_head[V,d] if untied).  A vector (norm gain) is stored as bf16, unchanged.  A matrix
[rows, K] is stored as `rows` little-endian fp32 scales followed by rows * K int8 codes, row-major; the weight it
stands for is the bf16 value nearest to float32(code) * scale in fp32 arithmetic (ties to even).  Installing the
quantised blob must leave the snapshot that installing the dequantised bf16 blob leaves.

Plain numpy, one tensor at a time, no blocking."""
from __future__ import annotations

from typing import List, Tuple

import numpy as np


def tensor_list(n_layers: int, hidden: int, n_q_heads: int, n_kv_heads: int, head_dim: int, ffn: int, vocab: int,
                qk_norm: bool, tie_embeddings: bool) -> List[Tuple[int, int]]:
    """(rows, K) of every tensor in blob order; rows == 0 marks a vector of K elements."""
    d, q, kv = hidden, n_q_heads * head_dim, n_kv_heads * head_dim
    t = [(vocab, d)]
    for _ in range(n_layers):
        t += [(0, d), (q, d), (kv, d), (kv, d)]
        if qk_norm:
            t += [(0, head_dim), (0, head_dim)]
        t += [(d, q), (0, d), (ffn, d), (ffn, d), (d, ffn)]
    t.append((0, d))
    if not tie_embeddings:
        t.append((vocab, d))
    return t


def q8_blob_bytes(tensors: List[Tuple[int, int]]) -> int:
    return sum(2 * k if rows == 0 else rows * 4 + rows * k for rows, k in tensors)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, on the bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def dequantize_q8(tensors: List[Tuple[int, int]], blob: np.ndarray) -> np.ndarray:
    """uint8 quantised blob -> uint16 array of the bf16 bit patterns of the whole dequantised blob."""
    blob = np.ascontiguousarray(blob, np.uint8)
    assert blob.size == q8_blob_bytes(tensors), (blob.size, q8_blob_bytes(tensors))
    out, off = [], 0
    for rows, k in tensors:
        if rows == 0:
            out.append(blob[off:off + 2 * k].view("<u2").copy())
            off += 2 * k
            continue
        scales = blob[off:off + 4 * rows].view("<f4")
        off += 4 * rows
        codes = blob[off:off + rows * k].view(np.int8).reshape(rows, k)
        off += rows * k
        w = codes.astype(np.float32) * scales[:, None].astype(np.float32)     # one fp32 product per weight
        out.append(f32_to_bf16_bits(w).reshape(-1))
    return np.concatenate(out)
