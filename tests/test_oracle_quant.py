"""Pins of the quantised-snapshot oracle (oracle/quant.py): sizes and order against the bf16 blob's tensor table,
closed-form dequantisation cases, the bf16 rounding against an independent library conversion and against its
definition by brute force."""
import numpy as np
import torch

from oracle import quant
from paper_2602_02192_amd import synth

MID = synth.ModelShape(2, 512, 8, 2, 128, 1024, 2048, dtype="bf16")


def tensors_of(s):
    return quant.tensor_list(s.n_layers, s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn, s.vocab, s.qk_norm, s.tie_embeddings)


def test_tensor_list_matches_the_bf16_blob_layout():
    for s in (MID, MID.replace(qk_norm=True), MID.replace(tie_embeddings=True), synth.DENSE_4B):
        t = tensors_of(s)
        table = synth.tensor_table(s)
        assert len(t) == len(table)
        for (rows, k), (_, shape, is_gain) in zip(t, table):
            assert ((k,) if rows == 0 else (rows, k)) == tuple(shape) and (rows == 0) == is_gain
        assert sum(k if rows == 0 else rows * k for rows, k in t) == synth.blob_numel(s)
        # a matrix costs one byte per weight and four per row, a gain two bytes
        n_mat = sum(rows * k for rows, k in t if rows)
        n_rows = sum(rows for rows, k in t if rows)
        n_vec = sum(k for rows, k in t if not rows)
        assert quant.q8_blob_bytes(t) == n_mat + 4 * n_rows + 2 * n_vec


def test_bf16_rounding_is_nearest_even():
    # hand cases on bit patterns: exact, below half, the two ties (to even), above half, negative
    cases = {0x3F800000: 0x3F80, 0x3F807FFF: 0x3F80, 0x3F808000: 0x3F80, 0x3F818000: 0x3F82, 0x3F808001: 0x3F81,
             0xBF808000: 0xBF80, 0xBF818000: 0xBF82, 0x00000000: 0x0000, 0x80000000: 0x8000}
    x = np.array(list(cases), np.uint32).view(np.float32)
    assert quant.f32_to_bf16_bits(x).tolist() == list(cases.values())
    # against the definition by brute force: the nearer of the two neighbouring bf16 values, the even one on a tie
    rng = np.random.default_rng(0)
    v = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    got = quant.f32_to_bf16_bits(v)
    lo = (v.view(np.uint32) >> 16).astype(np.uint32)                      # truncation: the neighbour towards zero
    hi = lo + 1
    flo = (lo << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    fhi = (hi << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    dlo, dhi = np.abs(v.astype(np.float64) - flo), np.abs(fhi - v.astype(np.float64))
    want = np.where(dlo < dhi, lo, np.where(dhi < dlo, hi, np.where(lo % 2 == 0, lo, hi)))
    assert np.array_equal(got, want.astype(np.uint16))
    # and against an independent library conversion
    assert np.array_equal(got, torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_dequantisation_closed_forms():
    t = [(0, 4), (3, 4)]                       # a gain of four elements, then a 3 x 4 matrix
    gains = np.array([0x3F80, 0x4000, 0xBF80, 0x3F00], "<u2")
    scales = np.array([0.5, 2.0 ** -7, 3.0], "<f4")
    codes = np.array([[0, 1, -1, 127], [-127, 64, 2, -3], [1, -1, 107, 109]], np.int8)
    blob = np.concatenate([gains.view(np.uint8), scales.view(np.uint8), codes.reshape(-1).view(np.uint8)])
    assert blob.size == quant.q8_blob_bytes(t) == 8 + 12 + 12
    bits = quant.dequantize_q8(t, blob)
    assert bits[:4].tolist() == gains.tolist()                       # vectors pass through unchanged
    w = (bits[4:].astype(np.uint32) << 16).view(np.float32).reshape(3, 4)
    # row 0 and 1: power-of-two scales, every product is exact in bf16 (|code| < 256)
    assert w[0].tolist() == [0.0, 0.5, -0.5, 63.5]
    assert w[1].tolist() == [-127 / 128, 0.5, 2 / 128, -3 / 128]
    # row 2: scale 3: 3, -3 exact; 321 = 0b101000001 needs nine significant bits and lies half-way between 320 and 322:
    # to the even significand, 320 (down); 327 = 0b101000111 half-way between 326 and 328: to 328 (up)
    assert w[2].tolist() == [3.0, -3.0, 320.0, 328.0]
    # the scale belongs to the row, not the column: transposing the roles would give 0.5 * 64 for element (1, 1)
    assert w[1, 1] == 64 * 2.0 ** -7


def test_a_generated_blob_dequantises_to_weights_of_the_expected_scale():
    s = MID.replace(qk_norm=True)
    t = tensors_of(s)
    q8 = synth.make_q8_weights(s, 3)
    assert q8.dtype == np.uint8 and q8.size == quant.q8_blob_bytes(t)
    bits = quant.dequantize_q8(t, q8)
    assert bits.size == synth.blob_numel(s)
    off = synth.blob_offsets(s)
    o, shp = off["layers.1.w_down"]
    w = (bits[o:o + int(np.prod(shp))].astype(np.uint32) << 16).view(np.float32)
    assert 0.012 < w.std() < 0.03 and abs(w.mean()) < 1e-3
    o, shp = off["layers.0.q_norm"]
    assert (bits[o:o + shp[0]] == 0x3F80).all()
    assert np.array_equal(quant.dequantize_q8(t, q8), bits)          # a pure function of the bytes
