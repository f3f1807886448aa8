"""The byte model behind bench.py's roofline figures, on cases small enough to count by hand (CPU only)."""
import importlib.util
import os
import subprocess
import sys

import numpy as np

from paper_2602_02192_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
bench = importlib.util.module_from_spec(spec)
spec.loader.exec_module(bench)

# 1 layer, 1 KV head of 64 dims, bf16: 2 * 1 * 1 * 64 * 2 = 256 bytes of K and V per key
SHAPE = synth.ModelShape(1, 64, 2, 1, 64, 128, 256, dtype="bf16")
KVB = 256
W_DEC = (64 * (2 + 2) * 64 + 2 * 64 * 64 + 3 * 64 * 128 + 256 * 64) * 2


def test_decode_bytes_of_one_sequence():
    # prompt 40, 3 tokens: decode passes s = 1, 2 read 40 + s keys and write one each
    total, w_dec, kvb = bench.algorithmic_bytes(SHAPE, [3], 40, group=1)
    assert (w_dec, kvb) == (W_DEC, KVB)
    assert total == 2 * W_DEC + ((40 + 1) + (40 + 2)) * KVB + 2 * KVB
    # every token out of a decode pass (continuous rollouts): s = 0 as well
    assert bench.algorithmic_bytes(SHAPE, [3], 40, group=1, first_step=0)[0] == total + W_DEC + 40 * KVB + KVB


def test_shared_prompt_tiles_count_once_per_group_with_an_active_sequence():
    # two sequences of one prompt of 70 tokens (two whole tiles = 64 shared keys), lengths 2 and 4
    gen = [2, 4]
    per_seq = bench.algorithmic_bytes(SHAPE, gen, 70, group=1)[0]
    shared = bench.algorithmic_bytes(SHAPE, gen, 70, group=2)[0]
    # pass 1 serves both sequences, passes 2 and 3 only the second: the 64 shared keys are saved once, in pass 1
    assert per_seq - shared == 64 * KVB
    want = 3 * W_DEC + ((64 + 2 * (6 + 1)) + (64 + 6 + 2) + (64 + 6 + 3)) * KVB + (2 + 1 + 1) * KVB
    assert shared == want


def test_attention_bytes_per_launch():
    gen = np.array([2, 4])
    per_key = 2 * 1 * 64 * 2                      # one layer's K and V of one key
    a = bench.attn_kv_bytes_per_launch(SHAPE, gen, 70, 2, [1, 3], whole_tiles=False)
    assert a == ((64 + 2 * 7) + (64 + 9)) * per_key / 2
    # whole tiles: a sequence's own 7 or 9 keys are fetched as one 32-key tile
    b = bench.attn_kv_bytes_per_launch(SHAPE, gen, 70, 2, [1, 3], whole_tiles=True)
    assert b == ((64 + 2 * 32) + (64 + 32)) * per_key / 2
    # the shared tiles attended by the prefix kernel are not this kernel's
    c = bench.attn_kv_bytes_per_launch(SHAPE, gen, 70, 2, [1, 3], whole_tiles=False, shared_elsewhere=True)
    assert c == (2 * 7 + 9) * per_key / 2


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
