"""Host-side checks that need no GPU: the shared library loads, exports every entry point that
include/echo.h declares, sizes its arena and blobs consistently, and rejects bad shapes."""
import ctypes as C
import os
import re

import pytest

from paper_2602_02192_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def echo():
    from paper_2602_02192_amd import echo as e
    return e


def _declared():
    text = open(os.path.join(ROOT, "include", "echo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(echo_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_entry_point(echo):
    names = _declared()
    assert "echo_load_policy" in names and "echo_rollout" in names and len(names) >= 10
    for n in names:
        assert hasattr(echo.lib, n), f"{n} is declared in include/echo.h but not exported"
    assert sorted(echo.EXPORTS) == names


def test_blob_and_arena_sizes(echo):
    for shape in (synth.TINY, synth.TINY.replace(dtype="bf16"), synth.DENSE_4B, synth.DENSE_8B, synth.DENSE_32B,
                  synth.TINY.replace(qk_norm=True), synth.TINY.replace(tie_embeddings=True)):
        d = echo.desc_from_shape(shape, 8, 64)
        elt = 4 if shape.dtype == "fp32" else 2
        assert echo.blob_bytes(d) == synth.blob_numel(shape) * elt
        assert echo.arena_bytes(d) > echo.blob_bytes(d)
    # the workloads fit one 288 GB GPU (weights + KV + activations)
    for shape, n, ctx, slots in ((synth.DENSE_4B, 64, 1536, 1), (synth.DENSE_4B, 256, 5120, 1),
                                 (synth.DENSE_8B, 128, 2560, 2), (synth.DENSE_32B, 64, 5120, 1)):
        d = echo.desc_from_shape(shape, n, ctx, n_weight_slots=slots)
        kv = n * ctx * 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2
        need = echo.arena_bytes(d)
        assert kv + slots * echo.blob_bytes(d) < need < 288e9
    # a second weight slot costs about one more packed copy of the model
    d1 = echo.desc_from_shape(synth.DENSE_8B, 128, 2560, n_weight_slots=1)
    d2 = echo.desc_from_shape(synth.DENSE_8B, 128, 2560, n_weight_slots=2)
    extra = echo.arena_bytes(d2) - echo.arena_bytes(d1)
    assert 0.95 * echo.blob_bytes(d1) < extra < 1.2 * echo.blob_bytes(d1)


@pytest.mark.parametrize("field,value", [("n_layers", 0), ("n_q_heads", 3), ("head_dim", 7), ("dtype", 5),
                                         ("max_seqs", 0), ("max_ctx", 1), ("n_weight_slots", 3), ("rope_base", 0.0)])
def test_invalid_shapes_are_rejected_with_a_message(echo, field, value):
    d = echo.desc_from_shape(synth.TINY, 8, 64)
    setattr(d, field, value)
    assert echo.arena_bytes(d) == 0 and echo.blob_bytes(d) == 0
    h = C.c_void_p()
    rc = echo.lib.echo_init(C.byref(d), 0, None, 0, None, None, C.byref(h))
    assert rc == echo.ECHO_EINVAL and not h.value
    assert b"invalid model description" in echo.lib.echo_last_error(None)


def test_mfma_path_shape_limits_are_reported(echo):
    ok = synth.TINY.replace(dtype="bf16")
    assert echo.arena_bytes(echo.desc_from_shape(ok, 8, 64)) > 0
    for bad in (ok.replace(hidden=250), ok.replace(head_dim=32, n_q_heads=8, n_kv_heads=4),
                ok.replace(head_dim=192, n_q_heads=4, n_kv_heads=2),
                ok.replace(n_q_heads=32, n_kv_heads=2, hidden=2048)):
        d = echo.desc_from_shape(bad, 8, 64)
        assert echo.arena_bytes(d) == 0
        # the same shape is accepted by the debug kernels
        assert echo.arena_bytes(echo.desc_from_shape(bad, 8, 64, debug_naive=True)) > 0


def test_init_argument_errors_need_no_device(echo):
    d = echo.desc_from_shape(synth.TINY, 8, 64)
    h = C.c_void_p()
    assert echo.lib.echo_init(C.byref(d), 0, None, 0, None, None, C.byref(h)) == echo.ECHO_EINVAL
    assert b"dev_arena" in echo.lib.echo_last_error(None)
    assert echo.lib.echo_init(C.byref(d), 0, C.c_void_p(256), 1024, None, None, C.byref(h)) == echo.ECHO_ENOMEM
    assert b"arena has 1024 bytes" in echo.lib.echo_last_error(None)
    assert echo.lib.echo_init(C.byref(d), 0, C.c_void_p(256), 1024, None, None, None) == echo.ECHO_EINVAL
    assert echo.lib.echo_rollout(None, None, 0, None, 0, 0, 0, 1.0, 0, None, None, None, None, None) == echo.ECHO_EINVAL
    echo.lib.echo_destroy(None)      # a no-op
