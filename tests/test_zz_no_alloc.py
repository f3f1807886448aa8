"""The entry point for callers that cannot allocate (echo_grpo_tensors_static: staging in the library's static device
array) against echo_grpo_tensors, through the C ABI: two calls in a row, the second smaller, results identical bit for
bit (same kernels on the same staged bytes), and both equal to the oracle; sizes beyond the array are refused."""
import numpy as np
import pytest

from paper_2602_02192_amd import synth

from gpu_util import make_ctx

pytestmark = pytest.mark.gpu

TAU = 11


def test_static_scratch_entry_point_matches_the_arena_entry_point(orc):
    from paper_2602_02192_amd import echo
    ctx = make_ctx(synth.DENSE_4B.replace(n_layers=1), 64, 64)      # a context whose arena stages the larger call in one go too
    for N, G, stride, seed in ((96, 8, 5000, 1), (24, 4, 1027, 2)):  # 4.3 MB of staging, then 0.2 MB over the stale 4.3
        toks, lens, rewards = synth.make_turn_records(N, stride, 2048, TAU, seed=seed)
        want = ctx.grpo_tensors(toks, lens, G, TAU, rewards)
        got = ctx.grpo_tensors(toks, lens, G, TAU, rewards, static_scratch=True)
        for a, b in zip(got, want):
            assert np.array_equal(a, b, equal_nan=True)
        rmask, radv, _ = orc.grpo_tensors(toks, lens, G, TAU, rewards.astype(np.float64), float(np.float32(1e-6)))
        assert np.array_equal(got[0], rmask)
        np.testing.assert_allclose(got[1], radv, rtol=1e-7, atol=1e-30)
        m2, a2, t2 = ctx.grpo_tensors(toks, lens, G, TAU, rewards, static_scratch=True, per_token=False)
        assert t2 is None and np.array_equal(m2, want[0]) and np.array_equal(a2, want[1], equal_nan=True)
    # one record more than the array holds is refused with a message that names both sizes
    stride = 9216
    n_fit = echo.STATIC_SCRATCH_BYTES // (9 * stride + 12)
    n_over = (n_fit // 2 + 1) * 2
    with pytest.raises(echo.EchoError) as e:
        ctx.grpo_tensors(np.zeros((n_over, stride), np.int32), np.zeros(n_over, np.int32), 2, TAU, np.zeros(n_over, np.float32),
                         static_scratch=True)
    assert e.value.code == echo.ECHO_ENOMEM and str(echo.STATIC_SCRATCH_BYTES) in str(e.value)
    with pytest.raises(echo.EchoError) as e:
        ctx.grpo_tensors(np.zeros((3, 8), np.int32), np.zeros(3, np.int32), 2, TAU, np.zeros(3, np.float32), static_scratch=True)
    assert e.value.code == echo.ECHO_EINVAL
    ctx.close()
