"""quartet_linear_bwd_static (the backward pass with its workspace in a device array of the library, for callers that
cannot allocate) against quartet_linear_bwd on the same inputs: two calls in a row, the second on a smaller layer,
so the second runs over what the first left in the array.  Both entry points launch the same kernels in the same
order, so the results must agree bit for bit (tighter than the 1e-5 Frobenius bar of the GEMM parity tests)."""
import numpy as np
import pytest

from paper_2505_14669_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def layer_tensors(t, i, o, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    x = synth.f32_to_bf16(rng.standard_t(3.0, size=(t, i)).astype(np.float32))
    w = synth.f32_to_bf16(rng.standard_normal((o, i), dtype=np.float32) * np.float32(0.02))
    dy = synth.f32_to_bf16(rng.standard_normal((t, o), dtype=np.float32) * np.float32(1e-3))
    return x, w, dy


def test_static_scratch_backward_matches_workspace_backward_twice(G):
    q = G.q
    assert q.quartet_static_scratch_bytes() == 64 << 20
    for n, (t, i, o) in enumerate([(1024, 512, 768), (256, 256, 128)]):       # the second call is the smaller one
        assert q.quartet_linear_workspace_bytes(t, i, o) <= q.quartet_static_scratch_bytes()
        x, w, dy = layer_tensors(t, i, o, 77 + n)
        for rounding in (0, 1):
            seed = 2 ** 33 + 5 * n + rounding
            lin = G.Linear(x, w)
            lin.fwd()
            dy_dev = G.to_dev(dy)
            lin.bwd(dy_dev, seed, rounding)                                      # existing entry point, caller's workspace
            want_dx, want_dw = G.to_host(lin.dx, np.uint32).copy(), G.to_host(lin.dw, np.uint32).copy()
            assert np.isfinite(want_dx.view(np.float32)).all() and np.isfinite(want_dw.view(np.float32)).all()
            dx = G.dev_empty((t, i), np.float32, float("nan"))
            dw = G.dev_empty((o, i), np.float32, float("nan"))
            q.check(q.quartet_linear_bwd_static(dy_dev, t, i, o, lin.xq_codes, lin.xq_scales, lin.x_mask, lin.wq_codes,
                                                lin.wq_scales, lin.w_mask, seed, rounding, dx, dw, q.QUARTET_DTYPE_F32))
            assert np.array_equal(G.to_host(dx, np.uint32), want_dx), (t, i, o, rounding)
            assert np.array_equal(G.to_host(dw, np.uint32), want_dw), (t, i, o, rounding)
