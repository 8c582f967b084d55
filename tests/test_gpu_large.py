"""GPU parity on tensors whose element counts and byte offsets do not fit 32 bits.

The entry points accept up to 2^31 groups; the benchmark's tensors stay far below 2^32 elements, so
these cases are the ones that walk the 64-bit index paths: element positions (they feed the
stochastic-rounding draw position L/16 of the backward quantizers), byte offsets into sources and
results beyond 4 GiB, and a GEMM result of more than 2^32 bytes.  Inputs are seeded blocks repeated
along the long dimension (the outputs still differ from block to block wherever the position enters);
the oracle computes row slabs with full-matrix indexing, among them the last rows, which lie past the
2^32 mark."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_14669_amd import binding as q
from paper_2505_14669_amd import synth
from indep import scales_from_tiled, scales_to_tiled

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def slabs(rows, width, n, seed):
    rng = np.random.default_rng(seed)
    starts = [0, rows - width] + [int(s) for s in rng.integers(1, rows - width - 1, size=n - 2)]
    return [(s, s + width) for s in starts]


def test_quantizers_past_2_pow_32_elements(G):
    block = synth.small_matrix(901, 4096, 32768, "outliers")
    x = np.tile(block, (34, 1))                    # 139264 x 32768 = 4.56e9 elements, 9.1 GB
    rows, k = x.shape
    assert rows * k > 2 ** 32
    xd = G.to_dev(x)
    sw, seed = 0xA5A5F00D, 2 ** 50 + 77

    def outputs(r, c, with_mask):
        return (G.dev_empty((r, c // 2), np.uint8, 0xEE), G.dev_empty((q.quartet_scale_bytes(r, c),), np.uint8, 0xFF),
                G.dev_empty((r, c // 32), np.uint32, 0x5A5A5A5A) if with_mask else None)

    # forward quantizer, row mode
    codes, scales, mask = outputs(rows, k, True)
    q.check(q.quartet_quant_fwd(xd, rows, k, k, 0, codes, scales, mask))
    hc, hs, hm = G.to_host(codes, np.uint8), scales_from_tiled(G.to_host(scales, np.uint8), rows, k), G.to_host(mask, np.uint32)
    for r0, r1 in slabs(rows, 32, 4, 1):
        wc, ws, wm = oracle.quant_fwd(x, rows_range=(r0, r1))
        assert np.array_equal(hc[r0:r1], wc) and np.array_equal(hs[r0:r1], ws) and np.array_equal(hm[r0:r1], wm)
    del mask, hm

    # backward quantizer with stochastic rounding, row mode: the draw position is the element position / 16
    q.check(q.quartet_quant_bwd_sr(xd, rows, k, k, 0, sw, seed, 1, 0, codes, scales))
    hc, hs = G.to_host(codes, np.uint8), scales_from_tiled(G.to_host(scales, np.uint8), rows, k)
    for r0, r1 in slabs(rows, 32, 4, 2):
        wc, ws = oracle.quant_bwd_sr(x, sw, seed, 1, 0, rows_range=(r0, r1))
        assert np.array_equal(hc[r0:r1], wc) and np.array_equal(hs[r0:r1], ws)
    # two blocks of the repeated input quantize to different codes: the position did enter
    assert not np.array_equal(hc[:64], hc[4096:4096 + 64])
    del codes, scales, hc, hs

    # the same source read along its other dimension: logical [32768 x 139264]
    codes, scales, _ = outputs(k, rows, False)
    q.check(q.quartet_quant_bwd_sr(xd, k, rows, k, 1, sw, seed, 2, 0, codes, scales))
    hc, hs = G.to_host(codes, np.uint8), scales_from_tiled(G.to_host(scales, np.uint8), k, rows)
    for r0, r1 in slabs(k, 16, 4, 3):
        wc, ws = oracle.quant_bwd_sr(x, sw, seed, 2, 0, transpose=True, rows_range=(r0, r1))
        assert np.array_equal(hc[r0:r1], wc) and np.array_equal(hs[r0:r1], ws)


def test_requantizer_past_2_pow_32_bytes_of_codes(G):
    rng = np.random.default_rng(902)
    k, rows = 278528, 32768                        # source MXFP4 [k x rows]: 9.1e9 elements, 4.56 GB of codes
    src_codes = np.tile(rng.integers(0, 256, size=(4096, rows // 2), dtype=np.uint8), (k // 4096, 1))
    src_scales = np.tile(rng.integers(118, 134, size=(4096, rows // 32), dtype=np.uint8), (k // 4096, 1))
    assert src_codes.nbytes > 2 ** 32
    sw, seed = 0x0F1E2D3C, 2 ** 41 + 5
    sc, ss = G.to_dev(src_codes), G.to_dev(scales_to_tiled(src_scales))
    codes = G.dev_empty((rows, k // 2), np.uint8, 0xEE)
    scales = G.dev_empty((q.quartet_scale_bytes(rows, k),), np.uint8, 0xFF)
    q.check(q.quartet_requant_transpose_sr(sc, ss, rows, k, sw, seed, 3, 0, codes, scales))
    hc, hs = G.to_host(codes, np.uint8), scales_from_tiled(G.to_host(scales, np.uint8), rows, k)
    for r0, r1 in slabs(rows, 8, 4, 4):
        wc, ws = oracle.requant_transpose_sr(src_codes, src_scales, sw, seed, 3, 0, rows_range=(r0, r1))
        assert np.array_equal(hc[r0:r1], wc) and np.array_equal(hs[r0:r1], ws)


@pytest.mark.parametrize("fused", [False, True])
def test_gemm_result_past_2_pow_32_bytes(G, fused):
    m, n, k = 40960, 32768, 64                     # fp32 result: 1.34e9 elements, 5.4 GB
    rng = np.random.default_rng(903 + fused)
    ac = rng.integers(0, 256, size=(m, k // 2), dtype=np.uint8)
    bc = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    asc = rng.integers(120, 132, size=(m, k // 32), dtype=np.uint8)
    bsc = rng.integers(120, 132, size=(n, k // 32), dtype=np.uint8)
    assert m * n * 4 > 2 ** 32
    d = G.dev_empty((m, n), np.float32, float("nan"))
    args = (G.to_dev(ac), G.to_dev(scales_to_tiled(asc)), G.to_dev(bc), G.to_dev(scales_to_tiled(bsc)), m, n, k)
    if fused:
        mask = rng.integers(0, 2 ** 32, size=(m, n // 32), dtype=np.uint32)
        q.check(q.quartet_mxfp4_gemm_grad(*args, G.to_dev(mask), oracle.FL_16_9, d, q.QUARTET_DTYPE_F32, n))
    else:
        q.check(q.quartet_mxfp4_gemm(*args, 1.0, d, q.QUARTET_DTYPE_F32, n))
    torch.cuda.synchronize()
    for r0, r1 in slabs(m, 16, 5, 5):
        got = d[r0:r1].cpu().numpy().astype(np.float64)
        want = oracle.mxfp4_gemm(ac[r0:r1], asc[r0:r1], bc, bsc)
        if fused:
            want = oracle.grad_epilogue(want.astype(np.float32), mask[r0:r1])
        assert np.linalg.norm(got - want) <= 1e-5 * np.linalg.norm(want)
