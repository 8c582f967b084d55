"""MXFP8 comparison path (Section 5, "Speedup results": the format the MXFP4 layers are measured against)
against the oracle: quantizer bit for bit, GEMM to the accuracy of the matrix cores' FP8 accumulation."""
import numpy as np
import pytest

import oracle
from indep import scales_from_tiled, scales_to_tiled
from paper_2505_14669_amd import synth

pytestmark = pytest.mark.gpu

# The FP8 matrix-core instruction aligns its 64 products to a common exponent before adding them and
# drops what falls below.  FP4 products span 8 binades and survive exactly; FP8 products span 30.
# Measured on operands with uniformly random codes (every exponent equally likely, the worst case for
# alignment): element errors up to 3.3e-4 of the sum of the products' magnitudes (mean 2e-5), relative
# Frobenius error 5e-5 .. 6.5e-5.  The bounds are those figures with a factor 3 of margin.
FP8_ABS_TERMS_TOL = 1e-3
FP8_FRO_TOL_RANDOM = 2e-4
FP8_FRO_TOL_GAUSSIAN = 1e-4


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _quant(G, x, ldx=None):
    from paper_2505_14669_amd import binding as q
    rows, k = x.shape
    full = x
    if ldx is not None:
        full = np.full((rows, ldx), 0x7FC1, dtype=np.uint16)
        full[:, :k] = x
    codes = G.dev_empty((rows, k), np.uint8, 0xEE)
    scales = G.dev_empty((max(q.quartet_scale_bytes(rows, k), 4),), np.uint8, 0xFF)
    q.check(q.quartet_mxfp8_quant(G.to_dev(full), rows, k, full.shape[1], codes, scales))
    return G.to_host(codes, np.uint8), scales_from_tiled(G.to_host(scales, np.uint8), rows, k)


@pytest.mark.parametrize("shape", [(1, 32), (64, 256), (37, 96), (129, 2080), (700, 160)])
def test_mxfp8_quant_bit_exact(G, shape):
    for j, kind in enumerate(("normal", "outliers", "heavy", "tiny", "zeros")):
        x = synth.small_matrix(600 + j, shape[0], shape[1], kind)
        want = oracle.mxfp8_quant(x)
        got = _quant(G, x)
        assert np.array_equal(got[1], want[1]), f"{shape} {kind} scales"
        assert np.array_equal(got[0], want[0]), f"{shape} {kind} codes"
    got = _quant(G, x, ldx=shape[1] + 40)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])


def _gemm(G, ac, asc, bc, bsc, alpha=1.0, bf16=False, ldd=None):
    from paper_2505_14669_amd import binding as q
    m, k = ac.shape
    n = bc.shape[0]
    ldd = n if ldd is None else ldd
    d = G.dev_empty((m, ldd), np.uint16 if bf16 else np.float32, 0x7FC0 if bf16 else float("nan"))
    q.check(q.quartet_mxfp8_gemm(G.to_dev(ac), G.to_dev(scales_to_tiled(asc)), G.to_dev(bc), G.to_dev(scales_to_tiled(bsc)),
                                 m, n, k, alpha, d, q.QUARTET_DTYPE_BF16 if bf16 else q.QUARTET_DTYPE_F32, ldd))
    return G.to_host(d, np.uint16 if bf16 else np.float32)


@pytest.mark.parametrize("mnk", [(1, 1, 32), (32, 32, 64), (130, 70, 96), (257, 129, 160), (64, 300, 1024), (520, 513, 800)])
def test_mxfp8_gemm_random_codes(G, mnk):
    m, n, k = mnk
    rng = np.random.default_rng(m * 1000 + n)
    ac = rng.integers(0, 0x7F, size=(m, k), dtype=np.uint8) | (rng.integers(0, 2, size=(m, k), dtype=np.uint8) << 7)
    bc = rng.integers(0, 0x7F, size=(n, k), dtype=np.uint8) | (rng.integers(0, 2, size=(n, k), dtype=np.uint8) << 7)
    asc = rng.integers(117, 137, size=(m, k // 32), dtype=np.uint8)
    bsc = rng.integers(117, 137, size=(n, k // 32), dtype=np.uint8)
    want = oracle.mxfp8_gemm(ac, asc, bc, bsc, alpha=0.75)
    got = _gemm(G, ac, asc, bc, bsc, alpha=0.75)
    terms = 0.75 * np.abs(oracle.mxfp8_dequant(ac, asc)) @ np.abs(oracle.mxfp8_dequant(bc, bsc)).T
    assert np.all(np.abs(got - want) <= FP8_ABS_TERMS_TOL * terms + 1e-30)
    assert np.linalg.norm(got - want) <= FP8_FRO_TOL_RANDOM * np.linalg.norm(want)
    got_ld = _gemm(G, ac, asc, bc, bsc, alpha=0.75, ldd=n + 5)
    assert np.array_equal(got_ld[:, :n], got) and np.all(np.isnan(got_ld[:, n:]))
    got_bf = synth.bf16_to_f32(_gemm(G, ac, asc, bc, bsc, alpha=0.75, bf16=True))
    assert np.array_equal(got_bf, synth.bf16_to_f32(synth.f32_to_bf16(got)))


def test_mxfp8_quant_then_gemm_on_gaussian_data(G):
    rng = np.random.default_rng(8)
    a = synth.f32_to_bf16(rng.standard_normal((384, 1024)).astype(np.float32))
    b = synth.f32_to_bf16((rng.standard_normal((320, 1024)) * 0.02).astype(np.float32))
    ac, asc = _quant(G, a)
    bc, bsc = _quant(G, b)
    want = oracle.mxfp8_gemm(ac, asc, bc, bsc)
    got = _gemm(G, ac, asc, bc, bsc)
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    print("relative Frobenius error of the FP8 GEMM on quantized Gaussian data:", rel)
    assert rel < FP8_FRO_TOL_GAUSSIAN
