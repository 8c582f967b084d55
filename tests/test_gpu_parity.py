"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: packed FP4 codes, scale bytes and mask words bit-exact; GEMM and gradient outputs within a
relative Frobenius error of 1e-5 (fp32 accumulation on the matrix cores against the oracle's fp64;
the bound sqrt(K/32) * 2^-24 is far below it)."""
import numpy as np
import pytest

import oracle
from paper_2505_14669_amd import synth
import indep
from indep import scale_tiled_bytes as q_scale_bytes, scales_from_tiled, scales_to_tiled

pytestmark = pytest.mark.gpu

FRO_TOL = 1e-5


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return np.linalg.norm(a - b) / den if den > 0 else np.linalg.norm(a)


def within_elem_bound(got, want, abs_products, k, alpha=1.0, grad_scale=None, block=32):
    """the per-element bar next to the Frobenius one: (K/64 + 3) 2^-23 sum |a||b| per product element
    (indep.gemm_elem_bound), carried through the Hadamard epilogue when grad_scale is given"""
    bound = indep.gemm_elem_bound(abs_products, k, alpha)
    if grad_scale is not None:
        bound = indep.grad_elem_bound(bound, abs_products, grad_scale, block)
    return indep.worst_excess(got, want, bound) <= 1.0


def same(a, b, what):
    a, b = np.asarray(a), np.asarray(b)
    assert a.shape == b.shape, (what, a.shape, b.shape)
    bad = np.argwhere(a != b)
    assert bad.size == 0, f"{what}: {len(bad)} mismatches, first at {bad[0]}: got {a[tuple(bad[0])]:#x} want {b[tuple(bad[0])]:#x}"


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


SHAPES = [(1, 32), (3, 64), (64, 256), (37, 96), (129, 2080), (256, 512), (700, 160)]
KINDS = ["normal", "outliers", "heavy", "tiny", "zeros"]


@pytest.mark.parametrize("shape", SHAPES)
def test_quant_fwd_row(G, shape):
    for j, kind in enumerate(KINDS):
        x = synth.small_matrix(100 + j, shape[0], shape[1], kind)
        got = G.quant_fwd(x)
        want = oracle.quant_fwd(x)
        for g, w, name in zip(got, want, ("codes", "scales", "mask")):
            same(g, w, f"fwd row {shape} {kind} {name}")
    got = G.quant_fwd(x, want_mask=False)
    same(got[0], want[0], "codes without mask")


def test_quant_fwd_row_strided(G):
    full = synth.small_matrix(7, 50, 256, "outliers")
    x = full[:, :160]
    import torch
    xd = G.to_dev(full)
    codes = G.dev_empty((50, 80), np.uint8, 0)
    scales = G.dev_empty((q_scale_bytes(50, 160),), np.uint8, 0)
    mask = G.dev_empty((50, 5), np.uint32, 0)
    from paper_2505_14669_amd import binding as q
    q.check(q.quartet_quant_fwd(xd, 50, 160, 256, 0, codes, scales, mask))
    want = oracle.quant_fwd(np.ascontiguousarray(x))
    same(G.to_host(codes, np.uint8), want[0], "strided codes")
    same(scales_from_tiled(G.to_host(scales, np.uint8), 50, 160), want[1], "strided scales")
    same(G.to_host(mask, np.uint32), want[2], "strided mask")


@pytest.mark.parametrize("transpose", [False, True])
def test_quant_strided_source_with_nan_padding(G, transpose):
    # the columns between the logical width and the leading dimension hold NaN patterns: the kernels read
    # past the logical width inside a row (their loads are range-checked per block, not per element) but
    # nothing of it may reach the output
    from paper_2505_14669_amd import binding as q
    src_rows, width, ld = (160, 96, 136) if transpose else (77, 160, 392)
    full = np.full((src_rows, ld), 0x7FC1, dtype=np.uint16)
    x = synth.small_matrix(21, src_rows, width, "heavy")
    full[:, :width] = x
    rows, k = (width, src_rows) if transpose else (src_rows, width)
    xd = G.to_dev(full)
    for mode in ("fwd", "rtn", "sr"):
        codes = G.dev_empty((rows, k // 2), np.uint8, 0)
        scales = G.dev_empty((q_scale_bytes(rows, k),), np.uint8, 0)
        if mode == "fwd":
            mask = G.dev_empty((rows, k // 32), np.uint32, 0)
            q.check(q.quartet_quant_fwd(xd, rows, k, ld, int(transpose), codes, scales, mask))
            want = oracle.quant_fwd(x, transpose=transpose)
            same(G.to_host(mask, np.uint32), want[2], f"{mode} mask")
        else:
            q.check(q.quartet_quant_bwd_sr(xd, rows, k, ld, int(transpose), 0x9E3779B9, 31, 2, int(mode == "rtn"), codes, scales))
            want = oracle.quant_bwd_sr(x, 0x9E3779B9, 31, 2, int(mode == "rtn"), transpose=transpose)
        same(scales_from_tiled(G.to_host(scales, np.uint8), rows, k), want[1], f"{mode} scales")
        same(G.to_host(codes, np.uint8), want[0], f"{mode} codes")


@pytest.mark.parametrize("shape", [(32, 8), (64, 128), (96, 40), (256, 136), (288, 264), (1056, 72)])
def test_quant_fwd_transposed(G, shape):
    # source stored [k, rows]
    for j, kind in enumerate(("normal", "outliers", "heavy")):
        x = synth.small_matrix(200 + j, shape[0], shape[1], kind)
        got = G.quant_fwd(x, transpose=True)
        want = oracle.quant_fwd(x, transpose=True)
        for g, w, name in zip(got, want, ("codes", "scales", "mask")):
            same(g, w, f"fwd transposed {shape} {kind} {name}")


@pytest.mark.parametrize("rounding", [1, 0])
@pytest.mark.parametrize("shape", [(1, 32), (64, 256), (37, 96), (129, 2080), (700, 160)])
def test_quant_bwd_row(G, shape, rounding):
    for j, (kind, sw, seed, sid) in enumerate([("normal", 0, 0, 0), ("outliers", 0xDEADBEEF, 12345, 1),
                                               ("heavy", 0xFFFFFFFF, 2 ** 63 + 5, 3), ("tiny", 0x1, 7, 2),
                                               ("zeros", 0xF0F0F0F0, 9, 0)]):
        x = synth.small_matrix(300 + j, shape[0], shape[1], kind, scale=1e-3)
        got = G.quant_bwd_sr(x, sw, seed, sid, rounding)
        want = oracle.quant_bwd_sr(x, sw, seed, sid, rounding)
        same(got[1], want[1], f"bwd row {shape} {kind} r={rounding} scales")
        same(got[0], want[0], f"bwd row {shape} {kind} r={rounding} codes")


@pytest.mark.parametrize("rounding", [1, 0])
@pytest.mark.parametrize("shape", [(32, 8), (64, 128), (96, 40), (288, 264), (1056, 72)])
def test_quant_bwd_transposed(G, shape, rounding):
    for j, (kind, sw, seed, sid) in enumerate([("normal", 0x13572468, 5, 2), ("heavy", 0x80000001, 2 ** 40 + 3, 0)]):
        x = synth.small_matrix(400 + j, shape[0], shape[1], kind, scale=1e-3)
        got = G.quant_bwd_sr(x, sw, seed, sid, rounding, transpose=True)
        want = oracle.quant_bwd_sr(x, sw, seed, sid, rounding, transpose=True)
        same(got[1], want[1], f"bwd transposed {shape} {kind} r={rounding} scales")
        same(got[0], want[0], f"bwd transposed {shape} {kind} r={rounding} codes")


@pytest.mark.parametrize("rounding", [1, 0])
@pytest.mark.parametrize("shape", [(32, 32), (64, 128), (96, 160), (288, 256), (1056, 96)])
def test_requant_transpose(G, shape, rounding):
    # source MXFP4 [k, rows] made by the oracle's forward quantizer
    x = synth.small_matrix(500, shape[0], shape[1], "outliers")
    sc, ss, _ = oracle.quant_fwd(x)
    got = G.requant_transpose_sr(sc, ss, 0xA5A5A5A5, 99, 1, rounding)
    want = oracle.requant_transpose_sr(sc, ss, 0xA5A5A5A5, 99, 1, rounding)
    same(got[1], want[1], f"requant {shape} r={rounding} scales")
    same(got[0], want[0], f"requant {shape} r={rounding} codes")


def test_dequant(G):
    rng = np.random.default_rng(1)
    codes = rng.integers(0, 256, size=(33, 48), dtype=np.uint8)
    scales = rng.integers(1, 250, size=(33, 3), dtype=np.uint8)
    got = G.dequant(codes, scales)
    want = oracle.mxfp4_dequant(codes, scales).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_gemm_exhaustive_code_pairs_bit_exact(G):
    # single group, every code pair, several scale pairs: sums of 32 multiples of 1/4 are exact in fp32
    a = np.array([[i | (i << 4)] * 16 for i in range(16)], dtype=np.uint8)
    for sa, sb in ((127, 127), (120, 131), (100, 150), (140, 100)):
        got = G.gemm(a, np.full((16, 1), sa, np.uint8), a, np.full((16, 1), sb, np.uint8))
        want = oracle.mxfp4_gemm(a, np.full((16, 1), sa, np.uint8), a, np.full((16, 1), sb, np.uint8))
        assert np.array_equal(got.astype(np.float64), want)
    # mixed codes, equal scales, several groups: still exact
    rng = np.random.default_rng(2)
    ac = rng.integers(0, 256, size=(40, 64), dtype=np.uint8)
    bc = rng.integers(0, 256, size=(24, 64), dtype=np.uint8)
    one_a, one_b = np.full((40, 4), 127, np.uint8), np.full((24, 4), 127, np.uint8)
    got = G.gemm(ac, one_a, bc, one_b)
    assert np.array_equal(got.astype(np.float64), oracle.mxfp4_gemm(ac, one_a, bc, one_b))


@pytest.fixture(params=["auto", "0", "1", "2"])
def gemm_variant(request, G):
    # every tile shape of the GEMM kernel is checked, not only the one the size heuristic picks
    G.q.check(G.q.quartet_debug_set_gemm_plan(-1 if request.param == "auto" else int(request.param), 0))
    yield request.param
    G.q.check(G.q.quartet_debug_set_gemm_plan(-1, 0))


@pytest.mark.parametrize("mnk", [(1, 1, 32), (32, 32, 64), (128, 128, 128), (130, 70, 96), (257, 129, 160),
                                 (64, 300, 1024), (384, 256, 2048), (520, 513, 800)])
def test_gemm_random(G, mnk, gemm_variant):
    m, n, k = mnk
    rng = np.random.default_rng(m * 1000 + n)
    ac = rng.integers(0, 256, size=(m, k // 2), dtype=np.uint8)
    bc = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    asc = rng.integers(117, 137, size=(m, k // 32), dtype=np.uint8)
    bsc = rng.integers(117, 137, size=(n, k // 32), dtype=np.uint8)
    want = oracle.mxfp4_gemm(ac, asc, bc, bsc, alpha=0.75)
    got = G.gemm(ac, asc, bc, bsc, alpha=0.75)
    assert rel_fro(got, want) < FRO_TOL
    assert within_elem_bound(got, want, indep.gemm_abs_products(ac, asc, bc, bsc), k, alpha=0.75)
    got_ld = G.gemm(ac, asc, bc, bsc, alpha=0.75, ldd=n + 5)
    assert np.array_equal(got_ld[:, :n], got) and np.all(np.isnan(got_ld[:, n:]))
    got_bf = synth.bf16_to_f32(G.gemm(ac, asc, bc, bsc, alpha=0.75, bf16=True))
    assert np.array_equal(got_bf, synth.bf16_to_f32(synth.f32_to_bf16(got)))


@pytest.mark.parametrize("mnk", [(1, 32, 32), (130, 96, 96), (257, 160, 160), (64, 320, 1024), (520, 544, 800)])
def test_gemm_grad_fused(G, mnk, gemm_variant):
    # GEMM_LP with the backward epilogue of Algorithm 1 in the same kernel against the oracle's two steps
    m, n, k = mnk
    rng = np.random.default_rng(m * 1000 + n + 7)
    ac = rng.integers(0, 256, size=(m, k // 2), dtype=np.uint8)
    bc = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    asc = rng.integers(117, 137, size=(m, k // 32), dtype=np.uint8)
    bsc = rng.integers(117, 137, size=(n, k // 32), dtype=np.uint8)
    mask = rng.integers(0, 2 ** 32, size=(m, n // 32), dtype=np.uint32)
    acc = oracle.mxfp4_gemm(ac, asc, bc, bsc).astype(np.float32)
    want = oracle.grad_epilogue(acc, mask)
    got = G.gemm_grad(ac, asc, bc, bsc, mask, oracle.FL_16_9)
    assert rel_fro(got, want) < FRO_TOL
    absp = indep.gemm_abs_products(ac, asc, bc, bsc)
    assert within_elem_bound(got, want, absp, k, grad_scale=oracle.FL_16_9)
    # the header promises the same bits as the library's own two separate steps
    two_step = G.grad_epilogue(G.gemm(ac, asc, bc, bsc), mask, oracle.FL_16_9)
    assert np.array_equal(got.view(np.uint32), two_step.view(np.uint32))
    got_ld = G.gemm_grad(ac, asc, bc, bsc, mask, oracle.FL_16_9, ldd=n + 3)
    assert np.array_equal(got_ld[:, :n].view(np.uint32), got.view(np.uint32)) and np.all(np.isnan(got_ld[:, n:]))
    got_bf = G.gemm_grad(ac, asc, bc, bsc, mask, oracle.FL_16_9, bf16=True)
    assert np.array_equal(got_bf, synth.f32_to_bf16(got))
    got_nomask = G.gemm_grad(ac, asc, bc, bsc, None, 1.0)
    assert rel_fro(got_nomask, oracle.grad_epilogue(acc, None, 1.0)) < FRO_TOL
    assert within_elem_bound(got_nomask, oracle.grad_epilogue(acc, None, 1.0), absp, k, grad_scale=1.0)


@pytest.mark.parametrize("shapes", [((40, 96, 64), (7, 32, 160)), ((300, 544, 192), (513, 288, 416)), ((300, 544, 512), (513, 288, 1280)),
                                    ((1, 32, 32), (260, 1056, 32)), ((4352, 4352, 64), (1100, 2080, 96))])
def test_gemm_grad_pair_matches_two_calls(G, shapes, gemm_variant):
    # Algorithm 1 Backward: the dW and the dx product in one launch -- the same bits as one launch each, for products
    # with different inner dimensions, ragged tiles, a product of one tile beside one of ten, 289 tiles beside 45 (more tiles
    # than compute units: blocks walk from one product into the other), and every tile shape
    # (with tiles below 256 x 256 the entry point launches the two products one after the other)
    prods = []
    for idx, (m, n, k) in enumerate(shapes):
        rng = np.random.default_rng(m * 1000 + n + k + idx)
        prods.append((rng.integers(0, 256, size=(m, k // 2), dtype=np.uint8),
                      rng.integers(117, 137, size=(m, k // 32), dtype=np.uint8),
                      rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8),
                      rng.integers(117, 137, size=(n, k // 32), dtype=np.uint8),
                      None if n == 1056 else rng.integers(0, 2 ** 32, size=(m, n // 32), dtype=np.uint32),
                      oracle.FL_16_9 if idx == 0 else 1.25))
    got = G.gemm_grad_pair(prods[0], prods[1])
    for g, pr in zip(got, prods):
        alone = G.gemm_grad(*pr)
        if gemm_variant != "auto":      # one tile shape for the pair and for each product alone: the same bits
            assert np.array_equal(g.view(np.uint32), alone.view(np.uint32))
        else:                           # the pair's shape may differ from a product's own: the same sums in another order
            assert rel_fro(g, alone) < FRO_TOL
        want = oracle.grad_epilogue(oracle.mxfp4_gemm(pr[0], pr[1], pr[2], pr[3]).astype(np.float32), pr[4], pr[5])
        assert rel_fro(g, want) < FRO_TOL
        absp = indep.gemm_abs_products(pr[0], pr[1], pr[2], pr[3])
        assert within_elem_bound(g, want, absp, pr[0].shape[1] * 2, grad_scale=pr[5])
    got_bf = G.gemm_grad_pair(prods[1], prods[0], bf16=True)     # the other order, bf16 results
    assert np.array_equal(got_bf[0], synth.f32_to_bf16(got[1])) and np.array_equal(got_bf[1], synth.f32_to_bf16(got[0]))


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("band", [1, 3, 5, 64])
def test_gemm_tile_order_covers_every_tile_for_any_band_height(G, variant, band):
    # the XCD-aware tile order (bands of `band` tile rows per XCD) is a tuning knob of the C ABI: whatever its value, every
    # tile must be computed exactly once -- the result (prefilled with NaN) is bit-identical to the default order's, for one
    # product and for two in one launch
    rng = np.random.default_rng(99)
    def operands(m, n, k):
        return (rng.integers(0, 256, size=(m, k // 2), dtype=np.uint8), rng.integers(117, 137, size=(m, k // 32), dtype=np.uint8),
                rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8), rng.integers(117, 137, size=(n, k // 32), dtype=np.uint8))
    one = operands(1300, 1100, 64)
    first = operands(2100, 800, 96) + (rng.integers(0, 2 ** 32, size=(2100, 25), dtype=np.uint32), 1.5)
    second = operands(700, 1568, 32) + (None, 0.75)
    try:
        G.q.check(G.q.quartet_debug_set_gemm_plan(variant, 0))
        want_one = G.gemm(*one)
        want_pair = G.gemm_grad_pair(first, second)
        G.q.check(G.q.quartet_debug_set_gemm_plan(variant, band))
        got_one = G.gemm(*one)
        got_pair = G.gemm_grad_pair(first, second)
    finally:
        G.q.check(G.q.quartet_debug_set_gemm_plan(-1, 0))
    assert np.isfinite(want_one).all() and np.array_equal(got_one.view(np.uint32), want_one.view(np.uint32))
    for g, w in zip(got_pair, want_pair):
        assert np.isfinite(w).all() and np.array_equal(g.view(np.uint32), w.view(np.uint32))


@pytest.mark.parametrize("shape", [(1, 32), (6, 96), (77, 160), (256, 512)])
def test_grad_epilogue(G, shape):
    rng = np.random.default_rng(shape[0])
    g = rng.standard_normal(shape).astype(np.float32)
    mask = rng.integers(0, 2 ** 32, size=(shape[0], shape[1] // 32), dtype=np.uint32)
    want = oracle.grad_epilogue(g, mask)
    got = G.grad_epilogue(g, mask, oracle.FL_16_9)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    got2 = G.grad_epilogue(g, mask, oracle.FL_16_9, in_place=True)
    assert np.array_equal(got2.view(np.uint32), want.view(np.uint32))
    got3 = G.grad_epilogue(g, None, 1.0)
    assert np.array_equal(got3.view(np.uint32), oracle.grad_epilogue(g, None, 1.0).view(np.uint32))
    got4 = G.grad_epilogue(g, mask, oracle.FL_16_9, bf16=True)
    assert np.array_equal(got4, synth.f32_to_bf16(want))


@pytest.mark.parametrize("tio", [(1, 32, 1), (50, 160, 7), (13, 1056, 300), (264, 2080, 96), (8, 64, 1000)])
def test_fwd_operands_match_the_two_quantizations(G, tio):
    # Algorithm 1 Forward: QuEST(H X) and QuEST(H W) from one launch, bit for bit the oracle's forward quantizer on each
    t, i, o = tio
    x = synth.small_matrix(400 + t, t, i, "outliers")
    w = synth.small_matrix(401 + o, o, i, "normal", 0.02)
    got = G.fwd_operands(x, w)
    for name, g, src in (("X", got[0], x), ("W", got[1], w)):
        want = oracle.quant_fwd(src)
        same(g[0], want[0], f"{name} codes")
        same(g[1], want[1], f"{name} scales")
        same(g[2], want[2], f"{name} mask")


@pytest.mark.parametrize("tio", [(32, 32, 32), (96, 160, 224), (288, 320, 352), (800, 544, 1056), (1024, 1280, 256)])
@pytest.mark.parametrize("rounding", [0, 1])
def test_bwd_operands_match_the_three_conversions(G, tio, rounding):
    # Algorithm 1 Backward: Q(dy^T), Q(X_q^T), Q(W_q^T) from one launch, bit for bit the oracle's three quantizations.
    # X_q and W_q come from the oracle's forward quantizer.
    t, i, o = tio
    dy = synth.small_matrix(300 + t, t, o, "normal", 1e-3)
    xq_codes, xq_scales, _ = oracle.quant_fwd(synth.small_matrix(301 + i, t, i, "heavy"))
    wq_codes, wq_scales, _ = oracle.quant_fwd(synth.small_matrix(302 + o, o, i, "normal", 0.02))
    sw, seed = 0xC3A5F00F ^ t, 2 ** 36 + 3 * o + rounding
    got = G.bwd_operands(dy, xq_codes, xq_scales, wq_codes, wq_scales, sw, seed, rounding)
    want = (oracle.quant_bwd_sr(dy, sw, seed, 2, rounding, transpose=True),
            oracle.requant_transpose_sr(xq_codes, xq_scales, sw, seed, 3, rounding),
            oracle.requant_transpose_sr(wq_codes, wq_scales, sw, seed, 1, rounding))
    for name, g, w in zip(("dy^T", "X_q^T", "W_q^T"), got, want):
        same(g[0], w[0], f"{name} codes")
        same(g[1], w[1], f"{name} scales")


def test_bwd_operands_with_no_tokens_still_convert_the_weights(G):
    # an empty dimension empties the conversions it belongs to, not the third one
    i, o = 64, 96
    wq_codes, wq_scales, _ = oracle.quant_fwd(synth.small_matrix(77, o, i, "normal", 0.02))
    sw, seed = 0x12345678, 99
    dummy = G.dev_empty((64,), np.uint8, 0)          # stands in for the pointers of the empty tensors (never read or written)
    wt_codes = G.dev_empty((i, o // 2), np.uint8, 0xEE)
    wt_scales = G.dev_empty((q_scale_bytes(i, o),), np.uint8, 0xFF)
    from paper_2505_14669_amd import binding as q
    q.check(q.quartet_bwd_operands(dummy, 0, i, o, dummy, dummy, G.to_dev(wq_codes), G.to_dev(scales_to_tiled(wq_scales)),
                                   sw, seed, 0, dummy, dummy, dummy, dummy, wt_codes, wt_scales))
    want = oracle.requant_transpose_sr(wq_codes, wq_scales, sw, seed, 1, 0)
    same(G.to_host(wt_codes, np.uint8), want[0], "W_q^T codes")
    same(scales_from_tiled(G.to_host(wt_scales, np.uint8), i, o), want[1], "W_q^T scales")
    assert int(dummy.sum()) == 0


def _check_linear(G, L, seed, roundings=(0, 1)):
    lin = G.Linear(L["x"], L["w"])
    lin.fwd()
    y_ref, ctx_ref = oracle.linear_fwd(L["x"], L["w"])
    ctx = lin.ctx_host()
    for key in ctx_ref:
        same(ctx[key], ctx_ref[key], f"ctx {key}")
    assert rel_fro(G.to_host(lin.y, np.float32), y_ref) < FRO_TOL
    xq, wq = (ctx_ref["xq_codes"], ctx_ref["xq_scales"]), (ctx_ref["wq_codes"], ctx_ref["wq_scales"])
    t, i, o = L["x"].shape[0], L["x"].shape[1], L["w"].shape[0]
    assert within_elem_bound(G.to_host(lin.y, np.float32), y_ref, indep.gemm_abs_products(*xq, *wq), i)
    dy = G.to_dev(L["dy"])
    sw = oracle.sign_word(seed)
    for rounding in roundings:
        lin.bwd(dy, seed, rounding)
        dx_ref, dw_ref = oracle.linear_bwd(L["dy"], ctx_ref, seed, rounding)
        assert rel_fro(G.to_host(lin.dx, np.float32), dx_ref) < FRO_TOL
        assert rel_fro(G.to_host(lin.dw, np.float32), dw_ref) < FRO_TOL
        # element by element: the bound needs the two products' sums of magnitudes, from the oracle's quantized operands
        gq = oracle.quant_bwd_sr(L["dy"], sw, seed, 0, rounding)
        wt = oracle.requant_transpose_sr(*wq, sw, seed, 1, rounding)
        assert within_elem_bound(G.to_host(lin.dx, np.float32), dx_ref, indep.gemm_abs_products(*gq, *wt), o,
                                 grad_scale=oracle.FL_16_9)
        gt = oracle.quant_bwd_sr(L["dy"], sw, seed, 2, rounding, transpose=True)
        xt = oracle.requant_transpose_sr(*xq, sw, seed, 3, rounding)
        assert within_elem_bound(G.to_host(lin.dw, np.float32), dw_ref, indep.gemm_abs_products(*gt, *xt), t,
                                 grad_scale=oracle.FL_16_9)


def test_linear_config1_full(G):
    # configuration 1: tokens 256, in 512, out 512, outlier channels, SR seed 0
    _check_linear(G, synth.make_layer(1, 0), seed=0)


def test_linear_ragged_small(G):
    L = dict(x=synth.small_matrix(1, 96, 160, "heavy"), w=synth.small_matrix(2, 224, 160, "normal", 0.02),
             dy=synth.small_matrix(3, 96, 224, "normal", 1e-3))
    _check_linear(G, L, seed=2 ** 33 + 17)
