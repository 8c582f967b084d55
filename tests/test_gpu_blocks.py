"""GPU parity of the larger Hadamard blocks (64, 128, 256 elements; MXFP4 group 32): the HIP path
through the C ABI against the oracle's *_block functions.  Same bars as for blocks of 32: codes, scale
bytes and mask words bit-exact, GEMM-derived outputs within a relative Frobenius error of 1e-5."""
import numpy as np
import pytest

import indep
import oracle
from paper_2505_14669_amd import synth

pytestmark = pytest.mark.gpu

FRO_TOL = 1e-5
BLOCKS = (64, 128, 256)


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def same(a, b, what):
    a, b = np.asarray(a), np.asarray(b)
    assert a.shape == b.shape, (what, a.shape, b.shape)
    bad = np.argwhere(a != b)
    assert bad.size == 0, f"{what}: {len(bad)} mismatches, first at {bad[0]}: got {a[tuple(bad[0])]:#x} want {b[tuple(bad[0])]:#x}"


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


# several row blocks, a ragged last K-quad (k not a multiple of 256 where the block allows), a wide case
def shapes_for(block):
    return [(1, block), (37, 3 * block), (129, 8 * block + block), (256, 1024)]


@pytest.mark.parametrize("block", BLOCKS)
@pytest.mark.parametrize("kind", ["normal", "outliers", "zeros"])
def test_quant_fwd_block_rows(G, block, kind):
    for i, (rows, k) in enumerate(shapes_for(block)):
        x = synth.small_matrix(100 + i, rows, k, kind)
        want = oracle.quant_fwd_block(x, block)
        got = G.quant_fwd_block(x, block)
        for a, b, what in zip(got, want, ("codes", "scales", "mask")):
            same(a, b, f"fwd block {block} {rows}x{k} {kind} {what}")


@pytest.mark.parametrize("block", BLOCKS)
@pytest.mark.parametrize("rounding", [0, 1])
def test_quant_bwd_block_rows(G, block, rounding):
    sw = oracle.sign_words(11)
    for i, (rows, k) in enumerate(shapes_for(block)):
        x = synth.small_matrix(200 + i, rows, k, "heavy")
        want = oracle.quant_bwd_sr_block(x, block, sw, 11, 2, rounding)
        got = G.quant_bwd_sr_block(x, block, sw, 11, 2, rounding)
        same(got[0], want[0], f"bwd block {block} {rows}x{k} codes")
        same(got[1], want[1], f"bwd block {block} {rows}x{k} scales")


@pytest.mark.parametrize("block", BLOCKS)
def test_quant_block_transposed(G, block):
    sw = oracle.sign_words(12)
    # stored [k x rows]: k spans several blocks and a ragged K-quad, rows a ragged column tile
    for i, (k, rows) in enumerate([(block, 8), (3 * block, 136), (8 * block + block, 264), (1024, 128)]):
        x = synth.small_matrix(300 + i, k, rows, "normal")
        for rounding in (0, 1):
            want = oracle.quant_bwd_sr_block(x, block, sw, 12, 1, rounding, transpose=True)
            got = G.quant_bwd_sr_block(x, block, sw, 12, 1, rounding, transpose=True)
            same(got[0], want[0], f"bwd^T block {block} {k}x{rows} codes r={rounding}")
            same(got[1], want[1], f"bwd^T block {block} {k}x{rows} scales r={rounding}")
        want = oracle.quant_fwd_block(x, block, transpose=True)
        got = G.quant_fwd_block(x, block, transpose=True)
        for a, b, what in zip(got, want, ("codes", "scales", "mask")):
            same(a, b, f"fwd^T block {block} {k}x{rows} {what}")


@pytest.mark.parametrize("block", BLOCKS)
def test_requant_transpose_block(G, block):
    sw = oracle.sign_words(13)
    for i, (k, rows) in enumerate([(block, 32), (3 * block, 96), (8 * block + block, 288), (512, 256)]):
        src = synth.small_matrix(400 + i, k, rows, "outliers")
        c, s, _ = oracle.quant_fwd(src)                   # MXFP4 [k x rows], groups along rows
        for rounding in (0, 1):
            want = oracle.requant_transpose_sr_block(c, s, block, sw, 13, 3, rounding)
            got = G.requant_transpose_sr_block(c, s, block, sw, 13, 3, rounding)
            same(got[0], want[0], f"requant block {block} {k}x{rows} codes r={rounding}")
            same(got[1], want[1], f"requant block {block} {k}x{rows} scales r={rounding}")


@pytest.mark.parametrize("block", BLOCKS)
def test_grad_epilogue_block(G, block):
    for m, n in [(1, block), (6, 3 * block), (77, 2 * block), (64, 1024)]:
        rng = np.random.default_rng(m + n)
        g = rng.standard_normal((m, n)).astype(np.float32)
        mask = rng.integers(0, 2 ** 32, size=(m, n // 32), dtype=np.uint32)
        want = oracle.grad_epilogue_block(g, mask, block)
        got = G.grad_epilogue_block(g, mask, block, oracle.FL_16_9)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        got_bf = G.grad_epilogue_block(g, mask, block, oracle.FL_16_9, bf16=True)
        assert np.array_equal(got_bf, synth.f32_to_bf16(want))
        got_nm = G.grad_epilogue_block(g, None, block, 1.0)
        assert np.array_equal(got_nm.view(np.uint32), oracle.grad_epilogue_block(g, None, block, 1.0).view(np.uint32))


@pytest.fixture(params=["auto", "0", "1", "2"])
def gemm_variant(request, G):
    # every tile shape of the GEMM kernel; a block of 128 columns does not fit the 64-column wave tile of variant 2,
    # the library switches to variant 1 by itself
    G.q.check(G.q.quartet_debug_set_gemm_plan(-1 if request.param == "auto" else int(request.param), 0))
    yield request.param
    G.q.check(G.q.quartet_debug_set_gemm_plan(-1, 0))


@pytest.mark.parametrize("block", (64, 128))
@pytest.mark.parametrize("mnk", [(1, 128, 32), (130, 256, 96), (257, 384, 160), (64, 1280, 1024), (520, 640, 800)])
def test_gemm_grad_block_fused(G, mnk, block, gemm_variant):
    # GEMM_LP with the gradient epilogue for Hadamard blocks of 64 or 128 columns in the same kernel against the
    # oracle's two steps, and bit for bit against the stand-alone epilogue kernel on the library's own product
    m, n, k = mnk
    rng = np.random.default_rng(m * 1000 + n + block)
    ac = rng.integers(0, 256, size=(m, k // 2), dtype=np.uint8)
    bc = rng.integers(0, 256, size=(n, k // 2), dtype=np.uint8)
    asc = rng.integers(117, 137, size=(m, k // 32), dtype=np.uint8)
    bsc = rng.integers(117, 137, size=(n, k // 32), dtype=np.uint8)
    mask = rng.integers(0, 2 ** 32, size=(m, n // 32), dtype=np.uint32)
    acc = oracle.mxfp4_gemm(ac, asc, bc, bsc).astype(np.float32)
    want = oracle.grad_epilogue_block(acc, mask, block)
    got = G.gemm_grad_block(ac, asc, bc, bsc, block, mask, oracle.FL_16_9)
    assert rel_fro(got, want) < FRO_TOL
    # element by element: (K/64 + 3) 2^-23 sum |a||b| per product element, carried through the block's Hadamard transform
    absp = indep.gemm_abs_products(ac, asc, bc, bsc)
    bound = indep.grad_elem_bound(indep.gemm_elem_bound(absp, k), absp, oracle.FL_16_9, block)
    assert indep.worst_excess(got, want, bound) <= 1.0
    plain = G.gemm(ac, asc, bc, bsc)
    two_steps = G.grad_epilogue_block(plain, mask, block, oracle.FL_16_9)
    assert np.array_equal(got.view(np.uint32), two_steps.view(np.uint32))
    got_bf = G.gemm_grad_block(ac, asc, bc, bsc, block, mask, oracle.FL_16_9, bf16=True)
    assert np.array_equal(got_bf, synth.f32_to_bf16(got))
    got_nomask = G.gemm_grad_block(ac, asc, bc, bsc, block, None, 1.0)
    assert rel_fro(got_nomask, oracle.grad_epilogue_block(acc, None, block, 1.0)) < FRO_TOL
    bound = indep.grad_elem_bound(indep.gemm_elem_bound(absp, k), absp, 1.0, block)
    assert indep.worst_excess(got_nomask, oracle.grad_epilogue_block(acc, None, block, 1.0), bound) <= 1.0


@pytest.mark.parametrize("block", BLOCKS)
def test_linear_block(G, block):
    t, i, o = 256, 512, 768
    L = dict(x=synth.small_matrix(1, t, i, "outliers"), w=synth.small_matrix(2, o, i, "normal", 0.02),
             dy=synth.small_matrix(3, t, o, "normal", 1e-3))
    lin = G.LinearBlock(L["x"], L["w"], block)
    lin.fwd()
    y_ref, ctx_ref = oracle.linear_fwd_block(L["x"], L["w"], block)
    ctx = lin.ctx_host()
    for key in ctx_ref:
        same(ctx[key], ctx_ref[key], f"ctx {key}")
    assert rel_fro(G.to_host(lin.y, np.float32), y_ref) < FRO_TOL
    xq, wq = (ctx_ref["xq_codes"], ctx_ref["xq_scales"]), (ctx_ref["wq_codes"], ctx_ref["wq_scales"])
    assert indep.worst_excess(G.to_host(lin.y, np.float32), y_ref,
                              indep.gemm_elem_bound(indep.gemm_abs_products(*xq, *wq), i)) <= 1.0
    dy = G.to_dev(L["dy"])
    seed = 2 ** 40 + 5
    sws = oracle.sign_words(seed)
    for rounding in (0, 1):
        lin.bwd(dy, seed, rounding)
        dx_ref, dw_ref = oracle.linear_bwd_block(L["dy"], ctx_ref, block, seed, rounding)
        assert rel_fro(G.to_host(lin.dx, np.float32), dx_ref) < FRO_TOL
        assert rel_fro(G.to_host(lin.dw, np.float32), dw_ref) < FRO_TOL
        # element by element, with the sums of magnitudes of the two products from the oracle's quantized operands
        gq = oracle.quant_bwd_sr_block(L["dy"], block, sws, seed, 0, rounding)
        wt = oracle.requant_transpose_sr_block(*wq, block, sws, seed, 1, rounding)
        absp = indep.gemm_abs_products(*gq, *wt)
        assert indep.worst_excess(G.to_host(lin.dx, np.float32), dx_ref,
                                  indep.grad_elem_bound(indep.gemm_elem_bound(absp, o), absp, oracle.FL_16_9, block)) <= 1.0
        gt = oracle.quant_bwd_sr_block(L["dy"], block, sws, seed, 2, rounding, transpose=True)
        xt = oracle.requant_transpose_sr_block(*xq, block, sws, seed, 3, rounding)
        absp = indep.gemm_abs_products(*gt, *xt)
        assert indep.worst_excess(G.to_host(lin.dw, np.float32), dw_ref,
                                  indep.grad_elem_bound(indep.gemm_elem_bound(absp, t), absp, oracle.FL_16_9, block)) <= 1.0


def test_block_32_entry_points_are_the_plain_ones(G):
    x = synth.small_matrix(5, 64, 256, "normal")
    sw = oracle.sign_words(3)
    a = G.quant_bwd_sr_block(x, 32, sw, 3, 0, 0)
    b = G.quant_bwd_sr(x, int(sw[0]), 3, 0, 0)
    same(a[0], b[0], "codes")
    same(a[1], b[1], "scales")
    import paper_2505_14669_amd.binding as q
    assert q.quartet_sign_words(3) == [int(w) for w in sw]
    assert q.quartet_sign_words(3)[0] == q.quartet_sign_word(3)


def test_block_argument_errors(G):
    import paper_2505_14669_amd.binding as q
    x = G.to_dev(synth.small_matrix(6, 8, 96, "normal"))
    codes = G.dev_empty((8, 48), np.uint8)
    scales = G.dev_empty((256,), np.uint8)
    assert q.quartet_quant_fwd_block(x, 8, 96, 96, 0, 64, codes, scales, None) == q.QUARTET_EINVAL   # 96 % 64
    assert q.quartet_quant_fwd_block(x, 8, 96, 96, 0, 48, codes, scales, None) == q.QUARTET_EINVAL   # unsupported block
    assert q.quartet_linear_workspace_bytes_block(64, 64, 96, 64) == 0
    assert q.quartet_linear_workspace_bytes_block(256, 256, 256, 256) > q.quartet_linear_workspace_bytes(256, 256, 256)
    assert q.quartet_linear_workspace_bytes_block(256, 256, 256, 128) == q.quartet_linear_workspace_bytes(256, 256, 256)
