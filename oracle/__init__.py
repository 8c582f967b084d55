"""CPU oracle for the Quartet MXFP4 linear-layer path (numpy front end of quartet_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product package never imports it, and it never imports
the product package.  bf16 tensors are numpy uint16 arrays holding the bit patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

G = 32
SR_BITS = 22
FL_16_9 = np.float32(16.0 / 9.0)

_lib = None


def lib():
    global _lib
    if _lib is None:
        # QUARTET_REF_LIB: another build of quartet_ref.c (the sanitizer leg of the tests loads an instrumented one)
        path = os.environ.get("QUARTET_REF_LIB") or _build.build(force=False)
        _lib = ctypes.CDLL(path)
        _declare(_lib)
    return _lib


_i64 = ctypes.c_int64
_u32 = ctypes.c_uint32
_u64 = ctypes.c_uint64
_p = ctypes.c_void_p


def _declare(L):
    L.quartet_ref_num_threads.restype = ctypes.c_int
    L.quartet_ref_set_num_threads.argtypes = [ctypes.c_int]
    L.quartet_ref_e2m1_decode.restype = ctypes.c_double
    L.quartet_ref_e2m1_decode.argtypes = [ctypes.c_uint8]
    L.quartet_ref_e8m0_decode.restype = ctypes.c_double
    L.quartet_ref_e8m0_decode.argtypes = [ctypes.c_uint8]
    L.quartet_ref_e2m1_rtn.restype = ctypes.c_uint8
    L.quartet_ref_e2m1_rtn.argtypes = [ctypes.c_float]
    L.quartet_ref_e2m1_sr.restype = ctypes.c_uint8
    L.quartet_ref_e2m1_sr.argtypes = [ctypes.c_float, _u32]
    L.quartet_ref_philox4x32_10.argtypes = [_p, _p, _p]
    L.quartet_ref_sr_draw.restype = _u32
    L.quartet_ref_sr_draw.argtypes = [_u64, _u32, _u64]
    L.quartet_ref_sr_draws.argtypes = [_u64, _u32, _u64, _i64, _p]
    L.quartet_ref_sign_word.restype = _u32
    L.quartet_ref_sign_word.argtypes = [_u64]
    L.quartet_ref_hadamard32.argtypes = [_p, _u32]
    L.quartet_ref_quant_fwd.argtypes = [_p, _i64, _i64, _i64, ctypes.c_int, _p, _p, _p]
    L.quartet_ref_quant_fwd_rows.argtypes = [_p, _i64, _i64, _i64, ctypes.c_int, _i64, _i64, _p, _p, _p]
    L.quartet_ref_quant_bwd_sr_rows.argtypes = [_p, _i64, _i64, _i64, ctypes.c_int, _u32, _u64, _u32,
                                                ctypes.c_int, _i64, _i64, _p, _p]
    L.quartet_ref_requant_transpose_sr_rows.argtypes = [_p, _p, _i64, _i64, _u32, _u64, _u32,
                                                        ctypes.c_int, _i64, _i64, _p, _p]
    L.quartet_ref_quant_bwd_sr.argtypes = [_p, _i64, _i64, _i64, ctypes.c_int, _u32, _u64, _u32,
                                           ctypes.c_int, _p, _p]
    L.quartet_ref_requant_transpose_sr.argtypes = [_p, _p, _i64, _i64, _u32, _u64, _u32,
                                                   ctypes.c_int, _p, _p]
    L.quartet_ref_mxfp4_dequant.argtypes = [_p, _p, _i64, _i64, _p]
    L.quartet_ref_mxfp4_gemm_rows.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, ctypes.c_double,
                                              _i64, _i64, _p]
    L.quartet_ref_e4m3_decode.restype = ctypes.c_double
    L.quartet_ref_e4m3_decode.argtypes = [ctypes.c_uint8]
    L.quartet_ref_e4m3_rtn.restype = ctypes.c_uint8
    L.quartet_ref_e4m3_rtn.argtypes = [ctypes.c_float]
    L.quartet_ref_mxfp8_quant.argtypes = [_p, _i64, _i64, _i64, _p, _p]
    L.quartet_ref_mxfp8_dequant.argtypes = [_p, _p, _i64, _i64, _p]
    L.quartet_ref_mxfp8_gemm.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, ctypes.c_double, _p]
    L.quartet_ref_grad_epilogue.argtypes = [_p, _p, _i64, _i64, ctypes.c_float, _p]
    L.quartet_ref_linear_fwd.argtypes = [_p, _p, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _p]
    L.quartet_ref_linear_bwd.argtypes = [_p, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _u64,
                                         ctypes.c_int, _p, _p]
    ci = ctypes.c_int
    L.quartet_ref_sign_words.argtypes = [_u64, _p]
    L.quartet_ref_hadamard.argtypes = [_p, ci, _p]
    L.quartet_ref_quant_fwd_block.argtypes = [_p, _i64, _i64, _i64, ci, ci, _p, _p, _p]
    L.quartet_ref_quant_bwd_sr_block.argtypes = [_p, _i64, _i64, _i64, ci, ci, _p, _u64, _u32, ci, _p, _p]
    L.quartet_ref_requant_transpose_sr_block.argtypes = [_p, _p, _i64, _i64, ci, _p, _u64, _u32, ci, _p, _p]
    L.quartet_ref_grad_epilogue_block.argtypes = [_p, _p, _i64, _i64, ci, ctypes.c_float, _p]
    L.quartet_ref_linear_fwd_block.argtypes = [_p, _p, _i64, _i64, _i64, ci, _p, _p, _p, _p, _p, _p, _p]
    L.quartet_ref_linear_bwd_block.argtypes = [_p, _i64, _i64, _i64, ci, _p, _p, _p, _p, _p, _p, _u64,
                                               ci, _p, _p]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ok(rc, name):
    if rc != 0:
        raise ValueError(f"oracle {name} failed with code {rc}")


def num_threads():
    return lib().quartet_ref_num_threads()


def set_num_threads(n):
    lib().quartet_ref_set_num_threads(int(n))


# ---------------------------------------------------------------- scalars

def e2m1_decode(code):
    return lib().quartet_ref_e2m1_decode(int(code) & 0xFF)


def e8m0_decode(b):
    return lib().quartet_ref_e8m0_decode(int(b) & 0xFF)


def e2m1_rtn(v):
    return lib().quartet_ref_e2m1_rtn(float(np.float32(v)))


def e2m1_sr(v, r):
    return lib().quartet_ref_e2m1_sr(float(np.float32(v)), int(r))


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().quartet_ref_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def sr_draw(seed, stream_id, L):
    return lib().quartet_ref_sr_draw(int(seed), int(stream_id), int(L))


def sr_draws(seed, stream_id, L0, count):
    """The 22-bit draws of positions L0 .. L0 + count - 1 (uint32 array)."""
    out = np.zeros(int(count), dtype=np.uint32)
    lib().quartet_ref_sr_draws(int(seed), int(stream_id), int(L0), int(count), _ptr(out))
    return out


def sign_word(seed):
    return lib().quartet_ref_sign_word(int(seed))


def hadamard32(v, sign_word=0):
    """H_32 (d . v) for one group of 32 fp32 values; returns a new array."""
    out = np.array(v, dtype=np.float32).reshape(32).copy()
    lib().quartet_ref_hadamard32(_ptr(out), int(sign_word))
    return out


# ------------------------------------------------------------- quantizers

def _logical_shape(x, transpose):
    if x.ndim != 2:
        raise ValueError("x must be 2-D")
    return (x.shape[1], x.shape[0]) if transpose else (x.shape[0], x.shape[1])


def _slab(rows_range, rows):
    r0, r1 = (0, rows) if rows_range is None else rows_range
    return int(r0), int(r1)


def quant_fwd(x_bf16, transpose=False, want_mask=True, rows_range=None):
    """Forward (QuEST) quantizer.  Returns codes [rows,k/2] u8, scales [rows,k/32] u8, mask u32.
    rows_range=(begin,end) computes only those logical rows and returns just that slab."""
    x = _c(x_bf16, np.uint16)
    rows, k = _logical_shape(x, transpose)
    r0, r1 = _slab(rows_range, rows)
    n = r1 - r0
    # slab outputs are written at full-matrix positions: hand the C code pointers shifted back by r0 rows
    cs = np.zeros((n, k // 2), dtype=np.uint8)
    ss = np.zeros((n, k // G), dtype=np.uint8)
    ms = np.zeros((n, k // G), dtype=np.uint32) if want_mask else None
    off = lambda a, per_row: None if a is None else ctypes.c_void_p(a.ctypes.data - r0 * per_row * a.itemsize)
    _ok(lib().quartet_ref_quant_fwd_rows(_ptr(x), rows, k, x.shape[1], int(bool(transpose)), r0, r1,
                                         off(cs, k // 2), off(ss, k // G), off(ms, k // G)), "quant_fwd")
    return cs, ss, ms


def quant_bwd_sr(x_bf16, sign_word, seed, stream_id, rounding=0, transpose=False, rows_range=None):
    """Backward quantizer (randomized Hadamard, AbsMax, 3/4, SR or RTN).  rows_range as in quant_fwd."""
    x = _c(x_bf16, np.uint16)
    rows, k = _logical_shape(x, transpose)
    r0, r1 = _slab(rows_range, rows)
    n = r1 - r0
    codes = np.zeros((n, k // 2), dtype=np.uint8)
    scales = np.zeros((n, k // G), dtype=np.uint8)
    off = lambda a, per_row: ctypes.c_void_p(a.ctypes.data - r0 * per_row * a.itemsize)
    _ok(lib().quartet_ref_quant_bwd_sr_rows(_ptr(x), rows, k, x.shape[1], int(bool(transpose)),
                                            int(sign_word), int(seed), int(stream_id), int(rounding), r0, r1,
                                            off(codes, k // 2), off(scales, k // G)), "quant_bwd_sr")
    return codes, scales


def requant_transpose_sr(src_codes, src_scales, sign_word, seed, stream_id, rounding=0, rows_range=None):
    """src is MXFP4 [k, rows] (codes [k, rows/2]); returns the backward quantization of its
    decoded transpose: codes [rows, k/2], scales [rows, k/32].  rows_range as in quant_fwd."""
    sc = _c(src_codes, np.uint8)
    ss = _c(src_scales, np.uint8)
    k, rows = sc.shape[0], sc.shape[1] * 2
    r0, r1 = _slab(rows_range, rows)
    n = r1 - r0
    codes = np.zeros((n, k // 2), dtype=np.uint8)
    scales = np.zeros((n, k // G), dtype=np.uint8)
    off = lambda a, per_row: ctypes.c_void_p(a.ctypes.data - r0 * per_row * a.itemsize)
    _ok(lib().quartet_ref_requant_transpose_sr_rows(_ptr(sc), _ptr(ss), rows, k, int(sign_word),
                                                    int(seed), int(stream_id), int(rounding), r0, r1,
                                                    off(codes, k // 2), off(scales, k // G)),
        "requant_transpose_sr")
    return codes, scales


def mxfp4_dequant(codes, scales):
    c = _c(codes, np.uint8)
    s = _c(scales, np.uint8)
    rows, k = c.shape[0], c.shape[1] * 2
    out = np.zeros((rows, k), dtype=np.float64)
    _ok(lib().quartet_ref_mxfp4_dequant(_ptr(c), _ptr(s), rows, k, _ptr(out)), "mxfp4_dequant")
    return out


def mxfp4_gemm(a_codes, a_scales, b_codes, b_scales, alpha=1.0, rows=None):
    """alpha * dec(A) dec(B)^T in fp64.  rows=(begin,end) computes only that slab of D (other rows
    are left zero)."""
    ac, as_ = _c(a_codes, np.uint8), _c(a_scales, np.uint8)
    bc, bs = _c(b_codes, np.uint8), _c(b_scales, np.uint8)
    m, k = ac.shape[0], ac.shape[1] * 2
    n = bc.shape[0]
    if bc.shape[1] * 2 != k:
        raise ValueError("inner dimensions differ")
    r0, r1 = (0, m) if rows is None else rows
    d = np.zeros((m, n), dtype=np.float64)
    _ok(lib().quartet_ref_mxfp4_gemm_rows(_ptr(ac), _ptr(as_), _ptr(bc), _ptr(bs), m, n, k,
                                          float(alpha), r0, r1, _ptr(d)), "mxfp4_gemm")
    return d


def e4m3_decode(code):
    return lib().quartet_ref_e4m3_decode(int(code) & 0xFF)


def e4m3_rtn(v):
    return lib().quartet_ref_e4m3_rtn(float(np.float32(v)))


def mxfp8_quant(x):
    """bf16 [rows, k] (uint16 bit patterns) -> (codes [rows, k] E4M3 bytes, scales [rows, k/32] E8M0 bytes)."""
    xx = _c(x, np.uint16)
    rows, k = xx.shape
    codes = np.zeros((rows, k), dtype=np.uint8)
    scales = np.zeros((rows, k // G), dtype=np.uint8)
    _ok(lib().quartet_ref_mxfp8_quant(_ptr(xx), rows, k, k, _ptr(codes), _ptr(scales)), "mxfp8_quant")
    return codes, scales


def mxfp8_dequant(codes, scales):
    c, s = _c(codes, np.uint8), _c(scales, np.uint8)
    rows, k = c.shape
    out = np.zeros((rows, k), dtype=np.float64)
    _ok(lib().quartet_ref_mxfp8_dequant(_ptr(c), _ptr(s), rows, k, _ptr(out)), "mxfp8_dequant")
    return out


def mxfp8_gemm(a_codes, a_scales, b_codes, b_scales, alpha=1.0):
    ac, as_ = _c(a_codes, np.uint8), _c(a_scales, np.uint8)
    bc, bs = _c(b_codes, np.uint8), _c(b_scales, np.uint8)
    m, k = ac.shape
    n = bc.shape[0]
    if bc.shape[1] != k:
        raise ValueError("inner dimensions differ")
    d = np.zeros((m, n), dtype=np.float64)
    _ok(lib().quartet_ref_mxfp8_gemm(_ptr(ac), _ptr(as_), _ptr(bc), _ptr(bs), m, n, k, float(alpha), _ptr(d)), "mxfp8_gemm")
    return d


def grad_epilogue(g, mask, scale=FL_16_9):
    gg = _c(g, np.float32)
    mm = None if mask is None else _c(mask, np.uint32)
    m, n = gg.shape
    out = np.zeros((m, n), dtype=np.float32)
    _ok(lib().quartet_ref_grad_epilogue(_ptr(gg), _ptr(mm), m, n, float(np.float32(scale)),
                                        _ptr(out)), "grad_epilogue")
    return out


# ---------------------------------------------------------- linear fwd/bwd

def linear_fwd(x_bf16, w_bf16):
    """Algorithm 1 Forward.  Returns y fp32 [tokens,out] and ctx dict."""
    x = _c(x_bf16, np.uint16)
    w = _c(w_bf16, np.uint16)
    tokens, in_f = x.shape
    out_f = w.shape[0]
    if w.shape[1] != in_f:
        raise ValueError("in features differ")
    y = np.zeros((tokens, out_f), dtype=np.float32)
    ctx = dict(
        xq_codes=np.zeros((tokens, in_f // 2), np.uint8), xq_scales=np.zeros((tokens, in_f // G), np.uint8),
        x_mask=np.zeros((tokens, in_f // G), np.uint32),
        wq_codes=np.zeros((out_f, in_f // 2), np.uint8), wq_scales=np.zeros((out_f, in_f // G), np.uint8),
        w_mask=np.zeros((out_f, in_f // G), np.uint32))
    _ok(lib().quartet_ref_linear_fwd(_ptr(x), _ptr(w), tokens, in_f, out_f, _ptr(y),
                                     _ptr(ctx["xq_codes"]), _ptr(ctx["xq_scales"]), _ptr(ctx["x_mask"]),
                                     _ptr(ctx["wq_codes"]), _ptr(ctx["wq_scales"]), _ptr(ctx["w_mask"])),
        "linear_fwd")
    return y, ctx


def linear_bwd(dy_bf16, ctx, seed, rounding=0):
    """Algorithm 1 Backward.  Returns dx fp32 [tokens,in], dw fp32 [out,in]."""
    dy = _c(dy_bf16, np.uint16)
    tokens, out_f = dy.shape
    in_f = ctx["xq_codes"].shape[1] * 2
    dx = np.zeros((tokens, in_f), dtype=np.float32)
    dw = np.zeros((out_f, in_f), dtype=np.float32)
    _ok(lib().quartet_ref_linear_bwd(_ptr(dy), tokens, in_f, out_f,
                                     _ptr(ctx["xq_codes"]), _ptr(ctx["xq_scales"]), _ptr(ctx["x_mask"]),
                                     _ptr(ctx["wq_codes"]), _ptr(ctx["wq_scales"]), _ptr(ctx["w_mask"]),
                                     int(seed), int(rounding), _ptr(dx), _ptr(dw)), "linear_bwd")
    return dx, dw


# ------------------------------------------ larger Hadamard blocks (32, 64, 128, 256)

def sign_words(seed):
    """The eight sign words of a backward pass (element i of a block negated iff bit i%32 of word i/32)."""
    out = np.zeros(8, dtype=np.uint32)
    lib().quartet_ref_sign_words(int(seed), _ptr(out))
    return out


def hadamard(v, block, sign_words=None):
    """H_block (d . v) for one block of fp32 values; returns a new array."""
    out = np.array(v, dtype=np.float32).reshape(block).copy()
    sw = None if sign_words is None else _c(sign_words, np.uint32)
    _ok(lib().quartet_ref_hadamard(_ptr(out), int(block), _ptr(sw)), "hadamard")
    return out


def quant_fwd_block(x_bf16, block, transpose=False, want_mask=True):
    x = _c(x_bf16, np.uint16)
    rows, k = _logical_shape(x, transpose)
    cs = np.zeros((rows, k // 2), dtype=np.uint8)
    ss = np.zeros((rows, k // G), dtype=np.uint8)
    ms = np.zeros((rows, k // G), dtype=np.uint32) if want_mask else None
    _ok(lib().quartet_ref_quant_fwd_block(_ptr(x), rows, k, x.shape[1], int(bool(transpose)), int(block),
                                          _ptr(cs), _ptr(ss), _ptr(ms)), "quant_fwd_block")
    return cs, ss, ms


def quant_bwd_sr_block(x_bf16, block, sign_words, seed, stream_id, rounding=0, transpose=False):
    x = _c(x_bf16, np.uint16)
    rows, k = _logical_shape(x, transpose)
    sw = _c(sign_words, np.uint32)
    codes = np.zeros((rows, k // 2), dtype=np.uint8)
    scales = np.zeros((rows, k // G), dtype=np.uint8)
    _ok(lib().quartet_ref_quant_bwd_sr_block(_ptr(x), rows, k, x.shape[1], int(bool(transpose)), int(block),
                                             _ptr(sw), int(seed), int(stream_id), int(rounding),
                                             _ptr(codes), _ptr(scales)), "quant_bwd_sr_block")
    return codes, scales


def requant_transpose_sr_block(src_codes, src_scales, block, sign_words, seed, stream_id, rounding=0):
    sc = _c(src_codes, np.uint8)
    ss = _c(src_scales, np.uint8)
    sw = _c(sign_words, np.uint32)
    k, rows = sc.shape[0], sc.shape[1] * 2
    codes = np.zeros((rows, k // 2), dtype=np.uint8)
    scales = np.zeros((rows, k // G), dtype=np.uint8)
    _ok(lib().quartet_ref_requant_transpose_sr_block(_ptr(sc), _ptr(ss), rows, k, int(block), _ptr(sw),
                                                     int(seed), int(stream_id), int(rounding),
                                                     _ptr(codes), _ptr(scales)), "requant_transpose_sr_block")
    return codes, scales


def grad_epilogue_block(g, mask, block, scale=FL_16_9):
    gg = _c(g, np.float32)
    mm = None if mask is None else _c(mask, np.uint32)
    m, n = gg.shape
    out = np.zeros((m, n), dtype=np.float32)
    _ok(lib().quartet_ref_grad_epilogue_block(_ptr(gg), _ptr(mm), m, n, int(block), float(np.float32(scale)),
                                              _ptr(out)), "grad_epilogue_block")
    return out


def linear_fwd_block(x_bf16, w_bf16, block):
    x = _c(x_bf16, np.uint16)
    w = _c(w_bf16, np.uint16)
    tokens, in_f = x.shape
    out_f = w.shape[0]
    if w.shape[1] != in_f:
        raise ValueError("in features differ")
    y = np.zeros((tokens, out_f), dtype=np.float32)
    ctx = dict(
        xq_codes=np.zeros((tokens, in_f // 2), np.uint8), xq_scales=np.zeros((tokens, in_f // G), np.uint8),
        x_mask=np.zeros((tokens, in_f // G), np.uint32),
        wq_codes=np.zeros((out_f, in_f // 2), np.uint8), wq_scales=np.zeros((out_f, in_f // G), np.uint8),
        w_mask=np.zeros((out_f, in_f // G), np.uint32))
    _ok(lib().quartet_ref_linear_fwd_block(_ptr(x), _ptr(w), tokens, in_f, out_f, int(block), _ptr(y),
                                           _ptr(ctx["xq_codes"]), _ptr(ctx["xq_scales"]), _ptr(ctx["x_mask"]),
                                           _ptr(ctx["wq_codes"]), _ptr(ctx["wq_scales"]), _ptr(ctx["w_mask"])),
        "linear_fwd_block")
    return y, ctx


def linear_bwd_block(dy_bf16, ctx, block, seed, rounding=0):
    dy = _c(dy_bf16, np.uint16)
    tokens, out_f = dy.shape
    in_f = ctx["xq_codes"].shape[1] * 2
    dx = np.zeros((tokens, in_f), dtype=np.float32)
    dw = np.zeros((out_f, in_f), dtype=np.float32)
    _ok(lib().quartet_ref_linear_bwd_block(_ptr(dy), tokens, in_f, out_f, int(block),
                                           _ptr(ctx["xq_codes"]), _ptr(ctx["xq_scales"]), _ptr(ctx["x_mask"]),
                                           _ptr(ctx["wq_codes"]), _ptr(ctx["wq_scales"]), _ptr(ctx["w_mask"]),
                                           int(seed), int(rounding), _ptr(dx), _ptr(dw)), "linear_bwd_block")
    return dx, dw
