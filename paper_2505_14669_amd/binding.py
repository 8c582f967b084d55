"""ctypes binding of the HIP library's C ABI (include/quartet.h).

Argument marshalling only: every function has the name and argument order of its C entry point,
takes torch CUDA tensors (or raw device addresses) for the pointer arguments and returns the C
return code.  `check()` turns a non-zero code into an exception.  PyTorch is used for device
memory and streams only; there is no CPU fallback, and importing this module fails loudly if the
library has not been built (python -m paper_2505_14669_amd.build, or __graft_entry__.build()).
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libquartet.so")

QUARTET_OK = 0
QUARTET_EINVAL = -1
QUARTET_ENOTSUP = -2
QUARTET_EHIP = -3
QUARTET_DTYPE_F32 = 0
QUARTET_DTYPE_BF16 = 1
QUARTET_ROUND_STOCHASTIC = 0
QUARTET_ROUND_NEAREST = 1

EXPORTS = [
    "quartet_last_hip_error", "quartet_sr_bits", "quartet_sign_word",
    "quartet_profile_enable", "quartet_profile_kinds", "quartet_profile_read", "quartet_scale_bytes",
    "quartet_profile_clock", "quartet_wall_clock_khz", "quartet_probe_mfma_ceiling",
    "quartet_quant_fwd", "quartet_quant_bwd_sr", "quartet_requant_transpose_sr", "quartet_fwd_operands", "quartet_bwd_operands",
    "quartet_mxfp4_gemm", "quartet_debug_set_gemm_plan", "quartet_mxfp4_gemm_grad", "quartet_mxfp4_gemm_grad_pair", "quartet_mxfp8_quant", "quartet_mxfp8_gemm", "quartet_grad_epilogue", "quartet_mxfp4_dequant",
    "quartet_linear_fwd", "quartet_linear_workspace_bytes", "quartet_linear_bwd",
    "quartet_static_scratch_bytes", "quartet_linear_bwd_static",
    "quartet_sign_words", "quartet_quant_fwd_block", "quartet_quant_bwd_sr_block",
    "quartet_requant_transpose_sr_block", "quartet_mxfp4_gemm_grad_block", "quartet_grad_epilogue_block", "quartet_linear_fwd_block",
    "quartet_linear_workspace_bytes_block", "quartet_linear_bwd_block",
]

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build the HIP library first "
                      "(python -m paper_2505_14669_amd.build); there is no fallback path")

_lib = ctypes.CDLL(LIB_PATH)

_i64, _u32, _u64, _p, _int, _f = (ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_void_p,
                                 ctypes.c_int, ctypes.c_float)
_lib.quartet_last_hip_error.restype = _int
_lib.quartet_sr_bits.restype = _int
_lib.quartet_profile_enable.argtypes = [_int]
_lib.quartet_profile_kinds.argtypes = [ctypes.c_uint]
_lib.quartet_profile_read.argtypes = [_p, _p, _int]
_lib.quartet_profile_clock.argtypes = [_p]
_lib.quartet_wall_clock_khz.restype = _int
_lib.quartet_probe_mfma_ceiling.argtypes = [_p, _p, _i64, _int, _p, _p, _p]
_lib.quartet_scale_bytes.restype = ctypes.c_size_t
_lib.quartet_scale_bytes.argtypes = [_i64, _i64]
_lib.quartet_sign_word.restype = _u32
_lib.quartet_sign_word.argtypes = [_u64]
_lib.quartet_quant_fwd.argtypes = [_p, _i64, _i64, _i64, _int, _p, _p, _p, _p]
_lib.quartet_quant_bwd_sr.argtypes = [_p, _i64, _i64, _i64, _int, _u32, _u64, _u32, _int, _p, _p, _p]
_lib.quartet_requant_transpose_sr.argtypes = [_p, _p, _i64, _i64, _u32, _u64, _u32, _int, _p, _p, _p]
_lib.quartet_fwd_operands.argtypes = [_p, _p, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _p]
_lib.quartet_bwd_operands.argtypes = [_p, _i64, _i64, _i64, _p, _p, _p, _p, _u32, _u64, _int, _p, _p, _p, _p, _p, _p, _p]
_lib.quartet_mxfp4_gemm.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, _f, _p, _int, _i64, _p]
_lib.quartet_debug_set_gemm_plan.argtypes = [_int, _int]
_lib.quartet_mxfp4_gemm_grad.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, _p, _f, _p, _int, _i64, _p]


class GemmGradArgs(ctypes.Structure):
    """quartet_gemm_grad_args: one product of quartet_mxfp4_gemm_grad_pair (host structure of device pointers and sizes)."""
    _fields_ = [("a_codes", _p), ("a_scales", _p), ("b_codes", _p), ("b_scales", _p),
                ("m", _i64), ("n", _i64), ("k", _i64), ("mask", _p), ("scale", _f), ("d", _p), ("ldd", _i64)]


_lib.quartet_mxfp4_gemm_grad_pair.argtypes = [ctypes.POINTER(GemmGradArgs), ctypes.POINTER(GemmGradArgs), _int, _p]
_lib.quartet_mxfp8_quant.argtypes = [_p, _i64, _i64, _i64, _p, _p, _p]
_lib.quartet_mxfp8_gemm.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, _f, _p, _int, _i64, _p]
_lib.quartet_grad_epilogue.argtypes = [_p, _p, _i64, _i64, _f, _p, _int, _p]
_lib.quartet_mxfp4_dequant.argtypes = [_p, _p, _i64, _i64, _p, _p]
_lib.quartet_linear_fwd.argtypes = [_p, _p, _i64, _i64, _i64, _p, _int, _p, _p, _p, _p, _p, _p, _p]
_lib.quartet_linear_workspace_bytes.restype = ctypes.c_size_t
_lib.quartet_linear_workspace_bytes.argtypes = [_i64, _i64, _i64]
_lib.quartet_linear_bwd.argtypes = [_p, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _u64, _int, _p, _p, _int,
                                    _p, ctypes.c_size_t, _p]
_lib.quartet_static_scratch_bytes.restype = ctypes.c_size_t
_lib.quartet_linear_bwd_static.argtypes = [_p, _i64, _i64, _i64, _p, _p, _p, _p, _p, _p, _u64, _int, _p, _p, _int, _p]
_lib.quartet_sign_words.argtypes = [_u64, _p]
_lib.quartet_quant_fwd_block.argtypes = [_p, _i64, _i64, _i64, _int, _int, _p, _p, _p, _p]
_lib.quartet_quant_bwd_sr_block.argtypes = [_p, _i64, _i64, _i64, _int, _int, _p, _u64, _u32, _int, _p, _p, _p]
_lib.quartet_requant_transpose_sr_block.argtypes = [_p, _p, _i64, _i64, _int, _p, _u64, _u32, _int, _p, _p, _p]
_lib.quartet_mxfp4_gemm_grad_block.argtypes = [_p, _p, _p, _p, _i64, _i64, _i64, _int, _p, _f, _p, _int, _i64, _p]
_lib.quartet_grad_epilogue_block.argtypes = [_p, _p, _i64, _i64, _int, _f, _p, _int, _p]
_lib.quartet_linear_fwd_block.argtypes = [_p, _p, _i64, _i64, _i64, _int, _p, _int, _p, _p, _p, _p, _p, _p, _p]
_lib.quartet_linear_workspace_bytes_block.restype = ctypes.c_size_t
_lib.quartet_linear_workspace_bytes_block.argtypes = [_i64, _i64, _i64, _int]
_lib.quartet_linear_bwd_block.argtypes = [_p, _i64, _i64, _i64, _int, _p, _p, _p, _p, _p, _p, _u64, _int, _p, _p, _int,
                                          _p, ctypes.c_size_t, _p]
for _name in EXPORTS:
    getattr(_lib, _name)  # AttributeError here = the library does not export what the header declares


class QuartetError(RuntimeError):
    pass


def check(rc):
    if rc != QUARTET_OK:
        names = {QUARTET_EINVAL: "QUARTET_EINVAL", QUARTET_ENOTSUP: "QUARTET_ENOTSUP", QUARTET_EHIP: "QUARTET_EHIP"}
        extra = f" (hipError_t {quartet_last_hip_error()})" if rc == QUARTET_EHIP else ""
        raise QuartetError(f"{names.get(rc, rc)}{extra}")
    return rc


def _ptr(t):
    """Device address of a torch tensor (must be a contiguous CUDA tensor), or a raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise QuartetError("pointer arguments must be CUDA (HIP) tensors: there is no CPU path")
    if not t.is_contiguous():
        raise QuartetError("tensor arguments must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def quartet_last_hip_error():
    return _lib.quartet_last_hip_error()


def quartet_sr_bits():
    return _lib.quartet_sr_bits()


KIND_NAMES = ["quant_fwd", "quant_bwd", "requant", "gemm", "epilogue", "dequant", "fp8_quant", "fp8_gemm"]
QUARTET_KIND_GEMM = 3


def quartet_profile_enable(max_records):
    return _lib.quartet_profile_enable(max_records)


def quartet_profile_kinds(kind_mask):
    return _lib.quartet_profile_kinds(kind_mask)


def quartet_profile_read(kinds, ms, capacity):
    """kinds: ctypes int array, ms: ctypes float array, both of length >= capacity."""
    return _lib.quartet_profile_read(ctypes.cast(kinds, _p), ctypes.cast(ms, _p), capacity)


def quartet_profile_clock(device_counters):
    """device_counters: a CUDA int64 tensor of two zeros, or None to switch the measurement off."""
    return _lib.quartet_profile_clock(_ptr(device_counters))


def quartet_wall_clock_khz():
    return _lib.quartet_wall_clock_khz()


def quartet_probe_mfma_ceiling(codes, scales, iterations, blocks, sink, device_counters=None, stream=None):
    return _lib.quartet_probe_mfma_ceiling(_ptr(codes), _ptr(scales), iterations, blocks, _ptr(sink), _ptr(device_counters),
                                           _stream(stream))


def quartet_scale_bytes(rows, k):
    return _lib.quartet_scale_bytes(rows, k)


def quartet_sign_word(seed):
    return _lib.quartet_sign_word(seed)


def quartet_quant_fwd(x_bf16, rows, k, ldx, transpose, codes, scales, mask, stream=None):
    return _lib.quartet_quant_fwd(_ptr(x_bf16), rows, k, ldx, int(transpose), _ptr(codes), _ptr(scales),
                                  _ptr(mask), _stream(stream))


def quartet_quant_bwd_sr(x_bf16, rows, k, ldx, transpose, sign_word, seed, stream_id, rounding, codes, scales,
                         stream=None):
    return _lib.quartet_quant_bwd_sr(_ptr(x_bf16), rows, k, ldx, int(transpose), sign_word, seed, stream_id,
                                     rounding, _ptr(codes), _ptr(scales), _stream(stream))


def quartet_requant_transpose_sr(src_codes, src_scales, rows, k, sign_word, seed, stream_id, rounding, codes,
                                 scales, stream=None):
    return _lib.quartet_requant_transpose_sr(_ptr(src_codes), _ptr(src_scales), rows, k, sign_word, seed,
                                             stream_id, rounding, _ptr(codes), _ptr(scales), _stream(stream))


def quartet_fwd_operands(x_bf16, w_bf16, tokens, in_features, out_features, xq_codes, xq_scales, x_mask, wq_codes,
                         wq_scales, w_mask, stream=None):
    return _lib.quartet_fwd_operands(_ptr(x_bf16), _ptr(w_bf16), tokens, in_features, out_features, _ptr(xq_codes),
                                     _ptr(xq_scales), _ptr(x_mask), _ptr(wq_codes), _ptr(wq_scales), _ptr(w_mask),
                                     _stream(stream))


def quartet_bwd_operands(dy_bf16, tokens, in_features, out_features, xq_codes, xq_scales, wq_codes, wq_scales, sign_word,
                         seed, rounding, dyt_codes, dyt_scales, xt_codes, xt_scales, wt_codes, wt_scales, stream=None):
    return _lib.quartet_bwd_operands(_ptr(dy_bf16), tokens, in_features, out_features, _ptr(xq_codes), _ptr(xq_scales),
                                     _ptr(wq_codes), _ptr(wq_scales), sign_word, seed, rounding, _ptr(dyt_codes),
                                     _ptr(dyt_scales), _ptr(xt_codes), _ptr(xt_scales), _ptr(wt_codes), _ptr(wt_scales),
                                     _stream(stream))


def quartet_mxfp4_gemm(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, d_dtype, ldd, stream=None):
    return _lib.quartet_mxfp4_gemm(_ptr(a_codes), _ptr(a_scales), _ptr(b_codes), _ptr(b_scales), m, n, k,
                                   alpha, _ptr(d), d_dtype, ldd, _stream(stream))


def quartet_debug_set_gemm_plan(variant, band_height):
    return _lib.quartet_debug_set_gemm_plan(variant, band_height)


def quartet_mxfp4_gemm_grad(a_codes, a_scales, b_codes, b_scales, m, n, k, mask, scale, d, d_dtype, ldd, stream=None):
    return _lib.quartet_mxfp4_gemm_grad(_ptr(a_codes), _ptr(a_scales), _ptr(b_codes), _ptr(b_scales), m, n, k,
                                        _ptr(mask), scale, _ptr(d), d_dtype, ldd, _stream(stream))


def gemm_grad_args(a_codes, a_scales, b_codes, b_scales, m, n, k, mask, scale, d, ldd):
    """One argument block of quartet_mxfp4_gemm_grad_pair (the tensors must stay alive until the call has been made)."""
    return GemmGradArgs(_ptr(a_codes), _ptr(a_scales), _ptr(b_codes), _ptr(b_scales), m, n, k, _ptr(mask), scale, _ptr(d), ldd)


def quartet_mxfp4_gemm_grad_pair(first, second, d_dtype, stream=None):
    return _lib.quartet_mxfp4_gemm_grad_pair(ctypes.byref(first) if first is not None else None,
                                             ctypes.byref(second) if second is not None else None, d_dtype, _stream(stream))


def quartet_mxfp8_quant(x_bf16, rows, k, ldx, codes, scales, stream=None):
    return _lib.quartet_mxfp8_quant(_ptr(x_bf16), rows, k, ldx, _ptr(codes), _ptr(scales), _stream(stream))


def quartet_mxfp8_gemm(a_codes, a_scales, b_codes, b_scales, m, n, k, alpha, d, d_dtype, ldd, stream=None):
    return _lib.quartet_mxfp8_gemm(_ptr(a_codes), _ptr(a_scales), _ptr(b_codes), _ptr(b_scales), m, n, k,
                                   alpha, _ptr(d), d_dtype, ldd, _stream(stream))


def quartet_grad_epilogue(g, mask, m, n, scale, out, out_dtype, stream=None):
    return _lib.quartet_grad_epilogue(_ptr(g), _ptr(mask), m, n, scale, _ptr(out), out_dtype, _stream(stream))


def quartet_mxfp4_dequant(codes, scales, rows, k, out, stream=None):
    return _lib.quartet_mxfp4_dequant(_ptr(codes), _ptr(scales), rows, k, _ptr(out), _stream(stream))


def quartet_linear_fwd(x_bf16, w_bf16, tokens, in_features, out_features, y, y_dtype, xq_codes, xq_scales,
                       x_mask, wq_codes, wq_scales, w_mask, stream=None):
    return _lib.quartet_linear_fwd(_ptr(x_bf16), _ptr(w_bf16), tokens, in_features, out_features, _ptr(y),
                                   y_dtype, _ptr(xq_codes), _ptr(xq_scales), _ptr(x_mask), _ptr(wq_codes),
                                   _ptr(wq_scales), _ptr(w_mask), _stream(stream))


def quartet_linear_workspace_bytes(tokens, in_features, out_features):
    return _lib.quartet_linear_workspace_bytes(tokens, in_features, out_features)


def quartet_linear_bwd(dy_bf16, tokens, in_features, out_features, xq_codes, xq_scales, x_mask, wq_codes,
                       wq_scales, w_mask, seed, rounding, dx, dw, grad_dtype, workspace, workspace_bytes,
                       stream=None):
    return _lib.quartet_linear_bwd(_ptr(dy_bf16), tokens, in_features, out_features, _ptr(xq_codes),
                                   _ptr(xq_scales), _ptr(x_mask), _ptr(wq_codes), _ptr(wq_scales),
                                   _ptr(w_mask), seed, rounding, _ptr(dx), _ptr(dw), grad_dtype,
                                   _ptr(workspace), workspace_bytes, _stream(stream))


def quartet_static_scratch_bytes():
    return _lib.quartet_static_scratch_bytes()


def quartet_linear_bwd_static(dy_bf16, tokens, in_features, out_features, xq_codes, xq_scales, x_mask, wq_codes,
                              wq_scales, w_mask, seed, rounding, dx, dw, grad_dtype, stream=None):
    return _lib.quartet_linear_bwd_static(_ptr(dy_bf16), tokens, in_features, out_features, _ptr(xq_codes),
                                          _ptr(xq_scales), _ptr(x_mask), _ptr(wq_codes), _ptr(wq_scales),
                                          _ptr(w_mask), seed, rounding, _ptr(dx), _ptr(dw), grad_dtype,
                                          _stream(stream))


# ---- Hadamard blocks of 32, 64, 128 or 256 elements (sign_words: sequence of host integers)

def _host_words(sign_words):
    words = [int(w) & 0xFFFFFFFF for w in sign_words]
    if len(words) < 8:
        words = words + [0] * (8 - len(words))
    return (ctypes.c_uint32 * len(words))(*words)


def quartet_sign_words(seed):
    """The eight sign words of a seed as a list of Python ints."""
    out = (ctypes.c_uint32 * 8)()
    check(_lib.quartet_sign_words(seed, ctypes.cast(out, _p)))
    return list(out)


def quartet_quant_fwd_block(x_bf16, rows, k, ldx, transpose, hadamard_block, codes, scales, mask, stream=None):
    return _lib.quartet_quant_fwd_block(_ptr(x_bf16), rows, k, ldx, int(transpose), hadamard_block, _ptr(codes),
                                        _ptr(scales), _ptr(mask), _stream(stream))


def quartet_quant_bwd_sr_block(x_bf16, rows, k, ldx, transpose, hadamard_block, sign_words, seed, stream_id,
                               rounding, codes, scales, stream=None):
    sw = _host_words(sign_words)
    return _lib.quartet_quant_bwd_sr_block(_ptr(x_bf16), rows, k, ldx, int(transpose), hadamard_block,
                                           ctypes.cast(sw, _p), seed, stream_id, rounding, _ptr(codes), _ptr(scales),
                                           _stream(stream))


def quartet_requant_transpose_sr_block(src_codes, src_scales, rows, k, hadamard_block, sign_words, seed, stream_id,
                                       rounding, codes, scales, stream=None):
    sw = _host_words(sign_words)
    return _lib.quartet_requant_transpose_sr_block(_ptr(src_codes), _ptr(src_scales), rows, k, hadamard_block,
                                                   ctypes.cast(sw, _p), seed, stream_id, rounding, _ptr(codes),
                                                   _ptr(scales), _stream(stream))


def quartet_mxfp4_gemm_grad_block(a_codes, a_scales, b_codes, b_scales, m, n, k, hadamard_block, mask, scale, d, d_dtype,
                                  ldd, stream=None):
    return _lib.quartet_mxfp4_gemm_grad_block(_ptr(a_codes), _ptr(a_scales), _ptr(b_codes), _ptr(b_scales), m, n, k,
                                              hadamard_block, _ptr(mask), scale, _ptr(d), d_dtype, ldd, _stream(stream))


def quartet_grad_epilogue_block(g, mask, m, n, hadamard_block, scale, out, out_dtype, stream=None):
    return _lib.quartet_grad_epilogue_block(_ptr(g), _ptr(mask), m, n, hadamard_block, scale, _ptr(out), out_dtype,
                                            _stream(stream))


def quartet_linear_fwd_block(x_bf16, w_bf16, tokens, in_f, out_f, hadamard_block, y, y_dtype, xq_codes, xq_scales,
                             x_mask, wq_codes, wq_scales, w_mask, stream=None):
    return _lib.quartet_linear_fwd_block(_ptr(x_bf16), _ptr(w_bf16), tokens, in_f, out_f, hadamard_block, _ptr(y),
                                         y_dtype, _ptr(xq_codes), _ptr(xq_scales), _ptr(x_mask), _ptr(wq_codes),
                                         _ptr(wq_scales), _ptr(w_mask), _stream(stream))


def quartet_linear_workspace_bytes_block(tokens, in_f, out_f, hadamard_block):
    return _lib.quartet_linear_workspace_bytes_block(tokens, in_f, out_f, hadamard_block)


def quartet_linear_bwd_block(dy_bf16, tokens, in_f, out_f, hadamard_block, xq_codes, xq_scales, x_mask, wq_codes,
                             wq_scales, w_mask, seed, rounding, dx, dw, grad_dtype, workspace, workspace_bytes,
                             stream=None):
    return _lib.quartet_linear_bwd_block(_ptr(dy_bf16), tokens, in_f, out_f, hadamard_block, _ptr(xq_codes),
                                         _ptr(xq_scales), _ptr(x_mask), _ptr(wq_codes), _ptr(wq_scales),
                                         _ptr(w_mask), seed, rounding, _ptr(dx), _ptr(dw), grad_dtype,
                                         _ptr(workspace), workspace_bytes, _stream(stream))
