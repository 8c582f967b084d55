"""Helpers for the GPU parity tests: move numpy arrays to the device, call the C ABI through the
binding, bring results back.  No arithmetic of the method lives here."""
import numpy as np
import torch

from paper_2505_14669_amd import binding as q
from indep import scales_from_tiled, scales_to_tiled

DEV = "cuda:0"


def to_dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def to_host(t, dtype):
    torch.cuda.synchronize()
    return t.cpu().numpy().view(dtype)


def dev_empty(shape, np_dtype, fill=None):
    tdt = {np.uint8: torch.uint8, np.uint16: torch.int16, np.uint32: torch.int32, np.float32: torch.float32}[np_dtype]
    t = torch.empty(shape, dtype=tdt, device=DEV)
    if fill is not None:
        t.fill_(fill)
    return t


def quant_fwd(x_u16, transpose=False, want_mask=True, ldx=None):
    x = to_dev(x_u16)
    ld = x_u16.shape[1] if ldx is None else ldx
    rows, k = (x_u16.shape[1], x_u16.shape[0]) if transpose else x_u16.shape
    codes = dev_empty((rows, k // 2), np.uint8, 0xEE)
    scales = dev_empty((max(q.quartet_scale_bytes(rows, k), 4),), np.uint8, 0xFF)
    mask = dev_empty((rows, k // 32), np.uint32, 0x5A5A5A5A) if want_mask else None
    q.check(q.quartet_quant_fwd(x, rows, k, ld, transpose, codes, scales, mask))
    return (to_host(codes, np.uint8), scales_from_tiled(to_host(scales, np.uint8), rows, k),
            to_host(mask, np.uint32) if want_mask else None)


def quant_bwd_sr(x_u16, sign_word, seed, stream_id, rounding=0, transpose=False):
    x = to_dev(x_u16)
    rows, k = (x_u16.shape[1], x_u16.shape[0]) if transpose else x_u16.shape
    codes = dev_empty((rows, k // 2), np.uint8, 0xEE)
    scales = dev_empty((max(q.quartet_scale_bytes(rows, k), 4),), np.uint8, 0xFF)
    q.check(q.quartet_quant_bwd_sr(x, rows, k, x_u16.shape[1], transpose, sign_word, seed, stream_id,
                                   rounding, codes, scales))
    return to_host(codes, np.uint8), scales_from_tiled(to_host(scales, np.uint8), rows, k)


def requant_transpose_sr(src_codes, src_scales, sign_word, seed, stream_id, rounding=0):
    k, rows = src_codes.shape[0], src_codes.shape[1] * 2
    sc, ss = to_dev(src_codes), to_dev(scales_to_tiled(src_scales))
    codes = dev_empty((rows, k // 2), np.uint8, 0xEE)
    scales = dev_empty((max(q.quartet_scale_bytes(rows, k), 4),), np.uint8, 0xFF)
    q.check(q.quartet_requant_transpose_sr(sc, ss, rows, k, sign_word, seed, stream_id, rounding, codes, scales))
    return to_host(codes, np.uint8), scales_from_tiled(to_host(scales, np.uint8), rows, k)


def fwd_operands(x_u16, w_u16):
    """quartet_fwd_operands on host arrays; returns (codes, scales row-major, mask) of X and of W."""
    t, i = x_u16.shape
    o = w_u16.shape[0]
    outs = []
    for r in (t, o):
        outs += [dev_empty((r, i // 2), np.uint8, 0xEE), dev_empty((max(q.quartet_scale_bytes(r, i), 4),), np.uint8, 0xFF),
                 dev_empty((r, i // 32), np.uint32, 0x5A5A5A5A)]
    q.check(q.quartet_fwd_operands(to_dev(x_u16), to_dev(w_u16), t, i, o, *outs))
    return [(to_host(outs[3 * n], np.uint8), scales_from_tiled(to_host(outs[3 * n + 1], np.uint8), r, i),
             to_host(outs[3 * n + 2], np.uint32)) for n, r in enumerate((t, o))]


def bwd_operands(dy_u16, xq_codes, xq_scales, wq_codes, wq_scales, sign_word, seed, rounding=0):
    """quartet_bwd_operands on host arrays (scales row-major); returns (codes, scales) of dy^T, X_q^T, W_q^T."""
    t, o = dy_u16.shape
    i = xq_codes.shape[1] * 2
    outs = []
    for r, c in ((o, t), (i, t), (i, o)):
        outs += [dev_empty((r, c // 2), np.uint8, 0xEE), dev_empty((max(q.quartet_scale_bytes(r, c), 4),), np.uint8, 0xFF)]
    q.check(q.quartet_bwd_operands(to_dev(dy_u16), t, i, o, to_dev(xq_codes), to_dev(scales_to_tiled(xq_scales)),
                                   to_dev(wq_codes), to_dev(scales_to_tiled(wq_scales)), sign_word, seed, rounding, *outs))
    res = []
    for n, (r, c) in enumerate(((o, t), (i, t), (i, o))):
        res.append((to_host(outs[2 * n], np.uint8), scales_from_tiled(to_host(outs[2 * n + 1], np.uint8), r, c)))
    return res


def dequant(codes, scales):
    rows, k = codes.shape[0], codes.shape[1] * 2
    out = dev_empty((rows, k), np.float32, float("nan"))
    q.check(q.quartet_mxfp4_dequant(to_dev(codes), to_dev(scales_to_tiled(scales)), rows, k, out))
    return to_host(out, np.float32)


def gemm(a_codes, a_scales, b_codes, b_scales, alpha=1.0, bf16=False, ldd=None):
    m, k = a_codes.shape[0], a_codes.shape[1] * 2
    n = b_codes.shape[0]
    ldd = n if ldd is None else ldd
    if bf16:
        d = dev_empty((m, ldd), np.uint16, 0x7FC0)
    else:
        d = dev_empty((m, ldd), np.float32, float("nan"))
    q.check(q.quartet_mxfp4_gemm(to_dev(a_codes), to_dev(scales_to_tiled(a_scales)), to_dev(b_codes),
                                 to_dev(scales_to_tiled(b_scales)), m, n, k,
                                 alpha, d, q.QUARTET_DTYPE_BF16 if bf16 else q.QUARTET_DTYPE_F32, ldd))
    return to_host(d, np.uint16 if bf16 else np.float32)


def gemm_grad(a_codes, a_scales, b_codes, b_scales, mask, scale, bf16=False, ldd=None):
    m, k = a_codes.shape[0], a_codes.shape[1] * 2
    n = b_codes.shape[0]
    ldd = n if ldd is None else ldd
    if bf16:
        d = dev_empty((m, ldd), np.uint16, 0x7FC0)
    else:
        d = dev_empty((m, ldd), np.float32, float("nan"))
    q.check(q.quartet_mxfp4_gemm_grad(to_dev(a_codes), to_dev(scales_to_tiled(a_scales)), to_dev(b_codes),
                                      to_dev(scales_to_tiled(b_scales)), m, n, k,
                                      None if mask is None else to_dev(mask), scale, d,
                                      q.QUARTET_DTYPE_BF16 if bf16 else q.QUARTET_DTYPE_F32, ldd))
    return to_host(d, np.uint16 if bf16 else np.float32)


def gemm_grad_pair(first, second, bf16=False):
    """first, second: (a_codes, a_scales, b_codes, b_scales, mask, scale) of the two products; returns both results."""
    keep, blocks, outs = [], [], []
    for (a_codes, a_scales, b_codes, b_scales, mask, scale) in (first, second):
        m, k = a_codes.shape[0], a_codes.shape[1] * 2
        n = b_codes.shape[0]
        d = dev_empty((m, n), np.uint16, 0x7FC0) if bf16 else dev_empty((m, n), np.float32, float("nan"))
        tensors = [to_dev(a_codes), to_dev(scales_to_tiled(a_scales)), to_dev(b_codes), to_dev(scales_to_tiled(b_scales)),
                   None if mask is None else to_dev(mask)]
        keep.append(tensors)
        blocks.append(q.gemm_grad_args(tensors[0], tensors[1], tensors[2], tensors[3], m, n, k, tensors[4], scale, d, n))
        outs.append(d)
    q.check(q.quartet_mxfp4_gemm_grad_pair(blocks[0], blocks[1], q.QUARTET_DTYPE_BF16 if bf16 else q.QUARTET_DTYPE_F32))
    return tuple(to_host(d, np.uint16 if bf16 else np.float32) for d in outs)


def grad_epilogue(g, mask, scale, bf16=False, in_place=False):
    m, n = g.shape
    gd = to_dev(g)
    md = None if mask is None else to_dev(mask)
    if in_place:
        out = gd
    elif bf16:
        out = dev_empty((m, n), np.uint16, 0)
    else:
        out = dev_empty((m, n), np.float32, float("nan"))
    q.check(q.quartet_grad_epilogue(gd, md, m, n, float(scale), out,
                                    q.QUARTET_DTYPE_BF16 if bf16 else q.QUARTET_DTYPE_F32))
    return to_host(out, np.uint16 if bf16 else np.float32)


class Linear:
    """Device buffers of one linear layer; fwd()/bwd() call the library's two entry points."""

    def __init__(self, x_u16, w_u16):
        self.t, self.i = x_u16.shape
        self.o = w_u16.shape[0]
        t, i, o = self.t, self.i, self.o
        self.x, self.w = to_dev(x_u16), to_dev(w_u16)
        self.y = dev_empty((t, o), np.float32, float("nan"))
        self.xq_codes = dev_empty((t, i // 2), np.uint8, 0)
        self.xq_scales = dev_empty((max(q.quartet_scale_bytes(t, i), 4),), np.uint8, 0xFF)
        self.x_mask = dev_empty((t, i // 32), np.uint32, 0)
        self.wq_codes = dev_empty((o, i // 2), np.uint8, 0)
        self.wq_scales = dev_empty((max(q.quartet_scale_bytes(o, i), 4),), np.uint8, 0xFF)
        self.w_mask = dev_empty((o, i // 32), np.uint32, 0)
        self.dx = dev_empty((t, i), np.float32, float("nan"))
        self.dw = dev_empty((o, i), np.float32, float("nan"))
        self.ws_bytes = q.quartet_linear_workspace_bytes(t, i, o)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=DEV)

    def fwd(self):
        q.check(q.quartet_linear_fwd(self.x, self.w, self.t, self.i, self.o, self.y, q.QUARTET_DTYPE_F32,
                                     self.xq_codes, self.xq_scales, self.x_mask,
                                     self.wq_codes, self.wq_scales, self.w_mask))

    def bwd(self, dy_dev, seed, rounding=0):
        q.check(q.quartet_linear_bwd(dy_dev, self.t, self.i, self.o, self.xq_codes, self.xq_scales, self.x_mask,
                                     self.wq_codes, self.wq_scales, self.w_mask, seed, rounding,
                                     self.dx, self.dw, q.QUARTET_DTYPE_F32, self.ws, self.ws_bytes))

    def ctx_host(self):
        return dict(xq_codes=to_host(self.xq_codes, np.uint8),
                    xq_scales=scales_from_tiled(to_host(self.xq_scales, np.uint8), self.t, self.i),
                    x_mask=to_host(self.x_mask, np.uint32), wq_codes=to_host(self.wq_codes, np.uint8),
                    wq_scales=scales_from_tiled(to_host(self.wq_scales, np.uint8), self.o, self.i),
                    w_mask=to_host(self.w_mask, np.uint32))


# ---- Hadamard blocks of 64, 128, 256 elements

def quant_fwd_block(x_u16, block, transpose=False, want_mask=True):
    x = to_dev(x_u16)
    rows, k = (x_u16.shape[1], x_u16.shape[0]) if transpose else x_u16.shape
    codes = dev_empty((rows, k // 2), np.uint8, 0xEE)
    scales = dev_empty((max(q.quartet_scale_bytes(rows, k), 4),), np.uint8, 0xFF)
    mask = dev_empty((rows, k // 32), np.uint32, 0x5A5A5A5A) if want_mask else None
    q.check(q.quartet_quant_fwd_block(x, rows, k, x_u16.shape[1], transpose, block, codes, scales, mask))
    return (to_host(codes, np.uint8), scales_from_tiled(to_host(scales, np.uint8), rows, k),
            to_host(mask, np.uint32) if want_mask else None)


def quant_bwd_sr_block(x_u16, block, sign_words, seed, stream_id, rounding=0, transpose=False):
    x = to_dev(x_u16)
    rows, k = (x_u16.shape[1], x_u16.shape[0]) if transpose else x_u16.shape
    codes = dev_empty((rows, k // 2), np.uint8, 0xEE)
    scales = dev_empty((max(q.quartet_scale_bytes(rows, k), 4),), np.uint8, 0xFF)
    q.check(q.quartet_quant_bwd_sr_block(x, rows, k, x_u16.shape[1], transpose, block, list(sign_words), seed,
                                         stream_id, rounding, codes, scales))
    return to_host(codes, np.uint8), scales_from_tiled(to_host(scales, np.uint8), rows, k)


def requant_transpose_sr_block(src_codes, src_scales, block, sign_words, seed, stream_id, rounding=0):
    k, rows = src_codes.shape[0], src_codes.shape[1] * 2
    sc, ss = to_dev(src_codes), to_dev(scales_to_tiled(src_scales))
    codes = dev_empty((rows, k // 2), np.uint8, 0xEE)
    scales = dev_empty((max(q.quartet_scale_bytes(rows, k), 4),), np.uint8, 0xFF)
    q.check(q.quartet_requant_transpose_sr_block(sc, ss, rows, k, block, list(sign_words), seed, stream_id, rounding,
                                                 codes, scales))
    return to_host(codes, np.uint8), scales_from_tiled(to_host(scales, np.uint8), rows, k)


def gemm_grad_block(a_codes, a_scales, b_codes, b_scales, block, mask, scale, bf16=False):
    m, k = a_codes.shape[0], a_codes.shape[1] * 2
    n = b_codes.shape[0]
    d = dev_empty((m, n), np.uint16, 0x7FC0) if bf16 else dev_empty((m, n), np.float32, float("nan"))
    q.check(q.quartet_mxfp4_gemm_grad_block(to_dev(a_codes), to_dev(scales_to_tiled(a_scales)), to_dev(b_codes),
                                            to_dev(scales_to_tiled(b_scales)), m, n, k, block,
                                            None if mask is None else to_dev(mask), scale, d,
                                            q.QUARTET_DTYPE_BF16 if bf16 else q.QUARTET_DTYPE_F32, n))
    return to_host(d, np.uint16 if bf16 else np.float32)


def grad_epilogue_block(g, mask, block, scale, bf16=False):
    m, n = g.shape
    gd = to_dev(g)
    md = None if mask is None else to_dev(mask)
    out = dev_empty((m, n), np.uint16, 0) if bf16 else dev_empty((m, n), np.float32, float("nan"))
    q.check(q.quartet_grad_epilogue_block(gd, md, m, n, block, float(scale), out,
                                          q.QUARTET_DTYPE_BF16 if bf16 else q.QUARTET_DTYPE_F32))
    return to_host(out, np.uint16 if bf16 else np.float32)


class LinearBlock(Linear):
    """The same layer with a Hadamard block of `block` elements."""

    def __init__(self, x_u16, w_u16, block):
        super().__init__(x_u16, w_u16)
        self.block = block
        self.ws_bytes = q.quartet_linear_workspace_bytes_block(self.t, self.i, self.o, block)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=DEV)

    def fwd(self):
        q.check(q.quartet_linear_fwd_block(self.x, self.w, self.t, self.i, self.o, self.block, self.y,
                                           q.QUARTET_DTYPE_F32, self.xq_codes, self.xq_scales, self.x_mask,
                                           self.wq_codes, self.wq_scales, self.w_mask))

    def bwd(self, dy_dev, seed, rounding=0):
        q.check(q.quartet_linear_bwd_block(dy_dev, self.t, self.i, self.o, self.block, self.xq_codes, self.xq_scales,
                                           self.x_mask, self.wq_codes, self.wq_scales, self.w_mask, seed, rounding,
                                           self.dx, self.dw, q.QUARTET_DTYPE_F32, self.ws, self.ws_bytes))
