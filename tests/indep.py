"""Independent numpy/scipy building blocks used only to pin the oracle.

Nothing here is shared with oracle/ or with the HIP path: the Hadamard matrix comes from
scipy, the E2M1 grid from the golden fixture, decoding is plain table look-up in fp64.
"""
import os

import numpy as np
from scipy.linalg import hadamard

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
H32 = hadamard(32).astype(np.float64)  # Sylvester order, entries +-1


def load_grid():
    vals = np.zeros(16)
    with open(os.path.join(GOLDEN, "e2m1_grid.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            c, v = line.split()
            vals[int(c)] = float(v)
    return vals


GRID = load_grid()


def unpack_codes(codes):
    """[rows, k/2] bytes -> [rows, k] 4-bit codes (element 2j = low nibble of byte j)."""
    c = np.asarray(codes, dtype=np.uint8)
    out = np.empty((c.shape[0], c.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = c & 15
    out[:, 1::2] = c >> 4
    return out


def decode(codes, scales):
    """fp64 values of an MXFP4 tensor."""
    nib = unpack_codes(codes)
    vals = GRID[nib]
    vals = np.where(nib == 8, -0.0, vals)
    s = np.ldexp(1.0, np.asarray(scales, dtype=np.int64) - 127)
    return vals * np.repeat(s, 32, axis=1)


def dense_hadamard_rows(x, sign_word=0):
    """Normalized block Hadamard along the last axis in fp64: each block of 32 becomes
    H32 @ (d * block) / sqrt(32)."""
    x = np.asarray(x, dtype=np.float64)
    d = np.array([-1.0 if (sign_word >> i) & 1 else 1.0 for i in range(32)])
    blocks = x.reshape(x.shape[0], -1, 32) * d
    return (blocks @ H32.T / np.sqrt(32.0)).reshape(x.shape)


def read_table1():
    out = {}
    with open(os.path.join(GOLDEN, "table1_gaussian_mse.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, paper, lo, hi = line.split()
            out[name] = (float(paper), float(lo), float(hi))
    return out


# ---- tiled scale layout of the HIP library <-> row-major [rows, k/32] (pure index permutation)

def scale_tile_index(rows, k):
    """int64 array [rows, k/32] of byte offsets into the tiled scale buffer."""
    r = np.arange(rows, dtype=np.int64)[:, None]
    g = np.arange(k // 32, dtype=np.int64)[None, :]
    kq = (k + 255) // 256
    return ((r // 32) * kq + g // 8) * 256 + ((g % 2) * 32 + r % 32) * 4 + (g % 8) // 2


def scale_tiled_bytes(rows, k):
    return ((rows + 31) // 32) * ((k + 255) // 256) * 256


def scales_to_tiled(scales_row_major, fill=0xFF):
    s = np.asarray(scales_row_major, dtype=np.uint8)
    rows, k = s.shape[0], s.shape[1] * 32
    out = np.full(max(scale_tiled_bytes(rows, k), 4), fill, dtype=np.uint8)
    if s.size:
        out[scale_tile_index(rows, k)] = s
    return out


def scales_from_tiled(tiled, rows, k):
    return np.asarray(tiled, dtype=np.uint8)[scale_tile_index(rows, k)] if rows * k else np.zeros((rows, k // 32), np.uint8)


# ---- per-element error bounds for products accumulated in fp32 (used next to the Frobenius bar)

def gemm_abs_products(a_codes, a_scales, b_codes, b_scales):
    """sum_k |dec(A)[m,k]| |dec(B)[n,k]| in fp64: what a rounding error of the accumulation is relative to."""
    return np.abs(decode(a_codes, a_scales)) @ np.abs(decode(b_codes, b_scales)).T


def gemm_elem_bound(abs_products, k, alpha=1.0):
    """Bound on |fp32-accumulated product - exact product| per element.  The products of E2M1 values and powers
    of two are exact; the matrix cores add 64 of them to the fp32 accumulator per instruction, K/64 instructions in
    a row, and each addition rounds (or truncates) the running sum once: at most 2^-23 of its magnitude, which never
    exceeds sum |a||b|.  Three more roundings of the same size cover the multiply by alpha, the result's own rounding
    and the conversion of the oracle's fp64 value.  c = K/64 + 3 ulps of 2^-23: a worst-case bound, not a fit."""
    return abs(alpha) * (k // 64 + 3) * 2.0 ** -23 * abs_products


def grad_elem_bound(product_bound, abs_exact_product, scale, block=32):
    """The same bound carried through the gradient epilogue scale * H_block(g . mask) along the last axis: a transformed
    element is a signed sum of its block's inputs over sqrt(block), so the input bounds add up; the log2(block)
    butterfly stages and the two multiplies round log2(block) + 2 more times, each at most 2^-24 of a magnitude that
    the block's sum of |inputs| over sqrt(block) bounds (12 x 2^-24 taken, enough up to block = 256)."""
    m, n = product_bound.shape
    per_block = (product_bound + 12 * 2.0 ** -24 * abs_exact_product).reshape(m, n // block, block).sum(-1, keepdims=True)
    return np.broadcast_to(abs(scale) / np.sqrt(float(block)) * per_block, (m, n // block, block)).reshape(m, n)


def worst_excess(got, want, bound):
    """max over elements of |got - want| / bound (elements with a zero bound must agree exactly)."""
    err = np.abs(np.asarray(got, dtype=np.float64) - np.asarray(want, dtype=np.float64))
    zero = bound == 0
    if np.any(err[zero] != 0):
        return np.inf
    return float(np.max(err[~zero] / bound[~zero])) if np.any(~zero) else 0.0
