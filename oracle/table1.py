"""Table 1's two measurable columns on Gaussian data, from the oracle's quantizers (CPU only).

For each scheme the relative quadratic error  |Q(h) - h|^2 / |h|^2  of the rotated data h, and the
projection magnitude misalignment  1 - E[1/S]  with  1/S = <h, Q(h)> / <h, h>  per MXFP4 group
(Section 4.3, "Backward pass: a novel error-bias trade-off").  Q is the de-quantized output, with the
backward quantizers' 3/4 range matching undone by 4/3.  Run as  python -m oracle.table1 [--block 64].

TEST INFRASTRUCTURE like the rest of oracle/: a reporting tool over the oracle, never used by the
product path.
"""
import argparse

import numpy as np

import oracle

_GRID = np.array([oracle.e2m1_decode(c) for c in range(16)])


def _decode(codes, scales):
    nib = np.stack([codes & 15, codes >> 4], axis=-1).reshape(codes.shape[0], -1)
    return _GRID[nib] * np.repeat(np.ldexp(1.0, scales.astype(np.int64) - 127), 32, axis=1)


def _bf16_bits(x):
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def _rotated(x_bits, block, sign_words):
    """fp64 H_block (d . x) of the bf16 data, by the dense Sylvester matrix."""
    from scipy.linalg import hadamard
    x = (x_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    d = np.ones(block)
    if sign_words is not None:
        for i in range(block):
            if (int(sign_words[i // 32]) >> (i % 32)) & 1:
                d[i] = -1.0
    H = hadamard(block).astype(np.float64) / np.sqrt(block)
    rows, k = x.shape
    return ((x.reshape(rows, k // block, block) * d) @ H.T).reshape(rows, k)


def _columns(h, q):
    """relative quadratic error over everything, and 1 - mean over groups of <h,q>/<h,h>"""
    hg, qg = h.reshape(-1, 32), q.reshape(-1, 32)
    mse = ((q - h) ** 2).sum() / (h ** 2).sum()
    inv_s = (hg * qg).sum(-1) / (hg * hg).sum(-1)
    return float(mse), float(1.0 - inv_s.mean())


def table1(rows=512, k=2048, seed=0, block=32, sr_seeds=4):
    """{scheme: (mse, misalignment)} for 'sr_absmax', 'rtn_absmax', 'quest' on N(0,1) data."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = _bf16_bits(rng.standard_normal((rows, k), dtype=np.float32))
    sw = oracle.sign_words(seed)
    out = {}
    h = _rotated(x, block, sw)
    acc = []
    for s in range(sr_seeds):
        c, sc = oracle.quant_bwd_sr_block(x, block, sw, seed + 1000 * s, 0, rounding=0)
        acc.append(_columns(h, _decode(c, sc) * (4.0 / 3.0)))
    out["sr_absmax"] = tuple(np.mean(acc, axis=0))
    c, sc = oracle.quant_bwd_sr_block(x, block, sw, seed, 0, rounding=1)
    out["rtn_absmax"] = _columns(h, _decode(c, sc) * (4.0 / 3.0))
    c, sc, _ = oracle.quant_fwd_block(x, block)
    out["quest"] = _columns(_rotated(x, block, None), _decode(c, sc))
    return out


PAPER = {"sr_absmax": (2.77e-2, 0.0), "rtn_absmax": (1.37e-2, 9.3e-3), "quest": (1.32e-2, 1.3e-2)}

if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--block", type=int, default=32, help="Hadamard block: 32, 64, 128 or 256")
    ap.add_argument("--rows", type=int, default=512)
    ap.add_argument("--k", type=int, default=2048)
    ap.add_argument("--seed", type=int, default=0)
    a = ap.parse_args()
    res = table1(a.rows, a.k, a.seed, a.block)
    print(f"Gaussian data {a.rows} x {a.k}, MXFP4 group 32, Hadamard block {a.block}")
    print(f"{'scheme':12s} {'MSE':>10s} {'paper':>10s} {'misalign.':>11s} {'paper':>10s}")
    for name, (mse, mis) in res.items():
        print(f"{name:12s} {mse:10.3e} {PAPER[name][0]:10.2e} {mis:11.2e} {PAPER[name][1]:10.1e}")
