"""Pins of the oracle's MXFP8 comparison format (E4M3 elements, E8M0 scale per 32; Section 3 names the
format, Section 5 "Speedup results" measures against it).  Independent of the oracle: the value
table below is rebuilt from the bit-field definition in numpy, the nearest search is brute force."""
import os

import numpy as np

import oracle
from indep import GOLDEN
from paper_2505_14669_amd import synth


def table():
    """All 256 E4M3 values from the field definition (NaN for S.1111.111)."""
    c = np.arange(256)
    e, m = (c >> 3) & 15, c & 7
    v = np.where(e == 0, m * 2.0 ** -9, (1 + m / 8.0) * 2.0 ** (e - 7.0))
    v = np.where((c & 0x7F) == 0x7F, np.nan, v)
    return np.where(c & 0x80, -v, v)


def test_decode_matches_the_specification_landmarks_and_the_field_definition():
    with open(os.path.join(GOLDEN, "e4m3_values.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            code, val = line.split()
            assert oracle.e4m3_decode(int(code, 16)) == float(val)
    t = table()
    for c in range(256):
        d = oracle.e4m3_decode(c)
        assert (np.isnan(d) and np.isnan(t[c])) or d == t[c]
    assert np.nanmax(t) == 448.0 and np.isnan(oracle.e4m3_decode(0x7F)) and np.isnan(oracle.e4m3_decode(0xFF))


def _nearest_even(a, mags):
    """brute force: index of the nearest magnitude, ties to the even code, above the top saturates"""
    d = np.abs(mags[None, :] - a[:, None])
    best = d.min(axis=1)
    idx = np.empty(a.shape, dtype=np.int64)
    for i in range(a.size):
        cands = np.nonzero(d[i] == best[i])[0]
        idx[i] = cands[0] if cands.size == 1 else [c for c in cands if c % 2 == 0][0]
    return idx


def test_rtn_is_nearest_ties_to_even_and_saturates():
    mags = table()[:0x7F]                           # codes 0x00..0x7e, increasing
    bf = synth.bf16_to_f32(np.arange(0, 0x7F80, dtype=np.uint16))     # every non-negative finite bf16
    rng = np.random.default_rng(0)
    rnd = (rng.standard_normal(20000) * np.exp(rng.uniform(-6, 7, 20000))).astype(np.float32)
    mid = ((mags[:-1] + mags[1:]) / 2).astype(np.float32)            # every tie point (exact in fp32)
    for vals in (bf, np.abs(rnd), mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9))):
        want = _nearest_even(np.minimum(vals.astype(np.float64), 448.0), mags)
        got = np.array([oracle.e4m3_rtn(v) for v in vals])
        assert np.array_equal(got, want)
        got_neg = np.array([oracle.e4m3_rtn(-v) for v in vals[:2000]])
        assert np.array_equal(got_neg, want[:2000] | 0x80)
    assert oracle.e4m3_rtn(1e30) == 0x7E and oracle.e4m3_rtn(-1e30) == 0xFE and oracle.e4m3_rtn(float("nan")) == 0x7F
    assert oracle.e4m3_rtn(464.0) == 0x7E and oracle.e4m3_rtn(448.0) == 0x7E


def test_quantizer_scale_rule_range_and_error_bound():
    for kind in ("normal", "outliers", "heavy", "tiny", "zeros"):
        x = synth.small_matrix(31, 40, 160, kind)
        codes, scales = oracle.mxfp8_quant(x)
        xf = synth.bf16_to_f32(x).astype(np.float64).reshape(40, 5, 32)
        amax = np.abs(xf).max(axis=2)
        # scale: the power of two that puts the largest magnitude into the format's top binade [256, 512)
        with np.errstate(divide="ignore"):
            want = np.where(amax > 0, np.maximum(np.floor(np.log2(np.maximum(amax, 1e-300))) - 8 + 127, 0), 0)
        assert np.array_equal(scales, want.astype(np.uint8))
        dec = oracle.mxfp8_dequant(codes, scales).reshape(40, 5, 32)
        s = 2.0 ** (scales.astype(np.float64) - 127)[:, :, None]
        assert not np.isnan(dec).any()
        # never off by more than half a grid step (2^-4 relative in a binade; 2^-10 of the scale near zero),
        # except where the largest magnitudes saturate at 448 scale
        err = np.abs(dec - xf)
        bound = np.maximum(np.abs(xf) * 2.0 ** -4, s * 2.0 ** -10)
        sat = np.abs(xf) > 448 * s
        assert np.all((err <= bound) | sat)
        assert np.all(np.abs(dec[sat]) == (448 * np.broadcast_to(s, dec.shape))[sat])


def test_gemm_matches_numpy_on_decoded_operands():
    rng = np.random.default_rng(5)
    a = synth.f32_to_bf16(rng.standard_normal((24, 96)).astype(np.float32))
    b = synth.f32_to_bf16((rng.standard_normal((17, 96)) * 0.02).astype(np.float32))
    ac, as_ = oracle.mxfp8_quant(a)
    bc, bs = oracle.mxfp8_quant(b)
    t = table()
    da = t[ac] * np.repeat(2.0 ** (as_.astype(np.float64) - 127), 32, axis=1)
    db = t[bc] * np.repeat(2.0 ** (bs.astype(np.float64) - 127), 32, axis=1)
    got = oracle.mxfp8_gemm(ac, as_, bc, bs, alpha=0.5)
    assert np.allclose(got, 0.5 * da @ db.T, rtol=1e-12, atol=0)
    # and the quantized product is close to the exact one: 3 mantissa bits on each side
    exact = synth.bf16_to_f32(a).astype(np.float64) @ synth.bf16_to_f32(b).astype(np.float64).T
    assert np.linalg.norm(2 * got - exact) / np.linalg.norm(exact) < 0.05
