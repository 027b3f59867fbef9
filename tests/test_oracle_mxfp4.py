"""Pins for the oracle's MXFP4 weight path (OCP Microscaling: FP4 E2M1 elements, one E8M0 scale per block of 32):
the element table typed in from the published format, rounding redone by brute force with exact rational
arithmetic, the block exponent against Python's own floor(log2) on exact binary fractions, the properties the
specification's conversion implies (block maximum lands on 4 or 6, error bounds, saturation zone), exactness of the
dequantised weights as bf16 numbers, and the quantised FFN against a numpy fp64 contraction.
"""
from fractions import Fraction
import math

import numpy as np
import pytest

import oracle
import workloads as wl

# E2M1: sign, two exponent bits (bias 1), one mantissa bit; exponent 0 is subnormal (0 and 0.5)
TABLE = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def test_element_table_is_the_published_one():
    got = oracle.e2m1_decode(np.arange(16, dtype=np.uint8))
    assert got[:8].tolist() == TABLE and got[8:].tolist() == [-v for v in TABLE]
    assert np.signbit(got[8])                                            # negative zero keeps its sign
    for c in range(8):                                                   # the same from the bit fields
        e, m = c >> 1, c & 1
        assert TABLE[c] == (m * 0.5 if e == 0 else (1 + m / 2) * 2.0 ** (e - 1))


def _nearest_even(fr):
    """Nearest table entry of a non-negative Fraction, ties to the even code, by exhaustive comparison."""
    best = min(range(8), key=lambda c: (abs(fr - Fraction(TABLE[c])), c & 1))
    return best


def test_rounding_by_brute_force_on_exact_rationals():
    rng = np.random.default_rng(0)
    vals = np.concatenate([rng.uniform(-7, 7, 4000), rng.standard_normal(2000) * 0.3,
                           np.arange(0, 7.01, 0.125), -np.arange(0, 7.01, 0.125),      # every midpoint and grid point
                           [6.0, 6.5, 100.0, 1e30, np.inf, -np.inf, 1e-30, -1e-30, 0.0, -0.0]]).astype(np.float32)
    got = oracle.e2m1_encode(vals)
    for v, c in zip(vals.tolist(), got.tolist()):
        a = Fraction(abs(v)) if math.isfinite(v) else Fraction(10 ** 40)
        want = _nearest_even(a) | (8 if math.copysign(1.0, v) < 0 else 0)
        assert c == want, (v, c, want)
    # the midpoints, spelled out: ties go to the code with mantissa bit 0
    mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0], np.float32)
    assert oracle.e2m1_encode(mids).tolist() == [0, 2, 2, 4, 4, 6, 6]
    assert oracle.e2m1_encode(np.nextafter(mids, np.float32(10))).tolist() == [1, 2, 3, 4, 5, 6, 7]
    assert oracle.e2m1_encode(np.nextafter(mids, np.float32(-10))).tolist() == [0, 1, 2, 3, 4, 5, 6]
    codes = np.arange(16, dtype=np.uint8)
    assert np.array_equal(oracle.e2m1_encode(oracle.e2m1_decode(codes).astype(np.float32)), codes)   # exact round trip


@pytest.mark.parametrize("shape", [(4, 32), (3, 5, 96), (2, 2, 2048)])
def test_block_scales_and_codes(shape):
    rng = np.random.default_rng(len(shape))
    w32 = (rng.standard_normal(shape) * 0.02 * np.exp(rng.uniform(-3, 3, shape[:-1] + (1,)))).astype(np.float32)
    W = wl.f32_to_bf16_bits(w32)
    flat = W.reshape(-1, shape[-1])
    flat[1, :32] = 0                                                      # an all-zero block
    flat[0, 32 * (shape[-1] // 32 - 1)] = wl.f32_to_bf16_bits(np.array([0.5], np.float32))[0]   # amax an exact power of two
    codes, E = oracle.quantize_mxfp4(W)
    w = wl.bf16_bits_to_f32(W).astype(np.float64)
    blocks = w.reshape(-1, 32)
    Eb, cb = E.reshape(-1), codes.reshape(-1, 32)
    for b in range(blocks.shape[0] if blocks.shape[0] < 400 else 400):
        amax = float(np.abs(blocks[b]).max())
        if amax == 0:
            assert Eb[b] == 127 and not cb[b].any()
            continue
        fl = math.floor(math.log2(amax))                                 # exact here: checked against the power itself
        assert 2.0 ** fl <= amax < 2.0 ** (fl + 1)
        assert Eb[b] == fl - 2 + 127
        X = 2.0 ** (fl - 2)
        for v, c in zip(blocks[b].tolist(), cb[b].tolist()):
            assert c == (_nearest_even(Fraction(abs(v)) / Fraction(X)) | (8 if math.copysign(1.0, v) < 0 else 0))
        top = np.abs(oracle.e2m1_decode(cb[b])).max()
        assert top in (4.0, 6.0)                                          # amax / X is in [4, 8)
    # error: half a step below 6 X (steps 0.5 X up to 2 X, X up to 4 X, 2 X up to 6 X); values in (6 X, 8 X) saturate to 6 X
    deq = oracle.e2m1_decode(codes).reshape(-1, 32) * (2.0 ** (Eb.astype(np.float64) - 127))[:, None]
    Xs = (2.0 ** (Eb.astype(np.float64) - 127))[:, None]
    a = np.abs(blocks)
    step = np.where(a < 2 * Xs, 0.5 * Xs, np.where(a < 4 * Xs, Xs, 2 * Xs))
    ok = np.where(a <= 6 * Xs, np.abs(deq - blocks) <= step / 2, (np.abs(deq) == 6 * Xs) & (a < 8 * Xs))
    assert ok.all()


def test_dequantised_weights_are_bf16_numbers():
    rng = np.random.default_rng(7)
    W = wl.f32_to_bf16_bits((rng.standard_normal((6, 128)) * 0.05).astype(np.float32))
    codes, E = oracle.quantize_mxfp4(W)
    D = oracle.dequantize_mxfp4(codes, E)
    want = oracle.e2m1_decode(codes) * np.repeat(2.0 ** (E.astype(np.float64) - 127), 32, axis=-1)
    assert np.array_equal(wl.bf16_bits_to_f32(D).astype(np.float64), want)
    assert np.array_equal(wl.f32_to_bf16_bits(want.astype(np.float32)), D)
    # quantising the dequantised weights again changes nothing (they are on the grid of their own blocks)
    codes2, E2 = oracle.quantize_mxfp4(D)
    assert np.array_equal(oracle.dequantize_mxfp4(codes2, E2), D)
    with pytest.raises(oracle.OracleError):
        oracle.quantize_mxfp4(W[:, :48])                                 # K must be a multiple of 32
    with pytest.raises(oracle.OracleError):
        oracle.dequantize_mxfp4(codes, np.full_like(E, 255))             # the NaN scale


def test_quantised_ffn_is_the_ffn_of_the_dequantised_weights():
    rng = np.random.default_rng(5)
    T, H, F, N, k, S, Fs = 7, 64, 96, 5, 2, 1, 32
    bits = lambda shape: wl.f32_to_bf16_bits((rng.standard_normal(shape) * 0.05).astype(np.float32))
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    Wg, Wu, Wd, Sg, Su, Sd = bits((N, F, H)), bits((N, F, H)), bits((N, H, F)), bits((S, Fs, H)), bits((S, Fs, H)), bits((S, H, Fs))
    q = {n: oracle.quantize_mxfp4(W) for n, W in dict(Wg=Wg, Wu=Wu, Wd=Wd, Sg=Sg, Su=Su, Sd=Sd).items()}
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    gate = rng.dirichlet(np.ones(k), T)
    y = oracle.moe_ffn_q4(x, q["Wg"][0], q["Wu"][0], q["Wd"][0], q["Wg"][1], q["Wu"][1], q["Wd"][1], idx, gate,
                          q["Sg"][0], q["Su"][0], q["Sd"][0], q["Sg"][1], q["Su"][1], q["Sd"][1])
    deq = lambda n: oracle.e2m1_decode(q[n][0]) * np.repeat(2.0 ** (q[n][1].astype(np.float64) - 127), 32, axis=-1)
    xs = wl.bf16_bits_to_f32(x).astype(np.float64)
    y_ref = np.zeros((T, H))
    silu = lambda a: a / (1 + np.exp(-a))
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            y_ref[t] += gate[t, j] * (deq("Wd")[e] @ (silu(deq("Wg")[e] @ xs[t]) * (deq("Wu")[e] @ xs[t])))
        y_ref[t] += deq("Sd")[0] @ (silu(deq("Sg")[0] @ xs[t]) * (deq("Su")[0] @ xs[t]))
    np.testing.assert_allclose(y, y_ref, rtol=1e-10, atol=1e-13)
    # against the unquantised layer the error is the few tens of percent per weight that four bits imply, averaged down
    y16 = oracle.moe_ffn(x, Wg, Wu, Wd, idx, gate, Sg, Su, Sd)
    rel = np.abs(y - y16).max(1) / np.abs(y16).max(1)
    assert rel.max() < 0.6 and rel.mean() > 1e-3
