"""Pins for the oracle's FP8 (OCP E4M3) weight path: the code table and the rounding against torch's
float8_e4m3fn casts (an independent implementation of the published format), the halfway cases and the
saturation by construction, the row scales against numpy's fp32 division, and the quantised FFN against a
numpy fp64 contraction of the dequantised weights and against the bf16 oracle on weights that E4M3
represents exactly.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl


def _torch_decode(codes):
    return torch.from_numpy(np.ascontiguousarray(codes, np.uint8)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


def _torch_encode(values):
    return torch.from_numpy(np.ascontiguousarray(values, np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_decode_table_matches_the_published_format():
    codes = np.arange(256, dtype=np.uint8)
    mine, ref = oracle.e4m3_decode(codes), _torch_decode(codes)
    assert np.array_equal(np.isnan(mine), np.isnan(ref)) and np.isnan(mine).sum() == 2          # 0x7f and 0xff
    ok = ~np.isnan(ref)
    assert np.array_equal(mine[ok], ref[ok]) and np.array_equal(np.signbit(mine[ok]), np.signbit(ref[ok]))
    assert mine[0x7e] == 448.0 and mine[0x08] == 2.0 ** -6 and mine[0x01] == 2.0 ** -9 and mine[0x38] == 1.0
    assert np.all(np.diff(mine[:0x7f]) > 0)                                                       # codes are ordered


def test_encode_rounds_to_nearest_even_like_the_library_cast():
    rng = np.random.default_rng(0)
    v = np.concatenate([rng.uniform(-448, 448, 20000), rng.standard_normal(20000) * np.exp(rng.uniform(-12, 6, 20000)),
                        [0.0, -0.0, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10, 2.0 ** -11, 1e-30]]).astype(np.float32)
    v = v[np.abs(v) <= 448]
    assert np.array_equal(oracle.e4m3_encode(v), _torch_encode(v))


def test_encode_halfway_cases_and_neighbours():
    vals = oracle.e4m3_decode(np.arange(0x7f, dtype=np.uint8))          # all non-negative finite values, ascending
    for c in range(0x7e):
        lo, hi = np.float32(vals[c]), np.float32(vals[c + 1])
        mid = np.float32((vals[c] + vals[c + 1]) / 2)                   # exactly representable in fp32
        even = c if c % 2 == 0 else c + 1
        got = oracle.e4m3_encode(np.array([mid, np.nextafter(mid, lo), np.nextafter(mid, hi), -mid], np.float32))
        assert got.tolist() == [even, c, c + 1, 0x80 | even], hex(c)
    assert oracle.e4m3_encode(np.array([448, 449, 464, 1e9, np.inf, -500], np.float32)).tolist() == [0x7e] * 5 + [0xfe]
    assert oracle.e4m3_encode(np.array([np.nan], np.float32))[0] & 0x7f == 0x7f
    codes = np.array([c for c in range(256) if c & 0x7f != 0x7f], np.uint8)
    assert np.array_equal(oracle.e4m3_encode(oracle.e4m3_decode(codes).astype(np.float32)), codes)   # exact round trip


@pytest.mark.parametrize("shape", [(5, 64), (3, 7, 96), (2, 4, 2048)])
def test_row_quantisation(shape):
    rng = np.random.default_rng(len(shape))
    W = wl.f32_to_bf16_bits((rng.standard_normal(shape) * 0.02).astype(np.float32))
    W.reshape(-1, shape[-1])[1] = 0                                     # an all-zero row
    codes, scales = oracle.quantize_rows_e4m3(W)
    w = wl.bf16_bits_to_f32(W)
    amax = np.abs(w).max(-1)
    want_s = np.where(amax == 0, np.float32(1), amax / np.float32(448)).astype(np.float32)        # numpy fp32 division
    assert np.array_equal(scales, want_s)
    q = (w / want_s[..., None]).astype(np.float32)
    assert np.array_equal(codes, _torch_encode(np.clip(q, -448, 448)))
    deq = oracle.e4m3_decode(codes) * scales[..., None].astype(np.float64)
    # never further than half a code step: steps are 2^-3 relative (normal) or 2^-9 absolute (subnormal), times the scale
    step = np.maximum(np.abs(w.astype(np.float64)) * 2.0 ** -3, scales[..., None].astype(np.float64) * 2.0 ** -9)
    assert np.all(np.abs(deq - w) <= step / 2 * (1 + 1e-6))
    nz = amax > 0
    assert np.all(np.abs(oracle.e4m3_decode(codes)).max(-1)[nz] == 448)                          # the row maximum maps to 448
    assert np.all(codes.reshape(-1, shape[-1])[1] == 0)


def _ffn_numpy(x, Wg, Wu, Wd, idx, gate, shared=None):
    """y = sum_j gate * Wd silu(Wg x) (Wu x) with numpy fp64 contractions; weights are float64 arrays."""
    T, H = x.shape
    y = np.zeros((T, H))
    for t in range(T):
        for j in range(idx.shape[1]):
            e = idx[t, j]
            a, b = Wg[e] @ x[t], Wu[e] @ x[t]
            y[t] += gate[t, j] * (Wd[e] @ ((a / (1 + np.exp(-a))) * b))
        for (Sg, Su, Sd) in shared or []:
            a, b = Sg @ x[t], Su @ x[t]
            y[t] += Sd @ ((a / (1 + np.exp(-a))) * b)
    return y


@pytest.mark.parametrize("T,H,F,N,k,S", [(5, 64, 96, 6, 2, 0), (9, 128, 64, 4, 3, 2)])
def test_quantised_ffn_is_the_ffn_of_the_dequantised_weights(T, H, F, N, k, S):
    rng = np.random.default_rng(T)
    bits = lambda shape: wl.f32_to_bf16_bits((rng.standard_normal(shape) * 0.05).astype(np.float32))
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    Wg, Wu, Wd = bits((N, F, H)), bits((N, F, H)), bits((N, H, F))
    (Qg, sg), (Qu, su), (Qd, sd) = (oracle.quantize_rows_e4m3(W) for W in (Wg, Wu, Wd))
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    gate = rng.dirichlet(np.ones(k), T)
    deq = lambda Q, s: oracle.e4m3_decode(Q) * s[..., None].astype(np.float64)
    kw, shared = {}, None
    if S:
        Sg, Su, Sd = bits((S, 32, H)), bits((S, 32, H)), bits((S, H, 32))
        (SQg, ssg), (SQu, ssu), (SQd, ssd) = (oracle.quantize_rows_e4m3(W) for W in (Sg, Su, Sd))
        kw = dict(SQg=SQg, SQu=SQu, SQd=SQd, ssg=ssg, ssu=ssu, ssd=ssd)
        shared = [(deq(SQg, ssg)[s], deq(SQu, ssu)[s], deq(SQd, ssd)[s]) for s in range(S)]
    y = oracle.moe_ffn_q8(x, Qg, Qu, Qd, sg, su, sd, idx, gate, **kw)
    y_ref = _ffn_numpy(wl.bf16_bits_to_f32(x).astype(np.float64), deq(Qg, sg), deq(Qu, su), deq(Qd, sd), idx, gate, shared)
    np.testing.assert_allclose(y, y_ref, rtol=1e-10, atol=1e-13)


def test_weights_that_e4m3_represents_exactly_give_the_bf16_result():
    """Weights of the form (E4M3 value) * 2^-5 with the row maximum at 448 * 2^-5 quantise without loss, so the
    quantised FFN must agree with the bf16 oracle."""
    rng = np.random.default_rng(3)
    T, H, F, N, k = 6, 64, 96, 4, 2
    def exact(shape):
        codes = rng.integers(0, 0x7f, size=shape).astype(np.uint8) | (rng.integers(0, 2, size=shape).astype(np.uint8) << 7)
        codes[..., 0] = 0x7e                                            # 448 in every row
        return codes, wl.f32_to_bf16_bits((oracle.e4m3_decode(codes) * 2.0 ** -5).astype(np.float32))
    (Cg, Wg), (Cu, Wu), (Cd, Wd) = exact((N, F, H)), exact((N, F, H)), exact((N, H, F))
    for C, W in ((Cg, Wg), (Cu, Wu), (Cd, Wd)):
        Q, s = oracle.quantize_rows_e4m3(W)
        assert np.array_equal(Q & 0x7f, C & 0x7f) and np.all(s == np.float32(2.0 ** -5))
        assert np.array_equal(oracle.e4m3_decode(Q), oracle.e4m3_decode(C))                     # also the sign of zeros' values
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32) * 0.1)
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    gate = rng.dirichlet(np.ones(k), T)
    (Qg, sg), (Qu, su), (Qd, sd) = (oracle.quantize_rows_e4m3(W) for W in (Wg, Wu, Wd))
    y8 = oracle.moe_ffn_q8(x, Qg, Qu, Qd, sg, su, sd, idx, gate)
    y16 = oracle.moe_ffn(x, Wg, Wu, Wd, idx, gate)
    np.testing.assert_allclose(y8, y16, rtol=1e-12, atol=1e-300)
