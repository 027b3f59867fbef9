"""Pins for the plain steps of the CPU oracle: router, top-k, permutation, SwiGLU FFN + combine.

Each of these steps has a textbook definition, so the oracle is checked against library routines
(numpy fp64 matmul, scipy softmax, numpy stable argsort, torch fp64 silu/matmul) and closed forms.
"""
import numpy as np
import pytest
import scipy.special
import torch

import oracle
import workloads as wl


def _f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def _lex_topk(z, k):
    """k largest per row, ties to the lower index: sort by (-z, index)."""
    T, N = z.shape
    out = np.zeros((T, k), np.int32)
    for t in range(T):
        order = np.lexsort((np.arange(N), -z[t].astype(np.float64)))
        out[t] = order[:k]
    return out


@pytest.mark.parametrize("T,H,N,k", [(5, 64, 8, 2), (16, 512, 8, 2), (7, 96, 60, 4), (3, 128, 128, 8), (1, 32, 4, 4)])
def test_route_matches_library(T, H, N, k):
    rng = np.random.default_rng(T * 1000 + N)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    Wr = (rng.standard_normal((N, H)) / np.sqrt(H)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    r = oracle.route(x, Wr, bias, k)
    z_ref = _f64(x) @ Wr.astype(np.float64).T + bias.astype(np.float64)
    # both are fp64 sums rounded once to fp32: at most 1 ulp apart
    assert np.all(np.abs(r["logits"].astype(np.float64) - z_ref) <= np.spacing(np.abs(z_ref).astype(np.float32)))
    assert np.array_equal(r["idx"], _lex_topk(r["logits"], k))
    p = scipy.special.softmax(r["logits"].astype(np.float64), axis=1)
    psel = np.take_along_axis(p, r["idx"].astype(np.int64), axis=1)
    np.testing.assert_allclose(r["psum"], psel.sum(1), rtol=1e-12)
    np.testing.assert_allclose(r["gate"], psel / psel.sum(1, keepdims=True), rtol=1e-12)
    np.testing.assert_allclose(r["gate"].sum(1), 1.0, rtol=1e-12)
    assert np.all(np.diff(r["gate"], axis=1) <= 0)


def test_route_bias_only_and_no_bias():
    H, N, k = 32, 6, 3
    x = np.zeros((2, H), np.uint16)
    Wr = np.ones((N, H), np.float32)
    bias = np.array([0.5, -1.0, 2.0, 2.0, 0.25, 1.0], np.float32)
    r = oracle.route(x, Wr, bias, k)
    assert np.array_equal(r["logits"], np.tile(bias, (2, 1)))
    assert np.array_equal(r["idx"], np.tile(np.array([2, 3, 5], np.int32), (2, 1)))  # tie 2.0: lower index first
    r0 = oracle.route(x, Wr, None, k)
    assert np.all(r0["logits"] == 0) and np.array_equal(r0["idx"][0], [0, 1, 2])
    np.testing.assert_allclose(r0["gate"], 1.0 / 3, rtol=1e-15)
    np.testing.assert_allclose(r0["psum"], 0.5, rtol=1e-15)


def test_route_exact_integer_logits_with_ties():
    # one-hot tokens pick out columns of an integer router: logits are exact small integers with many ties
    H = N = 8
    rng = np.random.default_rng(5)
    Wr = rng.integers(-2, 3, size=(N, H)).astype(np.float32)
    x = wl.f32_to_bf16_bits(np.eye(H, dtype=np.float32))
    r = oracle.route(x, Wr, None, 3)
    assert np.array_equal(r["logits"], Wr.T)  # z[t,e] = Wr[e,t]: a transposed operand would fail here
    assert np.array_equal(r["idx"], _lex_topk(Wr.T.copy(), 3))


def test_route_errors():
    x = np.zeros((1, 8), np.uint16)
    Wr = np.zeros((2, 8), np.float32)
    with pytest.raises(oracle.OracleError) as ei:
        oracle.route(x, Wr, None, 3)
    assert ei.value.code == oracle.ERR_UNSUPPORTED


@pytest.mark.parametrize("T,N,k,seed", [(1, 4, 2, 0), (16, 8, 2, 1), (37, 60, 4, 2), (128, 128, 8, 3), (0, 8, 2, 4)])
def test_permute_matches_stable_argsort(T, N, k, seed):
    rng = np.random.default_rng(seed)
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32) if T else np.zeros((0, k), np.int32)
    p = oracle.permute(idx, N)
    flat = idx.reshape(-1)
    assert np.array_equal(p["perm"], np.argsort(flat, kind="stable").astype(np.int32))
    counts = np.bincount(flat, minlength=N)
    assert np.array_equal(p["offsets"], np.concatenate([[0], np.cumsum(counts)]).astype(np.int32))
    act = np.nonzero(counts)[0]
    assert p["num_active"][0] == len(act)
    assert np.array_equal(p["active"][:len(act)], act) and np.all(p["active"][len(act):] == -1)


def _torch_moe(x, Wg, Wu, Wd, idx, gate, Sg=None, Su=None, Sd=None):
    """Independent dense fp64 statement: every (token, slot) pair computed on its own with torch."""
    xt = torch.from_numpy(_f64(x))
    T, H = xt.shape
    y = torch.zeros(T, H, dtype=torch.float64)

    def ffn(g, u, d, v):
        g, u, d = (torch.from_numpy(_f64(a)) for a in (g, u, d))
        return d @ (torch.nn.functional.silu(g @ v) * (u @ v))

    for t in range(T):
        for j in range(idx.shape[1]):
            e = int(idx[t, j])
            y[t] += float(gate[t, j]) * ffn(Wg[e], Wu[e], Wd[e], xt[t])
        if Sg is not None:
            for s in range(Sg.shape[0]):
                y[t] += ffn(Sg[s], Su[s], Sd[s], xt[t])
    return y.numpy()


@pytest.mark.parametrize("T,H,F,N,k,S,Fs", [(6, 64, 96, 5, 2, 0, 0), (9, 48, 80, 7, 3, 2, 40), (1, 32, 64, 3, 1, 1, 96)])
def test_ffn_matches_dense_torch(T, H, F, N, k, S, Fs):
    rng = np.random.default_rng(T + H)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    Wg, Wu = wl.bf16_normal(rng, (N, F, H), 0.3), wl.bf16_normal(rng, (N, F, H), 0.3)
    Wd = wl.bf16_normal(rng, (N, H, F), 0.3)
    Sg = Su = Sd = None
    if S:
        Sg, Su = wl.bf16_normal(rng, (S, Fs, H), 0.3), wl.bf16_normal(rng, (S, Fs, H), 0.3)
        Sd = wl.bf16_normal(rng, (S, H, Fs), 0.3)
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    gate = rng.random((T, k))
    gate /= gate.sum(1, keepdims=True)
    y = oracle.moe_ffn(x, Wg, Wu, Wd, idx, gate, Sg, Su, Sd)
    y_ref = _torch_moe(x, Wg, Wu, Wd, idx, gate, Sg, Su, Sd)
    np.testing.assert_allclose(y, y_ref, rtol=1e-10, atol=1e-12)
    assert np.abs(y_ref).max() > 1e-3  # not a vacuous comparison


def test_ffn_single_expert_is_plain_mlp_and_gate_scales():
    rng = np.random.default_rng(9)
    H, F = 16, 24
    x = wl.f32_to_bf16_bits(rng.standard_normal((1, H)).astype(np.float32))
    Wg, Wu, Wd = (wl.bf16_normal(rng, s, 0.5) for s in ((1, F, H), (1, F, H), (1, H, F)))
    idx = np.zeros((1, 1), np.int32)
    y1 = oracle.moe_ffn(x, Wg, Wu, Wd, idx, np.ones((1, 1)))
    a, b = _f64(Wg[0]) @ _f64(x[0]), _f64(Wu[0]) @ _f64(x[0])
    ref = _f64(Wd[0]) @ (a * scipy.special.expit(a) * b)
    np.testing.assert_allclose(y1[0], ref, rtol=1e-12)
    yh = oracle.moe_ffn(x, Wg, Wu, Wd, idx, np.full((1, 1), 0.25))
    np.testing.assert_allclose(yh, 0.25 * y1, rtol=1e-14)


def test_ffn_zero_tokens_and_errors():
    H, F, N = 8, 8, 2
    W = np.zeros((N, F, H), np.uint16)
    y = oracle.moe_ffn(np.zeros((0, H), np.uint16), W, W, np.zeros((N, H, F), np.uint16), np.zeros((0, 1), np.int32),
                       np.zeros((0, 1)))
    assert y.shape == (0, H)
    with pytest.raises(oracle.OracleError):
        oracle.moe_ffn(np.zeros((1, H), np.uint16), W, W, np.zeros((N, H, F), np.uint16),
                       np.full((1, 1), 5, np.int32), np.ones((1, 1)))


def test_bf16_rounding_helper_is_round_to_nearest_even():
    v = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 3.0e38], np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to even mantissa (1.0); 1 + 3*2^-9 rounds up
    got = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(v))
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == 1.0078125 and got[3] == 1.015625
    t = torch.from_numpy(v).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, t)
