"""GPU parity of the FP8 (E4M3, weight-only) expert-weight path against the oracle.

Quantisation decides integers (the codes), so codes and scales must be bit-exact; the FFN output is compared
with the oracle's FFN over the same codes and scales (per token row: max |y - y_ref| / max |y_ref| <= 1e-2, the
bar of the bf16 path: the conversion of the codes to bf16 is exact and the intermediate vector is rounded to
bf16 in both paths' GPU side only).
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import dev, host, row_rel_err, to_bf16_dev

pytestmark = pytest.mark.gpu

Y_TOL = 1e-2


@pytest.fixture(scope="module")
def L():
    import paper_2411_08982_amd as lib
    lib.lib()
    assert torch.cuda.is_available()
    return lib


def unpack_fp8(packed: np.ndarray, nmat: int) -> list:
    """[E, R/16, K/64, nmat, 64, 16] bytes -> nmat arrays [E, R, K]: entry (lane l, i) of a tile is row l%16,
    column (l//16)*16 + i."""
    E, RT, KT = packed.shape[:3]
    t = packed.reshape(E, RT, KT, nmat, 4, 16, 16)            # e, rt, kt, m, g, r, i
    t = t.transpose(3, 0, 1, 5, 2, 4, 6)                       # m, e, rt, r, kt, g, i
    return [np.ascontiguousarray(t[m]).reshape(E, RT * 16, KT * 64) for m in range(nmat)]


def test_hardware_decode_of_all_codes(L):
    """The conversion instruction the kernels use must decode every E4M3 code as the oracle does: checked through
    the FFN itself with one-hot tokens, which read single weight columns."""
    H = F = 64
    codes = np.arange(256, dtype=np.uint8)
    codes = codes[(codes & 0x7f) != 0x7f]                                     # all 254 finite codes
    vals = oracle.e4m3_decode(codes) * 2.0 ** -5                              # bf16-exact weights
    Wd = np.zeros((1, H, F), np.float32)
    for i, v in enumerate(vals):                                              # every code somewhere in columns 0..62
        Wd[0, i // 63, i % 63] = v
    Wd[0, :, 63] = 448 * 2.0 ** -5                                            # row maximum: scale 2^-5 in every row
    Wg = np.zeros((1, F, H), np.float32)
    Wu = np.zeros((1, F, H), np.float32)
    Wg[0, np.arange(F), np.arange(F)] = 448 * 2.0 ** -5                       # gate = up = 14 * x
    Wu[0, np.arange(F), np.arange(F)] = 448 * 2.0 ** -5
    bits = [wl.f32_to_bf16_bits(W) for W in (Wg, Wu, Wd)]
    q = L.lynx_quantize_weights_fp8(*(to_bf16_dev(b) for b in bits))
    x = np.zeros((F, H), np.float32)
    x[np.arange(F), np.arange(F)] = 0.25                                      # token t is 0.25 * e_t
    xb = wl.f32_to_bf16_bits(x)
    idx = np.zeros((F, 1), np.int32)
    gate = np.ones((F, 1), np.float32)
    p = L.lynx_permute(dev(idx), 1)
    y = L.lynx_moe_ffn_fp8(to_bf16_dev(xb), q, dev(idx), dev(gate), p, 1, F)
    torch.cuda.synchronize()
    (Qg, sg), (Qu, su), (Qd, sd) = (oracle.quantize_rows_e4m3(b) for b in bits)
    y_ref = oracle.moe_ffn_q8(xb, Qg, Qu, Qd, sg, su, sd, idx, gate.astype(np.float64))
    for i, c in enumerate(codes):
        assert Qd[0, i // 63, i % 63] & 0x7f == c & 0x7f                      # the weights quantise back to the codes
    # h_t = silu(3.5) * 3.5 in feature t only, so y[t, r] = Wd[r, t] * h_t: one code per output element, and the
    # only rounding besides fp32 is h to bf16 (2^-9 relative)
    got = host(y).astype(np.float64)
    assert np.all(np.abs(got - y_ref) <= 4e-3 * np.abs(y_ref)), np.abs(got - y_ref).max()
    assert np.count_nonzero(y_ref) >= 252


@pytest.mark.parametrize("E,H,F", [(3, 64, 128), (2, 256, 192), (8, 512, 1024)])
def test_quantize_weights(L, E, H, F):
    print(f"quantize E={E} H={H} F={F}", flush=True)
    rng = np.random.default_rng(E * H)
    bits = lambda shape: wl.f32_to_bf16_bits((rng.standard_normal(shape) * 0.02 * np.exp(rng.uniform(-2, 2, shape[:2] + (1,)))
                                             ).astype(np.float32))
    Wg, Wu, Wd = bits((E, F, H)), bits((E, F, H)), bits((E, H, F))
    Wg[0, 1] = 0                                                              # an all-zero row
    q = L.lynx_quantize_weights_fp8(to_bf16_dev(Wg), to_bf16_dev(Wu), to_bf16_dev(Wd))
    torch.cuda.synchronize()
    (Qg, sg), (Qu, su), (Qd, sd) = (oracle.quantize_rows_e4m3(W) for W in (Wg, Wu, Wd))
    s_gu = host(q.scales_gu)
    assert np.array_equal(s_gu[:, 0], sg) and np.array_equal(s_gu[:, 1], su) and np.array_equal(host(q.scales_d), sd)
    g, u = unpack_fp8(host(q.Wgu_q), 2)
    (d,) = unpack_fp8(host(q.Wd_q)[:, :, :, None], 1)
    assert np.array_equal(g, Qg) and np.array_equal(u, Qu) and np.array_equal(d, Qd)


FFN_CASES = [
    # T,  N,  k,  H,   F,  S, Fs
    (1, 4, 2, 128, 256, 0, 0),          # one token (direct path, K split)
    (8, 8, 2, 256, 512, 0, 0),
    (16, 20, 4, 128, 192, 1, 64),       # shared expert, direct
    (24, 6, 3, 192, 256, 1, 128),       # staged path, single launch
    (70, 5, 2, 128, 128, 2, 64),        # more than 64 tokens: 128-token passes
    (200, 16, 4, 64, 64, 0, 0),
    (8, 8, 2, 128, 64, 1, 256),         # shared expert wider than the routed ones: its down projection is split over K
    (20, 8, 2, 128, 64, 1, 192),        # the same on the staged path (3 slices of one 64-column tile each)
]


@pytest.mark.parametrize("T,N,k,H,F,S,Fs", FFN_CASES)
def test_ffn_fp8(L, T, N, k, H, F, S, Fs):
    print(f"ffn fp8 T={T} N={N} k={k} H={H} F={F} shared={S}x{Fs}", flush=True)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], name="fp8", H=H, F=F, N=N, k=k, n_shared=S, F_shared=Fs, seed=T + N)
    d = wl.make_layer(cfg, T)
    x, Wr, bias = to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"])
    q = L.lynx_quantize_weights_fp8(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
    sh = L.lynx_quantize_weights_fp8(to_bf16_dev(d["Sg"]), to_bf16_dev(d["Su"]), to_bf16_dev(d["Sd"])) if S else None
    (Qg, sg), (Qu, su), (Qd, sd) = (oracle.quantize_rows_e4m3(d[n]) for n in ("Wg", "Wu", "Wd"))
    kw = {}
    if S:
        (SQg, ssg), (SQu, ssu), (SQd, ssd) = (oracle.quantize_rows_e4m3(d[n]) for n in ("Sg", "Su", "Sd"))
        kw = dict(SQg=SQg, SQu=SQu, SQd=SQd, ssg=ssg, ssu=ssu, ssd=ssd)
    # whole layer through the fused entry point ...
    b = L.lynx_moe_layer_fp8(x, Wr, bias, q, F, k, 2.0, 2, 1, sh, S, Fs)
    torch.cuda.synchronize()
    from paper_2411_08982_amd.binding import WAIT_FLAG_WORD
    assert int(b.workspace.view(torch.int32)[WAIT_FLAG_WORD]) == 0
    z = host(b.logits)
    a = oracle.affinity_bin(z, oracle.topk(z, k)["idx"], 2.0, 2, 1)
    assert np.array_equal(host(b.new_idx), a["new_idx"])
    y_ref = oracle.moe_ffn_q8(d["x"], Qg, Qu, Qd, sg, su, sd, a["new_idx"], a["new_gate"], **kw)
    err = row_rel_err(host(b.y), y_ref)
    assert err.max() <= Y_TOL, f"layer: max row error {err.max():.3e}"
    # ... and the FFN alone after the separate routing calls: identical output
    p = L.lynx_permute(b.new_idx, N)
    y2 = L.lynx_moe_ffn_fp8(x, q, b.new_idx, b.new_gate, p, N, F, sh, S, Fs)
    torch.cuda.synchronize()
    assert np.array_equal(host(y2), host(b.y))
    # quantisation error itself (against the bf16 weights) stays at the few-percent level E4M3 implies
    y16 = oracle.moe_ffn(d["x"], d["Wg"], d["Wu"], d["Wd"], a["new_idx"], a["new_gate"], d["Sg"], d["Su"], d["Sd"])
    assert row_rel_err(y_ref, y16).max() < 0.2
