"""GPU parity of the MXFP4 (E2M1 elements, E8M0 block scales, weight-only) expert-weight path against the oracle.

Quantisation decides integers (codes and scale exponents), so both must be bit-exact.  A code times its scale is
exactly a bf16 number, so the FFN output is compared with the oracle's bf16 FFN over the dequantised weights, at
the bar of the bf16 path (per token row: max |y - y_ref| / max |y_ref| <= 1e-2).
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


def unpack_fp4(packed: np.ndarray, nmat: int) -> list:
    """[E, R/16, K/128, nmat, 64, 16] bytes -> nmat arrays [E, R, K] of codes: byte j of lane l of a tile holds
    row l%16, columns (l//16)*32 + 2j (low nibble) and 2j+1."""
    E, RT, KT = packed.shape[:3]
    lo, hi = packed & 0xf, packed >> 4
    codes = np.stack([lo, hi], axis=-1).reshape(E, RT, KT, nmat, 4, 16, 32)       # e, rt, kt, m, g, r, c
    t = codes.transpose(3, 0, 1, 5, 2, 4, 6)                                       # m, e, rt, r, kt, g, c
    return [np.ascontiguousarray(t[m]).reshape(E, RT * 16, KT * 128) for m in range(nmat)]


def unpack_scales(words: np.ndarray, K: int, gate_up: bool) -> list:
    """[E, groups, KT4, 64, 2] int32 -> arrays [E, R, K/32] of exponents (gate and up, or the one down matrix)."""
    E, G, KT4 = words.shape[:3]
    KT = K // 128
    b = words.view(np.uint8).reshape(E, G, KT4, 4, 16, 2, 4)                      # e, grp, kt4, g, r, which, byte
    t = b.transpose(5, 0, 1, 4, 2, 6, 3)                                           # which, e, grp, r, kt4, byte, g
    t = t.reshape(2, E, G, 16, KT4 * 4, 4)[:, :, :, :, :KT]                        # which, e, grp, r, kt, g
    if gate_up:
        return [np.ascontiguousarray(t[m]).reshape(E, G * 16, KT * 4) for m in range(2)]
    both = t.transpose(1, 2, 0, 3, 4, 5)                                           # e, pair, which, r, kt, g
    return [np.ascontiguousarray(both).reshape(E, G * 32, KT * 4)]


@pytest.mark.parametrize("E,H,F", [(2, 128, 128), (3, 256, 384), (2, 640, 1408)])
def test_quantize_weights(L, E, H, F):
    print(f"quantize fp4 E={E} H={H} F={F}", flush=True)
    rng = np.random.default_rng(E * H)
    bits = lambda shape: wl.f32_to_bf16_bits((rng.standard_normal(shape) * 0.02 * np.exp(rng.uniform(-2, 2, shape[:2] + (1,)))
                                             ).astype(np.float32))
    Wg, Wu, Wd = bits((E, F, H)), bits((E, F, H)), bits((E, H, F))
    Wg[0, 1, :64] = 0                                                         # two all-zero blocks
    Wd[0, 0, 0] = wl.f32_to_bf16_bits(np.array([2.0 ** -3], np.float32))[0]   # powers of two and the values around them
    Wd[0, 0, 1:32] = 0
    q = L.lynx_quantize_weights_fp4(to_bf16_dev(Wg), to_bf16_dev(Wu), to_bf16_dev(Wd))
    torch.cuda.synchronize()
    (Qg, eg), (Qu, eu), (Qd, ed) = (oracle.quantize_mxfp4(W) for W in (Wg, Wu, Wd))
    g, u = unpack_fp4(host(q.Wgu_q), 2)
    (d,) = unpack_fp4(host(q.Wd_q)[:, :, :, None], 1)
    sg, su = unpack_scales(host(q.scales_gu), H, True)
    (sd,) = unpack_scales(host(q.scales_d), F, False)
    assert np.array_equal(sg, eg) and np.array_equal(su, eu) and np.array_equal(sd, ed)
    assert np.array_equal(g, Qg) and np.array_equal(u, Qu) and np.array_equal(d, Qd)


FFN_CASES = [
    # T,  N,  k,  H,   F,  S, Fs
    (1, 4, 2, 128, 256, 0, 0),          # one token (direct path, K split)
    (8, 8, 2, 256, 512, 0, 0),
    (16, 20, 4, 128, 384, 1, 128),      # shared expert, direct
    (24, 6, 3, 256, 256, 1, 128),       # staged path, single launch
    (70, 5, 2, 128, 128, 2, 128),       # more than 64 tokens: 128-token passes
    (200, 16, 4, 128, 128, 0, 0),
    (8, 8, 2, 128, 128, 1, 640),        # shared expert wider than the routed ones: its down projection is split over K
    (20, 8, 2, 128, 128, 1, 384),       # the same on the staged path
]


@pytest.mark.parametrize("T,N,k,H,F,S,Fs", FFN_CASES)
def test_ffn_fp4(L, T, N, k, H, F, S, Fs):
    print(f"ffn fp4 T={T} N={N} k={k} H={H} F={F} shared={S}x{Fs}", flush=True)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], name="fp4", H=H, F=F, N=N, k=k, n_shared=S, F_shared=Fs, seed=T + N)
    d = wl.make_layer(cfg, T)
    x, Wr, bias = to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"])
    q = L.lynx_quantize_weights_fp4(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
    sh = L.lynx_quantize_weights_fp4(to_bf16_dev(d["Sg"]), to_bf16_dev(d["Su"]), to_bf16_dev(d["Sd"])) if S else None
    (Qg, eg), (Qu, eu), (Qd, ed) = (oracle.quantize_mxfp4(d[n]) for n in ("Wg", "Wu", "Wd"))
    shared = ()
    if S:
        (SQg, seg), (SQu, seu), (SQd, sed) = (oracle.quantize_mxfp4(d[n]) for n in ("Sg", "Su", "Sd"))
        shared = (SQg, SQu, SQd, seg, seu, sed)
    # whole layer through the fused entry point ...
    b = L.lynx_moe_layer_fp4(x, Wr, bias, q, F, k, 2.0, 2, 1, sh, S, Fs)
    torch.cuda.synchronize()
    from paper_2411_08982_amd.binding import WAIT_FLAG_WORD
    assert int(b.workspace.view(torch.int32)[WAIT_FLAG_WORD]) == 0
    z = host(b.logits)
    a = oracle.affinity_bin(z, oracle.topk(z, k)["idx"], 2.0, 2, 1)
    assert np.array_equal(host(b.new_idx), a["new_idx"])
    y_ref = oracle.moe_ffn_q4(d["x"], Qg, Qu, Qd, eg, eu, ed, a["new_idx"], a["new_gate"], *shared)
    err = row_rel_err(host(b.y), y_ref)
    assert err.max() <= Y_TOL, f"layer: max row error {err.max():.3e}"
    # ... and the FFN alone after the separate routing calls: identical output
    p = L.lynx_permute(b.new_idx, N)
    y2 = L.lynx_moe_ffn_fp4(x, q, b.new_idx, b.new_gate, p, N, F, sh, S, Fs)
    torch.cuda.synchronize()
    assert np.array_equal(host(y2), host(b.y))
    # quantisation error itself (against the bf16 weights) stays at the level four bits imply
    y16 = oracle.moe_ffn(d["x"], d["Wg"], d["Wu"], d["Wd"], a["new_idx"], a["new_gate"], d["Sg"], d["Su"], d["Sd"])
    assert row_rel_err(y_ref, y16).max() < 0.6


def test_argument_errors(L):
    one = torch.zeros(16, dtype=torch.int32, device="cuda")
    lib = L.lib()
    p = one.data_ptr()
    assert lib.lynx_quantize_weights_fp4(p, p, p, 1, 192, 128, p, p, p, p, None) == -2       # H not a multiple of 128
    assert lib.lynx_quantize_weights_fp4(p, p, p, 1, 128, 128, p, None, p, p, None) == -1    # null pointer
    assert lib.lynx_fp4_scale_words(2, 256, 640, 1) == 2 * 16 * 2 * 128 and lib.lynx_fp4_scale_words(2, 256, 640, 0) == 2 * 8 * 2 * 128
