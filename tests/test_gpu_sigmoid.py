"""GPU parity of the sigmoid-gated router calls against the oracle (paper Sec. 3.2.1, routers without softmax).

Selections, counts, histogram and permutation are integers: bit-exact given the GPU's own fp32 logits, and identical
to what the softmax calls give on the same logits (the bins use logit differences only).  Gates (selected sigmoid
scores over their sum) and the sum of the selected scores within 1e-5; the layer output per token row within
max |y - y_ref| / max |y_ref| <= 1e-2.
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
LOGIT_TOL = 1e-5
GATE_TOL = 1e-5


@pytest.fixture(scope="module")
def L():
    import paper_2411_08982_amd as lib
    lib.lib()
    assert torch.cuda.is_available()
    return lib


@pytest.mark.parametrize("T,H,N,k", [(1, 256, 8, 2), (16, 512, 8, 2), (33, 256, 60, 4), (130, 128, 200, 9), (64, 2048, 128, 8)])
def test_route_sigmoid(L, T, H, N, k):
    print(f"route_sigmoid T={T} H={H} N={N} k={k}", flush=True)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], H=H, N=N, k=k, seed=T)
    d = wl.make_layer(cfg, T, weights=False)
    out = L.lynx_route_sigmoid(to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"]), k)
    torch.cuda.synchronize()
    ref = oracle.route(d["x"], d["Wr"], d["bias"], k)
    z = host(out["logits"])
    assert np.all(np.abs(z - ref["logits"]) <= LOGIT_TOL * np.maximum(1.0, np.abs(ref["logits"])))
    r = oracle.topk_sigmoid(z, k)
    assert np.array_equal(host(out["idx"]), r["idx"])
    np.testing.assert_allclose(host(out["gate"]), r["gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(out["psum"]), r["ssum"], rtol=GATE_TOL, atol=1e-7)
    # far from the softmax gates of the same selection
    assert not np.allclose(host(out["gate"]), oracle.topk(z, k)["gate"], rtol=1e-3) or k == 1


@pytest.mark.parametrize("T,N,k", [(8, 8, 2), (16, 64, 6), (17, 60, 4), (70, 128, 8), (300, 200, 12), (1, 8, 2)])
def test_affinity_bin_sigmoid(L, T, N, k):
    for alpha, beta, enable in [(2.0, 2, 1), (4.0, 1, 1), (0.5, 6, 1), (2.0, 2, 0)]:
        print(f"affinity_bin_sigmoid T={T} N={N} k={k} alpha={alpha} beta={beta} enable={enable}", flush=True)
        z = wl.make_logits(T, N, seed=T + N, quantum=[None, 0.25][beta % 2])
        idx = oracle.topk_sigmoid(z, k)["idx"]
        ref = oracle.affinity_bin_sigmoid(z, idx, alpha, beta, enable)
        out = L.lynx_affinity_bin_sigmoid(dev(z), dev(idx), alpha, beta, enable)
        soft = L.lynx_affinity_bin(dev(z), dev(idx), alpha, beta, enable)
        torch.cuda.synchronize()
        for key in ("new_idx", "cnt_before", "cnt_after", "bin_hist", "num_active"):
            assert np.array_equal(host(out[key]), ref[key]), key
            assert np.array_equal(host(out[key]), host(soft[key])), key      # only the gates differ from the softmax call
        np.testing.assert_allclose(host(out["new_gate"]), ref["new_gate"], rtol=GATE_TOL, atol=1e-7)
        np.testing.assert_allclose(host(out["new_psum"]), ref["new_psum"], rtol=GATE_TOL, atol=1e-7)   # sum of the scores


@pytest.mark.parametrize("T,shared", [(8, 0), (16, 1), (40, 1), (130, 0)])
def test_layer_sigmoid(L, T, shared):
    print(f"layer_sigmoid T={T} shared={shared}", flush=True)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], name="sig", H=256, F=256, N=24, k=4, n_shared=shared, F_shared=128, seed=40 + T)
    d = wl.make_layer(cfg, T)
    alpha, beta = 2.0, 2
    x, Wr, bias = to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"])
    Wgu, Wdp = L.lynx_pack_weights(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
    Sgu, Sdp = L.lynx_pack_weights(to_bf16_dev(d["Sg"]), to_bf16_dev(d["Su"]), to_bf16_dev(d["Sd"])) if shared else (None, None)
    b = L.lynx_moe_layer_sigmoid(x, Wr, bias, Wgu, Wdp, cfg.F, cfg.k, alpha, beta, 1, Sgu, Sdp, cfg.n_shared, cfg.F_shared)
    torch.cuda.synchronize()
    z = host(b.logits)
    r = oracle.route(d["x"], d["Wr"], d["bias"], cfg.k)
    assert np.all(np.abs(z - r["logits"]) <= LOGIT_TOL * np.maximum(1.0, np.abs(r["logits"])))
    tk = oracle.topk_sigmoid(z, cfg.k)
    assert np.array_equal(host(b.topk_idx), tk["idx"])
    np.testing.assert_allclose(host(b.topk_gate), tk["gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(b.topk_psum), tk["ssum"], rtol=GATE_TOL, atol=1e-7)
    a = oracle.affinity_bin_sigmoid(z, tk["idx"], alpha, beta, 1)
    for key, got in (("new_idx", b.new_idx), ("cnt_before", b.cnt_before), ("cnt_after", b.cnt_after),
                     ("bin_hist", b.bin_hist), ("num_active", b.num_active)):
        assert np.array_equal(host(got), a[key]), key
    np.testing.assert_allclose(host(b.new_gate), a["new_gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(b.new_psum), a["new_psum"], rtol=GATE_TOL, atol=1e-7)
    p = oracle.permute(a["new_idx"], cfg.N)
    for key, got in (("offsets", b.offsets), ("perm", b.perm), ("active", b.active), ("num_active", b.num_active_perm)):
        assert np.array_equal(host(got), p[key]), key
    y_ref = oracle.moe_ffn(d["x"], d["Wg"], d["Wu"], d["Wd"], a["new_idx"], a["new_gate"], d["Sg"], d["Su"], d["Sd"])
    assert row_rel_err(host(b.y), y_ref).max() <= Y_TOL
    # the separate calls give the same bits as the fused one
    r2 = L.lynx_route_sigmoid(x, Wr, bias, cfg.k)
    a2 = L.lynx_affinity_bin_sigmoid(r2["logits"], r2["idx"], alpha, beta, 1)
    p2 = L.lynx_permute(a2["new_idx"], cfg.N)
    y2 = L.lynx_moe_ffn(x, Wgu, Wdp, a2["new_idx"], a2["new_gate"], p2, cfg.N, cfg.F, Sgu, Sdp, cfg.n_shared, cfg.F_shared)
    torch.cuda.synchronize()
    assert np.array_equal(host(a2["new_gate"]), host(b.new_gate)) and np.array_equal(host(y2), host(b.y))
