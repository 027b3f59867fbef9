"""GPU parity of the group-limited router calls against the oracle (paper Sec. 1 names expert grouping; the rule is
this build's reading, stated in include/lynx.h).

Selections, counts, histogram and permutation are integers: bit-exact given the GPU's own fp32 logits.  Gates and the
third output within 1e-5; the layer output per token row within max |y - y_ref| / max |y_ref| <= 1e-2.  Outputs and
workspace are filled with 0xFF bytes before every call.
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


def _poisoned(shape, dtype):
    t = torch.empty(shape, dtype=dtype, device="cuda")
    t.view(torch.uint8).fill_(0xFF)
    return t


def _bin_out(T, N, k, beta):
    I, F = torch.int32, torch.float32
    return dict(idx=_poisoned((T, k), I), gate=_poisoned((T, k), F), psum=_poisoned((T,), F), new_idx=_poisoned((T, k), I),
                new_gate=_poisoned((T, k), F), new_psum=_poisoned((T,), F), cnt_before=_poisoned((N,), I), cnt_after=_poisoned((N,), I),
                bin_hist=_poisoned((N, beta), I), num_active=_poisoned((2,), I))


def _check_bin(out, z, k, G, tg, alpha, beta, enable, gate_fn):
    tk = oracle.topk_grouped(z, k, G, tg, gate_fn)
    assert np.array_equal(host(out["idx"]), tk["idx"])
    np.testing.assert_allclose(host(out["gate"]), tk["gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(out["psum"]), tk["third"], rtol=GATE_TOL, atol=1e-7)
    ref = oracle.affinity_bin_grouped(z, tk["idx"], G, tg, alpha, beta, enable, gate_fn)
    for key in ("new_idx", "cnt_before", "cnt_after", "bin_hist", "num_active"):
        assert np.array_equal(host(out[key]), ref[key]), key
    np.testing.assert_allclose(host(out["new_gate"]), ref["new_gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(out["new_psum"]), ref["new_psum"], rtol=GATE_TOL, atol=1e-7)
    return ref


# (T, N, k, n_group, topk_group): one workgroup (T <= 16) and many; one, two and four logits per lane; groups that
# straddle the 64-expert slots (N=160: groups of 20; N=192: groups of 48) and single-expert groups
GROUP_CASES = [(1, 8, 2, 4, 2), (8, 16, 3, 4, 2), (16, 64, 6, 8, 3), (13, 160, 6, 8, 3), (16, 256, 8, 8, 4),
               (17, 60, 4, 3, 2), (70, 128, 8, 4, 2), (64, 160, 6, 8, 3), (130, 256, 8, 8, 4), (300, 192, 9, 4, 1),
               (33, 48, 5, 48, 7), (257, 64, 6, 64, 12), (40, 256, 16, 16, 2)]


@pytest.mark.parametrize("T,N,k,G,tg", GROUP_CASES)
def test_affinity_bin_grouped(L, T, N, k, G, tg):
    for i, (alpha, beta, enable) in enumerate([(1.0, 2, 1), (4.0, 1, 1), (0.5, 6, 1), (2.0, 2, 0)]):
        gate_fn = (i + T) % 2
        print(f"affinity_bin_grouped T={T} N={N} k={k} G={G} tg={tg} alpha={alpha} beta={beta} enable={enable} gate_fn={gate_fn}",
              flush=True)
        z = wl.make_logits(T, N, seed=T + N + G, quantum=[None, 0.25][beta % 2])
        ws = torch.full((65536,), 0xFF, dtype=torch.uint8, device="cuda")
        out = L.lynx_affinity_bin_grouped(dev(z), k, G, tg, alpha, beta, gate_fn, enable, ws, _bin_out(T, N, k, beta))
        torch.cuda.synchronize()
        _check_bin(out, z, k, G, tg, alpha, beta, enable, gate_fn)


@pytest.mark.parametrize("T,N,k", [(8, 64, 6), (70, 128, 8), (33, 200, 9)])
def test_no_limit_gives_the_ungrouped_calls_bit_for_bit(L, T, N, k):
    z = wl.make_logits(T, N, seed=T)
    zd = dev(z)
    for G, tg in [(1, 1), (4, 4)] if N % 4 == 0 else [(1, 1)]:
        for gate_fn in (0, 1):
            print(f"no_limit T={T} N={N} k={k} G={G} gate_fn={gate_fn}", flush=True)
            out = L.lynx_affinity_bin_grouped(zd, k, G, tg, 1.0, 2, gate_fn)
            idx = dev((oracle.topk_sigmoid if gate_fn else oracle.topk)(z, k)["idx"])
            ref = (L.lynx_affinity_bin_sigmoid if gate_fn else L.lynx_affinity_bin)(zd, idx, 1.0, 2)
            torch.cuda.synchronize()
            assert np.array_equal(host(out["idx"]), host(idx))
            for key in ("new_idx", "new_gate", "cnt_before", "cnt_after", "bin_hist", "num_active"):
                assert np.array_equal(host(out[key]), host(ref[key])), key


def test_short_tokens_keep_their_own_picks(L):
    # one group per token and one narrow bin: many tokens find fewer than k active experts in their group
    for T in (12, 48):
        z = wl.make_logits(T, 64, seed=9)
        out = L.lynx_affinity_bin_grouped(dev(z), 6, 8, 1, 4.0, 1, 0, 1, None, _bin_out(T, 64, 6, 1))
        torch.cuda.synchronize()
        ref = _check_bin(out, z, 6, 8, 1, 4.0, 1, 1, 0)
        outside = [set(ref["new_idx"][t].tolist()) - set(np.nonzero(ref["active"])[0].tolist()) for t in range(T)]
        assert any(outside), "the case is not exercised"
    # the hand-worked case of the oracle's pins
    z = np.array([[5.0, 4.9, 0.0, 0.0], [0.0, 0.0, 5.0, -20.0]], np.float32)
    out = L.lynx_affinity_bin_grouped(dev(z), 2, 2, 1, 1.0, 1)
    torch.cuda.synchronize()
    assert host(out["new_idx"]).tolist() == [[0, 1], [2, 3]] and host(out["num_active"]).tolist() == [4, 4]


@pytest.mark.parametrize("T,H,N,k,G,tg,gate_fn", [(1, 256, 8, 2, 4, 2, 0), (16, 512, 64, 6, 8, 3, 1), (33, 256, 160, 6, 8, 3, 0),
                                                  (130, 128, 256, 8, 8, 4, 1)])
def test_route_grouped(L, T, H, N, k, G, tg, gate_fn):
    print(f"route_grouped T={T} H={H} N={N} k={k} G={G} tg={tg} gate_fn={gate_fn}", flush=True)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], H=H, N=N, k=k, seed=T)
    d = wl.make_layer(cfg, T, weights=False)
    out = L.lynx_route_grouped(to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"]), k, G, tg, gate_fn)
    torch.cuda.synchronize()
    ref = oracle.route(d["x"], d["Wr"], d["bias"], k)
    z = host(out["logits"])
    assert np.all(np.abs(z - ref["logits"]) <= LOGIT_TOL * np.maximum(1.0, np.abs(ref["logits"])))
    r = oracle.topk_grouped(z, k, G, tg, gate_fn)
    assert np.array_equal(host(out["idx"]), r["idx"])
    np.testing.assert_allclose(host(out["gate"]), r["gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(out["psum"]), r["third"], rtol=GATE_TOL, atol=1e-7)
    assert np.take_along_axis(oracle.group_allowed(z, G, tg), host(out["idx"]), 1).all()


@pytest.mark.parametrize("T,shared,gate_fn", [(8, 0, 1), (16, 1, 0), (40, 1, 1), (130, 0, 0)])
def test_layer_grouped(L, T, shared, gate_fn):
    print(f"layer_grouped T={T} shared={shared} gate_fn={gate_fn}", flush=True)
    G, tg = 6, 2
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], name="grp", H=256, F=256, N=24, k=4, n_shared=shared, F_shared=128, seed=60 + T)
    d = wl.make_layer(cfg, T)
    alpha, beta = 1.0, 2
    x, Wr, bias = to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"])
    Wgu, Wdp = L.lynx_pack_weights(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
    Sgu, Sdp = L.lynx_pack_weights(to_bf16_dev(d["Sg"]), to_bf16_dev(d["Su"]), to_bf16_dev(d["Sd"])) if shared else (None, None)
    b = L.lynx_moe_layer_grouped(x, Wr, bias, Wgu, Wdp, cfg.F, cfg.k, G, tg, alpha, beta, gate_fn, 1, Sgu, Sdp, cfg.n_shared,
                                 cfg.F_shared)
    torch.cuda.synchronize()
    z = host(b.logits)
    r = oracle.route(d["x"], d["Wr"], d["bias"], cfg.k)
    assert np.all(np.abs(z - r["logits"]) <= LOGIT_TOL * np.maximum(1.0, np.abs(r["logits"])))
    got = dict(idx=b.topk_idx, gate=b.topk_gate, psum=b.topk_psum, new_idx=b.new_idx, new_gate=b.new_gate,
               new_psum=b.new_psum, cnt_before=b.cnt_before, cnt_after=b.cnt_after, bin_hist=b.bin_hist, num_active=b.num_active)
    a = _check_bin(got, z, cfg.k, G, tg, alpha, beta, 1, gate_fn)
    p = oracle.permute(a["new_idx"], cfg.N)
    for key, val in (("offsets", b.offsets), ("perm", b.perm), ("active", b.active), ("num_active", b.num_active_perm)):
        assert np.array_equal(host(val), p[key]), key
    y_ref = oracle.moe_ffn(d["x"], d["Wg"], d["Wu"], d["Wd"], a["new_idx"], a["new_gate"], d["Sg"], d["Su"], d["Sd"])
    assert row_rel_err(host(b.y), y_ref).max() <= Y_TOL
    # the separate calls give the same bits as the fused one
    r2 = L.lynx_route_grouped(x, Wr, bias, cfg.k, G, tg, gate_fn)
    a2 = L.lynx_affinity_bin_grouped(r2["logits"], cfg.k, G, tg, alpha, beta, gate_fn, 1)
    p2 = L.lynx_permute(a2["new_idx"], cfg.N)
    y2 = L.lynx_moe_ffn(x, Wgu, Wdp, a2["new_idx"], a2["new_gate"], p2, cfg.N, cfg.F, Sgu, Sdp, cfg.n_shared, cfg.F_shared)
    torch.cuda.synchronize()
    assert np.array_equal(host(r2["idx"]), host(b.topk_idx)) and np.array_equal(host(a2["new_idx"]), host(b.new_idx))
    assert np.array_equal(host(a2["new_gate"]), host(b.new_gate)) and np.array_equal(host(y2), host(b.y))


def test_bad_arguments(L):
    z = torch.zeros((4, 12), dtype=torch.float32, device="cuda")
    for G, tg, k, gate_fn, code in [(5, 2, 2, 0, L.binding.ERR_INVALID_ARG), (4, 5, 2, 0, L.binding.ERR_INVALID_ARG),
                                    (0, 1, 2, 0, L.binding.ERR_INVALID_ARG), (4, 1, 4, 0, L.binding.ERR_INVALID_ARG),
                                    (4, 2, 2, 2, L.binding.ERR_INVALID_ARG)]:
        with pytest.raises(L.LynxError) as e:
            L.lynx_affinity_bin_grouped(z, k, G, tg, 1.0, 2, gate_fn)
        assert e.value.code == code
    z = torch.zeros((4, 256), dtype=torch.float32, device="cuda")
    with pytest.raises(L.LynxError) as e:
        L.lynx_affinity_bin_grouped(z, 2, 128, 2, 1.0, 2)
    assert e.value.code == L.binding.ERR_UNSUPPORTED


def test_zero_tokens_and_single_token(L):
    cfg = wl.CONFIGS["tiny"]                                        # 8 experts, top-2
    d = wl.make_layer(cfg, 0)
    Wgu, Wdp = L.lynx_pack_weights(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
    x = torch.empty((0, cfg.H), dtype=torch.bfloat16, device="cuda")
    b = L.lynx_moe_layer_grouped(x, dev(d["Wr"]), dev(d["bias"]), Wgu, Wdp, cfg.F, cfg.k, 4, 2, 2.0, 2, 1)
    torch.cuda.synchronize()
    assert host(b.num_active).tolist() == [0, 0] and host(b.num_active_perm).tolist() == [0]
    assert np.all(host(b.offsets) == 0) and np.all(host(b.active) == -1) and np.all(host(b.cnt_before) == 0)
    # one token: nothing to share, the group-limited selection stays
    d = wl.make_layer(cfg, 1)
    b = L.lynx_moe_layer_grouped(to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"]), Wgu, Wdp, cfg.F, cfg.k, 4, 1, 2.0, 2, 0)
    torch.cuda.synchronize()
    z = host(b.logits)
    tk = oracle.topk_grouped(z, cfg.k, 4, 1, 0)
    assert np.array_equal(host(b.topk_idx), tk["idx"]) and np.array_equal(host(b.new_idx), tk["idx"])
    assert host(b.topk_idx)[0, 0] // 2 == host(b.topk_idx)[0, 1] // 2      # both picks in the one allowed group of two
    y_ref = oracle.moe_ffn(d["x"], d["Wg"], d["Wu"], d["Wd"], tk["idx"], tk["gate"])
    assert row_rel_err(host(b.y), y_ref).max() <= Y_TOL
