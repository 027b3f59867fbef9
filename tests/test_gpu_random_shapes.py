"""GPU parity on seeded random shapes: the whole MoE decode layer (bf16 / FP8 / MXFP4 expert weights), the FFN alone
with token distributions no router produces, and the binning entry points alone.

The hand-picked cases elsewhere aim at known boundaries (tile edges, the 16-, 64- and 128-token limits).  This
sweep draws shapes nobody chose: token counts, hidden and FFN widths that are odd multiples of the tile sizes,
expert counts from 2 to 256, k up to 16, zero to two shared experts narrower or wider than the routed ones, and
binning parameters over their whole range.  Inputs sit in front of a poisoned tail and outputs and workspace start
poisoned, so that a read past an input's end or of memory nobody wrote shows in the result.  Every case goes through
the fused entry point and is compared
with the oracle step by step: logits within 1e-5 (relative to max(1, |z|)), every integer of routing, binning and
permutation bit-exact given the GPU's logits, gates within 1e-5, and the layer output per token row within
max |y - y_ref| / max |y_ref| <= 1e-2.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import host, row_rel_err, with_poisoned_tail
from gpu_util import dev as plain_dev, to_bf16_dev as plain_to_bf16_dev

pytestmark = pytest.mark.gpu

Y_TOL = 1e-2
LOGIT_TOL = 1e-5
GATE_TOL = 1e-5
N_CASES = 30


def dev(a):
    return with_poisoned_tail(plain_dev(a))


def to_bf16_dev(bits):
    return with_poisoned_tail(plain_to_bf16_dev(bits))


@pytest.fixture(scope="module")
def L():
    import paper_2411_08982_amd as lib
    lib.lib()
    assert torch.cuda.is_available()
    return lib


def draw_case(i):
    """Case i of the sweep: (weight format, config, T, alpha, beta, enable).  The formats rotate; the column
    multiple of a weight tile is 32 (bf16), 64 (FP8) or 128 (MXFP4)."""
    rng = np.random.default_rng([2411, 8982, i])
    fmt = ("bf16", "fp8", "fp4")[i % 3]
    mult = {"bf16": 32, "fp8": 64, "fp4": 128}[fmt]
    T = int(rng.choice([1, 2, 3, 5, 9, 15, 16, 17, 23, 31, 33, 47, 64, 65, 90, 129, 150, 200]))
    N = int(rng.choice([2, 3, 5, 8, 13, 31, 60, 64, 65, 100, 128, 129, 200, 256]))
    k = int(rng.integers(1, min(N, 16) + 1))
    wide = N < 100    # many experts: narrower ones, so that the oracle's quantisers stay in seconds
    H = mult * int(rng.integers(1, (512 if wide else 256) // mult + 1))
    F = mult * int(rng.integers(1, (384 if wide else 128) // mult + 1))
    S = int(rng.choice([0, 0, 1, 2]))
    Fs = mult * int(rng.integers(1, 640 // mult + 1)) if S else 0
    alpha = float(rng.choice([0.5, 1.0, 2.0, 4.0, 8.0]))
    beta = int(rng.integers(1, 7))
    enable = int(rng.random() < 0.85)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], name=f"random{i}", H=H, F=F, N=N, k=k, n_shared=S, F_shared=Fs,
                              zipf_s=float(rng.choice([0.0, 0.9, 1.3])), bias_scale=float(rng.choice([0.0, 0.5, 2.0])),
                              tail_frac=float(rng.choice([0.0, 0.1])), seed=1000 + i)
    return fmt, cfg, T, alpha, beta, enable


def poisoned_buffers(L, cfg, T, beta):
    """Outputs and workspace of a layer call filled with NaN / -1 patterns: the library must not rely on anything a
    fresh allocation happens to hold (in a new process that is usually zeros, which hides a missing clear or an
    output row nobody writes)."""
    b = L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, beta, cfg.n_shared, cfg.F_shared)
    for t in vars(b).values():
        if torch.is_tensor(t):
            t.view(torch.uint8).fill_(0xFF)
    return b


def run_layer(L, fmt, cfg, d, alpha, beta, enable, sigmoid=False):
    """The fused layer call for the given weight format, and the oracle's FFN over the same (quantised) weights."""
    x, Wr, bias = to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"])
    buf = poisoned_buffers(L, cfg, x.shape[0], beta)
    routed = [to_bf16_dev(d[n]) for n in ("Wg", "Wu", "Wd")]
    shared = [to_bf16_dev(d[n]) for n in ("Sg", "Su", "Sd")] if cfg.n_shared else None
    tail = (cfg.n_shared, cfg.F_shared)
    if fmt == "bf16":
        Wgu, Wdp = L.lynx_pack_weights(*routed)
        Sgu, Sdp = L.lynx_pack_weights(*shared) if shared else (None, None)
        entry = L.lynx_moe_layer_sigmoid if sigmoid else L.lynx_moe_layer
        b = entry(x, Wr, bias, Wgu, Wdp, cfg.F, cfg.k, alpha, beta, enable, Sgu, Sdp, *tail, buffers=buf)

        def ffn(idx, gate):
            return oracle.moe_ffn(d["x"], d["Wg"], d["Wu"], d["Wd"], idx, gate, d["Sg"], d["Su"], d["Sd"])
        return b, ffn
    quantize, layer, oq, offn = {
        "fp8": (L.lynx_quantize_weights_fp8, L.lynx_moe_layer_fp8, oracle.quantize_rows_e4m3, oracle.moe_ffn_q8),
        "fp4": (L.lynx_quantize_weights_fp4, L.lynx_moe_layer_fp4, oracle.quantize_mxfp4, oracle.moe_ffn_q4),
    }[fmt]
    q = quantize(*routed)
    sh = quantize(*shared) if shared else None
    b = layer(x, Wr, bias, q, cfg.F, cfg.k, alpha, beta, enable, sh, *tail, buffers=buf)
    (Qg, sg), (Qu, su), (Qd, sd) = (oq(d[n]) for n in ("Wg", "Wu", "Wd"))
    extra = ()
    if shared:
        (SQg, ssg), (SQu, ssu), (SQd, ssd) = (oq(d[n]) for n in ("Sg", "Su", "Sd"))
        extra = (SQg, SQu, SQd, ssg, ssu, ssd)

    def ffn(idx, gate):
        return offn(d["x"], Qg, Qu, Qd, sg, su, sd, idx, gate, *extra)
    return b, ffn


@pytest.mark.parametrize("i", range(N_CASES))
def test_layer_random_shape(L, i):
    fmt, cfg, T, alpha, beta, enable = draw_case(i)
    sigmoid = fmt == "bf16" and i % 2 == 0           # every other bf16 case sits behind a sigmoid-gated router
    print(f"random layer {i}: {fmt} T={T} H={cfg.H} F={cfg.F} N={cfg.N} k={cfg.k} shared={cfg.n_shared}x{cfg.F_shared} "
          f"alpha={alpha} beta={beta} enable={enable} router={'sigmoid' if sigmoid else 'softmax'}", flush=True)
    d = wl.make_layer(cfg, T)
    b, ffn = run_layer(L, fmt, cfg, d, alpha, beta, enable, sigmoid)
    torch.cuda.synchronize()
    from paper_2411_08982_amd.binding import WAIT_FLAG_WORD
    assert int(b.workspace.view(torch.int32)[WAIT_FLAG_WORD]) == 0, "a bounded wait inside the launch ran out"
    r = oracle.route(d["x"], d["Wr"], d["bias"], cfg.k)
    z = host(b.logits)
    assert np.all(np.abs(z - r["logits"]) <= LOGIT_TOL * np.maximum(1.0, np.abs(r["logits"])))
    tk = (oracle.topk_sigmoid if sigmoid else oracle.topk)(z, cfg.k)
    assert np.array_equal(host(b.topk_idx), tk["idx"])
    np.testing.assert_allclose(host(b.topk_gate), tk["gate"], rtol=GATE_TOL, atol=1e-7)
    a = (oracle.affinity_bin_sigmoid if sigmoid else oracle.affinity_bin)(z, tk["idx"], alpha, beta, enable)
    for key, got in (("new_idx", b.new_idx), ("cnt_before", b.cnt_before), ("cnt_after", b.cnt_after),
                     ("bin_hist", b.bin_hist), ("num_active", b.num_active)):
        assert np.array_equal(host(got), a[key]), key
    np.testing.assert_allclose(host(b.new_gate), a["new_gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(b.new_psum), a["new_psum"], rtol=GATE_TOL, atol=1e-7)
    assert int(host(b.status)[0]) == 0
    p = oracle.permute(a["new_idx"], cfg.N)
    for key, got in (("offsets", b.offsets), ("perm", b.perm), ("active", b.active), ("num_active", b.num_active_perm)):
        assert np.array_equal(host(got), p[key]), key
    y = host(b.y)
    assert np.all(np.isfinite(y))
    err = row_rel_err(y, ffn(a["new_idx"], a["new_gate"]))
    assert err.max() <= Y_TOL, f"max row error {err.max():.3e}"
    print(f"  invoked {a['num_active'].tolist()}, max row err {err.max():.3e}", flush=True)


# ---- the FFN alone: token distributions a router would not produce -------------------------------------------------

N_FFN_CASES = 24


def draw_ffn_case(i):
    """Weight format, shapes, and picks concentrated on `hot` experts (up to hundreds of tokens on one expert, most
    experts idle), some pairs invalid (an index outside [0, N): documented as skipped)."""
    rng = np.random.default_rng([8982, 2411, i])
    fmt = ("bf16", "fp8", "fp4")[i % 3]
    mult = {"bf16": 32, "fp8": 64, "fp4": 128}[fmt]
    T = int(rng.integers(130, 600)) if i % 4 == 0 else int(rng.integers(1, 150))
    N = int(rng.integers(1, 65))
    k = int(rng.integers(1, min(N, 8) + 1))
    hot = int(rng.integers(k, N + 1)) if rng.random() < 0.6 else N
    H = mult * int(rng.integers(1, 256 // mult + 1))
    F = mult * int(rng.integers(1, 256 // mult + 1))
    S = int(rng.choice([0, 0, 1, 2]))
    Fs = mult * int(rng.integers(1, 1280 // mult)) if S else 0
    idx = np.stack([rng.permutation(hot)[:k] for _ in range(T)]).astype(np.int32)
    gate = rng.random((T, k)).astype(np.float32) + 0.1
    gate /= gate.sum(1, keepdims=True)
    invalid = np.zeros((T, k), bool)
    if rng.random() < 0.4:
        invalid = rng.random((T, k)) < 0.1
        invalid[0, 0] = False
    bad = np.where(invalid, np.where(rng.random((T, k)) < 0.5, -1, N + 5), idx).astype(np.int32)
    return fmt, (T, H, F, N, k, S, Fs, hot), rng, idx, bad, gate, invalid


@pytest.mark.parametrize("i", range(N_FFN_CASES))
def test_ffn_random_tokens(L, i):
    fmt, (T, H, F, N, k, S, Fs, hot), rng, idx, bad, gate, invalid = draw_ffn_case(i)
    print(f"random ffn {i}: {fmt} T={T} H={H} F={F} N={N} k={k} hot={hot} shared={S}x{Fs} invalid={int(invalid.sum())}",
          flush=True)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    Wg, Wu, Wd = (wl.bf16_normal(rng, shape, 0.05) for shape in ((N, F, H), (N, F, H), (N, H, F)))
    Sg = Su = Sd = None
    if S:
        Sg, Su, Sd = (wl.bf16_normal(rng, shape, 0.05) for shape in ((S, Fs, H), (S, Fs, H), (S, H, Fs)))
    g_ref = np.where(invalid, 0.0, gate.astype(np.float64))      # a skipped pair = its gate at zero
    idx_d = dev(bad)
    p = L.lynx_permute(idx_d, N)
    ws = L.new_workspace(T, H, F, N, k, S, Fs, "cuda")
    ws.fill_(0xFF)
    y0 = torch.full((T, H), float("nan"), dtype=torch.float32, device="cuda")
    routed = [to_bf16_dev(W) for W in (Wg, Wu, Wd)]
    shared = [to_bf16_dev(W) for W in (Sg, Su, Sd)] if S else None
    if fmt == "bf16":
        y_ref = oracle.moe_ffn(x, Wg, Wu, Wd, idx, g_ref, Sg, Su, Sd)
        Wgu, Wdp = L.lynx_pack_weights(*routed)
        Sgu, Sdp = L.lynx_pack_weights(*shared) if S else (None, None)
        y = L.lynx_moe_ffn(to_bf16_dev(x), Wgu, Wdp, idx_d, dev(gate), p, N, F, Sgu, Sdp, S, Fs, workspace=ws, y=y0)
    else:
        quantize, ffn, oq, offn = {
            "fp8": (L.lynx_quantize_weights_fp8, L.lynx_moe_ffn_fp8, oracle.quantize_rows_e4m3, oracle.moe_ffn_q8),
            "fp4": (L.lynx_quantize_weights_fp4, L.lynx_moe_ffn_fp4, oracle.quantize_mxfp4, oracle.moe_ffn_q4),
        }[fmt]
        (Qg, sg), (Qu, su), (Qd, sd) = (oq(W) for W in (Wg, Wu, Wd))
        extra = ()
        if S:
            (SQg, ssg), (SQu, ssu), (SQd, ssd) = (oq(W) for W in (Sg, Su, Sd))
            extra = (SQg, SQu, SQd, ssg, ssu, ssd)
        y_ref = offn(x, Qg, Qu, Qd, sg, su, sd, idx, g_ref, *extra)
        y = ffn(to_bf16_dev(x), quantize(*routed), idx_d, dev(gate), p, N, F, quantize(*shared) if S else None, S, Fs,
                workspace=ws, y=y0)
    torch.cuda.synchronize()
    y = host(y)
    assert np.all(np.isfinite(y))
    err = row_rel_err(y, y_ref)
    assert err.max() <= Y_TOL, f"max row error {err.max():.3e}"


# ---- binning alone: top-k picks, picks in arbitrary order, the score-biased variant -------------------------------

@pytest.mark.parametrize("block", range(4))
def test_affinity_bin_random(L, block):
    for i in range(block * 40, block * 40 + 40):
        rng = np.random.default_rng([89, 82, i])
        T = int(rng.integers(1, 1025)) if rng.random() < 0.25 else int(rng.integers(1, 100))
        N = int(rng.integers(2, 257))
        k = int(rng.integers(1, min(N, 16) + 1))
        alpha = float(rng.choice([0.0, 0.25, 0.5, 1.0, 2.0, 3.0, 4.0, 8.0, 64.0, 1e6]))
        beta = int(rng.integers(1, 7))
        while float(T) ** beta >= 2.0 ** 62:
            beta -= 1
        gamma = float(rng.choice([0.0, 0.5, 1.0, 4.0, 1e6]))
        quantum = [None, 0.25, 1.0][int(rng.integers(0, 3))]
        mode = int(rng.integers(0, 3))    # 0: top-k picks, 1: k distinct experts in any order, 2: score-biased variant
        enable = int(rng.random() < 0.9)
        print(f"random bin {i}: T={T} N={N} k={k} alpha={alpha} beta={beta} gamma={gamma} quantum={quantum} mode={mode} "
              f"enable={enable}", flush=True)
        z = wl.make_logits(T, N, seed=7000 + i, zipf_s=float(rng.choice([0.0, 1.0, 1.5])),
                           tail_frac=float(rng.choice([0.0, 0.1])), quantum=quantum)
        if mode == 1:
            idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
        else:
            idx = oracle.topk(z, k)["idx"]
        if mode == 2:
            ref = oracle.affinity_bin_biased(z, idx, alpha, beta, gamma, enable)
            out = L.lynx_affinity_bin_biased(dev(z), dev(idx), alpha, beta, gamma, enable)
        else:
            ref = oracle.affinity_bin(z, idx, alpha, beta, enable)
            out = L.lynx_affinity_bin(dev(z), dev(idx), alpha, beta, enable)
        torch.cuda.synchronize()
        for key in ("new_idx", "cnt_before", "cnt_after", "bin_hist", "num_active"):
            assert np.array_equal(host(out[key]), ref[key]), key
        np.testing.assert_allclose(host(out["new_gate"]), ref["new_gate"], rtol=GATE_TOL, atol=1e-7)
        p = L.lynx_permute(out["new_idx"], N)
        torch.cuda.synchronize()
        pr = oracle.permute(ref["new_idx"], N)
        for key in ("offsets", "perm", "active", "num_active"):
            assert np.array_equal(host(p[key]), pr[key]), key


def grouped_case(L, i):
    """One random group-limited case: sizes, groups, gate function, bin parameters and logit structure all drawn."""
    rng = np.random.default_rng([71, 82, i])
    G = int(rng.choice([1, 2, 3, 4, 8, 16, 64])) if rng.random() < 0.7 else int(rng.integers(1, 65))
    gs = int(rng.integers(1, 256 // G + 1))
    N = G * gs
    tg = int(rng.integers(1, G + 1))
    k = int(rng.integers(1, min(tg * gs, 16) + 1))
    T = int(rng.integers(1, 1025)) if rng.random() < 0.2 else int(rng.integers(1, 100))
    alpha = float(rng.choice([0.0, 0.25, 0.5, 1.0, 2.0, 4.0, 8.0, 1e6]))
    beta = int(rng.integers(1, 7))
    while float(T) ** beta >= 2.0 ** 62:
        beta -= 1
    quantum = [None, 0.25, 1.0][int(rng.integers(0, 3))]
    gate_fn = int(rng.integers(0, 2))
    enable = int(rng.random() < 0.9)
    print(f"random grouped {i}: T={T} N={N} k={k} G={G} tg={tg} alpha={alpha} beta={beta} quantum={quantum} "
          f"gate_fn={gate_fn} enable={enable}", flush=True)
    z = wl.make_logits(T, N, seed=9000 + i, zipf_s=float(rng.choice([0.0, 1.0, 1.5])),
                       tail_frac=float(rng.choice([0.0, 0.1])), quantum=quantum)
    I, F = torch.int32, torch.float32

    def poisoned(shape, dtype):
        t = torch.empty(shape, dtype=dtype, device="cuda")
        t.view(torch.uint8).fill_(0xFF)
        return t
    o = dict(idx=poisoned((T, k), I), gate=poisoned((T, k), F), psum=poisoned((T,), F), new_idx=poisoned((T, k), I),
             new_gate=poisoned((T, k), F), new_psum=poisoned((T,), F), cnt_before=poisoned((N,), I), cnt_after=poisoned((N,), I),
             bin_hist=poisoned((N, beta), I), num_active=poisoned((2,), I))
    ws = torch.full((65536,), 0xFF, dtype=torch.uint8, device="cuda")
    out = L.lynx_affinity_bin_grouped(dev(z), k, G, tg, alpha, beta, gate_fn, enable, ws, o)
    torch.cuda.synchronize()
    tk = oracle.topk_grouped(z, k, G, tg, gate_fn)
    assert np.array_equal(host(out["idx"]), tk["idx"])
    np.testing.assert_allclose(host(out["gate"]), tk["gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(out["psum"]), tk["third"], rtol=GATE_TOL, atol=1e-7)
    ref = oracle.affinity_bin_grouped(z, tk["idx"], G, tg, alpha, beta, enable, gate_fn)
    for key in ("new_idx", "cnt_before", "cnt_after", "bin_hist", "num_active"):
        assert np.array_equal(host(out[key]), ref[key]), key
    np.testing.assert_allclose(host(out["new_gate"]), ref["new_gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(out["new_psum"]), ref["new_psum"], rtol=GATE_TOL, atol=1e-7)


@pytest.mark.parametrize("block", range(3))
def test_affinity_bin_grouped_random(L, block):
    for i in range(block * 40, block * 40 + 40):
        grouped_case(L, i)
