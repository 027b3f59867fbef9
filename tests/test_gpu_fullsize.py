"""GPU parity at the full sizes of the benchmark configurations, through the same fused entry point
(`lynx_moe_layer`) and launch configuration that bench.py times.

Routing outputs are small, so they are compared in full: logits against the oracle's own router, and
every integer output (indices, counts, histogram, offsets, permutation, invoked-expert list) bit-exact
against the oracle fed with the GPU's fp32 logits.  The layer output is compared on sampled tokens,
which the oracle computes one by one from the weights of just the experts those tokens use; properties
that hold at any size (finite output, gates summing to 1, invoked experts not rising) are checked on
the whole batch.  Inputs are synthetic (workloads.py); expert weights are drawn on the device.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import bf16_bits, dev, host, row_rel_err, tile_covering_tokens, to_bf16_dev

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


class DeviceLayer:
    def __init__(self, L, cfg, T):
        d = wl.make_layer_device(cfg, T, "cuda")
        self.cfg, self.d = cfg, d
        self.Wgu, self.Wdp = L.lynx_pack_weights(d["Wg"], d["Wu"], d["Wd"])
        self.Sgu = self.Sdp = None
        if cfg.n_shared:
            self.Sgu, self.Sdp = L.lynx_pack_weights(d["Sg"], d["Su"], d["Sd"])
        torch.cuda.synchronize()

    def tokens(self, T):
        Wr, bias = host(self.d["Wr"]), host(self.d["bias"])
        return wl.make_tokens(self.cfg, T, Wr, bias)


_layers = {}


def _layer(L, name):
    if name not in _layers:
        _layers.clear()          # one large layer resident at a time
        torch.cuda.empty_cache()
        cfg = wl.CONFIGS[name]
        _layers[name] = DeviceLayer(L, cfg, cfg.batches[0])
    return _layers[name]


def _check_layer(L, lay, T, alpha, beta, enable, n_sample=5, seed=0, sigmoid=False, groups=None):
    cfg, d = lay.cfg, lay.d
    xb = lay.tokens(T)
    x = to_bf16_dev(xb)
    if groups:
        b = L.lynx_moe_layer_grouped(x, d["Wr"], d["bias"], lay.Wgu, lay.Wdp, cfg.F, cfg.k, groups[0], groups[1], alpha, beta,
                                     int(sigmoid), enable, lay.Sgu, lay.Sdp, cfg.n_shared, cfg.F_shared)
    else:
        entry = L.lynx_moe_layer_sigmoid if sigmoid else L.lynx_moe_layer
        b = entry(x, d["Wr"], d["bias"], lay.Wgu, lay.Wdp, cfg.F, cfg.k, alpha, beta, enable, lay.Sgu, lay.Sdp,
                  cfg.n_shared, cfg.F_shared)
    torch.cuda.synchronize()
    Wr, bias = host(d["Wr"]), host(d["bias"])
    # routing, whole batch
    r = oracle.route(xb, Wr, bias, cfg.k)
    z = host(b.logits)
    assert np.all(np.abs(z - r["logits"]) <= LOGIT_TOL * np.maximum(1.0, np.abs(r["logits"])))
    if groups:
        tk = oracle.topk_grouped(z, cfg.k, groups[0], groups[1], int(sigmoid))
        third = tk["third"]
    else:
        tk = (oracle.topk_sigmoid if sigmoid else oracle.topk)(z, cfg.k)
        third = tk["ssum" if sigmoid else "psum"]
    assert np.array_equal(host(b.topk_idx), tk["idx"])
    np.testing.assert_allclose(host(b.topk_gate), tk["gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(b.topk_psum), third, rtol=GATE_TOL, atol=1e-7)
    if groups:
        a = oracle.affinity_bin_grouped(z, tk["idx"], groups[0], groups[1], alpha, beta, enable, int(sigmoid))
        assert np.take_along_axis(oracle.group_allowed(z, groups[0], groups[1]), a["new_idx"], 1).all()
    else:
        a = (oracle.affinity_bin_sigmoid if sigmoid else oracle.affinity_bin)(z, tk["idx"], alpha, beta, enable)
    for key, got in (("new_idx", b.new_idx), ("cnt_before", b.cnt_before), ("cnt_after", b.cnt_after),
                     ("bin_hist", b.bin_hist), ("num_active", b.num_active)):
        assert np.array_equal(host(got), a[key]), key
    g = host(b.new_gate)
    np.testing.assert_allclose(g, a["new_gate"], rtol=GATE_TOL, atol=1e-7)
    np.testing.assert_allclose(host(b.new_psum), a["new_psum"], rtol=GATE_TOL, atol=1e-7)
    assert int(host(b.status)[0]) == 0
    p = oracle.permute(a["new_idx"], cfg.N)
    for key, got in (("offsets", b.offsets), ("perm", b.perm), ("active", b.active), ("num_active", b.num_active_perm)):
        assert np.array_equal(host(got), p[key]), key
    # properties on the whole batch
    from paper_2411_08982_amd.binding import WAIT_FLAG_WORD
    assert int(b.workspace.view(torch.int32)[WAIT_FLAG_WORD]) == 0, "a workgroup gave up waiting for its expert's gate/up results"
    y = host(b.y)
    assert np.all(np.isfinite(y))
    np.testing.assert_allclose(g.sum(1), 1.0, rtol=1e-5)
    assert a["num_active"][1] <= a["num_active"][0]
    # sampled tokens against the oracle, with only the experts those tokens use copied to the host: the first and the
    # last token, some at random, and tokens chosen by where they sit in their expert's sorted range (see below)
    rng = np.random.default_rng(seed)
    toks = sorted(set([0, T - 1] + rng.choice(T, size=min(T, n_sample), replace=False).tolist()
                      + tile_covering_tokens(p["offsets"], p["perm"], cfg.k)))
    sel = a["new_idx"][toks]
    used = np.unique(sel)
    remap = {int(e): i for i, e in enumerate(used)}
    sel_c = np.vectorize(remap.get)(sel).astype(np.int32)
    ue = torch.from_numpy(used.astype(np.int64)).cuda()
    Wg, Wu, Wd = (bf16_bits(d[k_].index_select(0, ue)) for k_ in ("Wg", "Wu", "Wd"))
    Sg = Su = Sd = None
    if cfg.n_shared:
        Sg, Su, Sd = (bf16_bits(d[k_]) for k_ in ("Sg", "Su", "Sd"))
    y_ref = oracle.moe_ffn(xb[toks], Wg, Wu, Wd, sel_c, a["new_gate"][toks], Sg, Su, Sd)
    err = row_rel_err(y[toks], y_ref)
    assert err.max() <= Y_TOL, f"max row error {err.max():.3e} on tokens {toks}"
    return a["num_active"], err.max()


FULL = [("mixtral", 8, "aggressive"), ("mixtral", 1, "aggressive"), ("mixtral", 32, "moderate"), ("mixtral", 128, "off"),
        ("qwen15moe", 8, "aggressive"), ("qwen15moe", 64, "moderate"), ("qwen15moe", 256, "aggressive"),
        ("dsv2lite", 16, "aggressive"), ("dsv2lite", 128, "moderate"), ("dsv2lite", 256, "aggressive"),
        ("qwen3", 32, "aggressive"), ("qwen3", 128, "moderate"), ("qwen3", 512, "aggressive")]


@pytest.mark.parametrize("name,T,preset", FULL)
def test_full_size_layer(L, name, T, preset):
    print(f"full-size layer {name} T={T} remap={preset}", flush=True)
    lay = _layer(L, name)
    if preset == "off":
        alpha, beta, enable = 2.0, 2, 0
    else:
        (alpha, beta), enable = wl.PRESETS[preset], 1
    na, err = _check_layer(L, lay, T, alpha, beta, enable)
    print(f"  invoked {na.tolist()}, max sampled row err {err:.3e}", flush=True)


@pytest.mark.parametrize("T,preset,groups", [(8, "aggressive", None), (64, "moderate", None), (32, "moderate", (8, 4))])
def test_full_size_layer_sigmoid_router(L, T, preset, groups):
    """A DeepSeek-V3-shaped layer (256 experts of 88 MB, top-8, one shared expert) behind the sigmoid-gated router,
    without and with the group limit (4 of 8 groups): routing of the whole batch against the oracle, sampled tokens'
    outputs against the oracle's FFN."""
    print(f"full-size layer dsv3 T={T} remap={preset}, sigmoid-gated router, groups={groups}", flush=True)
    lay = _layer(L, "dsv3")
    alpha, beta = wl.PRESETS[preset]
    na, err = _check_layer(L, lay, T, alpha, beta, 1, n_sample=2, sigmoid=True, groups=groups)
    print(f"  invoked {na.tolist()}, max sampled row err {err:.3e}", flush=True)
    _layers.clear()              # 45 GB of row-major and packed weights: release them before the next test
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,T", [("dsv2lite", 128), ("qwen3", 256), ("qwen15moe", 64)])
def test_single_launch_reads_no_stale_intermediates(L, name, T):
    """With more than 16 tokens both projections run in one launch and the down workgroups read the intermediate
    vectors that gate/up workgroups of the same launch wrote.  Alternating two batches on ONE workspace (which
    then always holds the other batch's intermediates) must give, bit for bit, what each batch gives on a
    freshly zeroed workspace: a read of anything but this launch's values would differ between the two."""
    print(f"stale-read check {name} T={T}", flush=True)
    lay = _layer(L, name)
    cfg, d = lay.cfg, lay.d
    assert L.lynx_moe_ffn_launches(T, cfg.F) == 1
    xa = to_bf16_dev(lay.tokens(T))
    xb = to_bf16_dev(wl.make_tokens(cfg, T, host(d["Wr"]), host(d["bias"]), seed=1234))
    (alpha, beta) = wl.PRESETS["moderate"]

    def run(x, buffers):
        b = L.lynx_moe_layer(x, d["Wr"], d["bias"], lay.Wgu, lay.Wdp, cfg.F, cfg.k, alpha, beta, 1, lay.Sgu, lay.Sdp,
                             cfg.n_shared, cfg.F_shared, buffers=buffers)
        torch.cuda.synchronize()
        return host(b.y).copy()

    fresh = []
    for x in (xa, xb):
        buf = L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, beta, cfg.n_shared, cfg.F_shared)
        buf.workspace.zero_()
        fresh.append(run(x, buf))
    assert not np.array_equal(fresh[0], fresh[1])
    shared_buf = L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, beta, cfg.n_shared, cfg.F_shared)
    for rep in range(6):
        y = run((xa, xb)[rep % 2], shared_buf)
        assert np.array_equal(y, fresh[rep % 2]), f"repetition {rep}"


def test_release_large_layers():
    _layers.clear()
    torch.cuda.empty_cache()


# ---- limits and ragged sizes through the fused entry point, small H / F so that the oracle does the whole batch ----

EDGE = [
    # T,    N,   k,  H,  F, S, Fs
    (1024, 256, 16, 64, 64, 0, 0),     # every documented maximum at once
    (17, 20, 3, 96, 160, 1, 64),       # just past the single-workgroup routing path
    (16, 20, 3, 96, 160, 0, 0),        # the largest batch of the single-workgroup routing path
    (65, 9, 9, 64, 96, 2, 32),         # k = N: nothing to remap; 65 tokens on every expert (two staged passes)
    (33, 128, 8, 32, 32, 0, 0),        # smallest H and F
    (2, 5, 1, 64, 64, 0, 0),           # k = 1
]


@pytest.mark.parametrize("T,N,k,H,F,S,Fs", EDGE)
def test_edge_sizes(L, T, N, k, H, F, S, Fs):
    print(f"edge layer T={T} N={N} k={k} H={H} F={F} shared={S}x{Fs}", flush=True)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], name="edge", H=H, F=F, N=N, k=k, n_shared=S, F_shared=Fs, seed=T + N)
    d = wl.make_layer(cfg, T)
    x, Wr, bias = to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"])
    Wgu, Wdp = L.lynx_pack_weights(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
    Sgu = Sdp = None
    if S:
        Sgu, Sdp = L.lynx_pack_weights(to_bf16_dev(d["Sg"]), to_bf16_dev(d["Su"]), to_bf16_dev(d["Sd"]))
    for alpha, beta in ((4.0, 1), (1.0, 3)):
        b = L.lynx_moe_layer(x, Wr, bias, Wgu, Wdp, F, k, alpha, beta, 1, Sgu, Sdp, S, Fs)
        torch.cuda.synchronize()
        from paper_2411_08982_amd.binding import WAIT_FLAG_WORD
        assert int(b.workspace.view(torch.int32)[WAIT_FLAG_WORD]) == 0
        z = host(b.logits)
        r = oracle.route(d["x"], d["Wr"], d["bias"], k)
        assert np.all(np.abs(z - r["logits"]) <= LOGIT_TOL * np.maximum(1.0, np.abs(r["logits"])))
        tk = oracle.topk(z, k)
        a = oracle.affinity_bin(z, tk["idx"], alpha, beta, 1)
        p = oracle.permute(a["new_idx"], N)
        for key, got in (("new_idx", b.new_idx), ("cnt_after", b.cnt_after), ("bin_hist", b.bin_hist),
                         ("num_active", b.num_active)):
            assert np.array_equal(host(got), a[key]), key
        for key, got in (("offsets", b.offsets), ("perm", b.perm), ("active", b.active)):
            assert np.array_equal(host(got), p[key]), key
        y_ref = oracle.moe_ffn(d["x"], d["Wg"], d["Wu"], d["Wd"], a["new_idx"], a["new_gate"], d["Sg"], d["Su"], d["Sd"])
        err = row_rel_err(host(b.y), y_ref)
        assert err.max() <= Y_TOL, f"max row error {err.max():.3e}"


QUANTISED = [("dsv2lite", 16, "fp8"), ("dsv2lite", 16, "fp4"), ("qwen3", 128, "fp8"), ("qwen3", 128, "fp4"),
             ("qwen15moe", 64, "fp4"), ("mixtral", 8, "fp4")]


@pytest.mark.parametrize("name,T,fmt", QUANTISED)
def test_full_size_layer_quantised_weights(L, name, T, fmt):
    """The FP8 and MXFP4 weight paths at benchmark sizes: routing as above; the layer output on sampled tokens
    against the oracle, which quantises the weights of just the experts those tokens use by itself."""
    print(f"full-size layer {name} T={T} weights={fmt}", flush=True)
    lay = _layer(L, name)
    cfg, d = lay.cfg, lay.d
    (alpha, beta), enable = wl.PRESETS["aggressive"], 1
    quant = L.lynx_quantize_weights_fp8 if fmt == "fp8" else L.lynx_quantize_weights_fp4
    run = L.lynx_moe_layer_fp8 if fmt == "fp8" else L.lynx_moe_layer_fp4
    q = quant(d["Wg"], d["Wu"], d["Wd"])
    sh = quant(d["Sg"], d["Su"], d["Sd"]) if cfg.n_shared else None
    xb = lay.tokens(T)
    b = run(to_bf16_dev(xb), d["Wr"], d["bias"], q, cfg.F, cfg.k, alpha, beta, enable, sh, cfg.n_shared, cfg.F_shared)
    torch.cuda.synchronize()
    from paper_2411_08982_amd.binding import WAIT_FLAG_WORD
    assert int(b.workspace.view(torch.int32)[WAIT_FLAG_WORD]) == 0
    z = host(b.logits)
    a = oracle.affinity_bin(z, oracle.topk(z, cfg.k)["idx"], alpha, beta, enable)
    assert np.array_equal(host(b.new_idx), a["new_idx"])
    y = host(b.y)
    assert np.all(np.isfinite(y))
    toks = sorted({0, T - 1, T // 2})                     # few tokens: the oracle quantises every expert they use
    sel = a["new_idx"][toks]
    used = np.unique(sel)
    remap = {int(e): i for i, e in enumerate(used)}
    sel_c = np.vectorize(remap.get)(sel).astype(np.int32)
    ue = torch.from_numpy(used.astype(np.int64)).cuda()
    W = [bf16_bits(d[k_].index_select(0, ue)) for k_ in ("Wg", "Wu", "Wd")]
    S = [bf16_bits(d[k_]) for k_ in ("Sg", "Su", "Sd")] if cfg.n_shared else []
    oq = oracle.quantize_rows_e4m3 if fmt == "fp8" else oracle.quantize_mxfp4
    ffn = oracle.moe_ffn_q8 if fmt == "fp8" else oracle.moe_ffn_q4
    (Qg, sg), (Qu, su), (Qd, sd) = (oq(w) for w in W)
    shared = ()
    if S:
        (SQg, ssg), (SQu, ssu), (SQd, ssd) = (oq(w) for w in S)
        shared = (SQg, SQu, SQd, ssg, ssu, ssd)
    y_ref = ffn(xb[toks], Qg, Qu, Qd, sg, su, sd, sel_c, a["new_gate"][toks], *shared)
    err = row_rel_err(y[toks], y_ref)
    print(f"  invoked {a['num_active'].tolist()}, experts quantised by the oracle {len(used)}, max sampled row err {err.max():.3e}",
          flush=True)
    assert err.max() <= Y_TOL
