"""GPU tests of a chained stack of MoE layers, x_{l+1} = bf16(x_l + y_l), as the benchmark times it.

Parity is checked per layer with the GPU's own layer input fed to the oracle (a comparison along the chain
would turn legitimate bf16 differences into different routing further down).  The stack is also captured
into a HIP graph: every replay, with eager work and synchronisations in between, must reproduce the eager
result bit for bit (the kernels use no floating-point atomics, so the result does not depend on timing).
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


@pytest.fixture(scope="module")
def L():
    import paper_2411_08982_amd as lib
    lib.lib()
    assert torch.cuda.is_available()
    return lib


class Stack:
    """`n_layers` small layers with their own routers and expert weights, resident on the GPU."""

    def __init__(self, L, cfg, T, n_layers, alpha, beta, policy=None, weights="bf16"):
        self.L, self.cfg, self.T, self.weights = L, cfg, T, weights
        # per-layer (alpha, beta, enable): the remapping policy may differ from layer to layer (paper Sec. 3.2.1,
        # layer sensitivity); one setting for all layers by default
        self.policy = list(policy) if policy else [(alpha, beta, 1)] * n_layers
        self.host_layers = [wl.make_layer(cfg, T, layer=l) for l in range(n_layers)]
        self.dev_layers = []
        quant = {"fp8": L.lynx_quantize_weights_fp8, "fp4": L.lynx_quantize_weights_fp4}.get(weights)
        for d in self.host_layers:
            if quant:      # quantised experts: (routed, shared) weight objects in the slots of the packed tensors
                q = quant(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
                sh = quant(to_bf16_dev(d["Sg"]), to_bf16_dev(d["Su"]), to_bf16_dev(d["Sd"])) if cfg.n_shared else None
                self.dev_layers.append((dev(d["Wr"]), dev(d["bias"]), q, None, sh, None))
                continue
            Wgu, Wdp = L.lynx_pack_weights(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
            Sgu = Sdp = None
            if cfg.n_shared:
                Sgu, Sdp = L.lynx_pack_weights(to_bf16_dev(d["Sg"]), to_bf16_dev(d["Su"]), to_bf16_dev(d["Sd"]))
            self.dev_layers.append((dev(d["Wr"]), dev(d["bias"]), Wgu, Wdp, Sgu, Sdp))
        self.x0 = to_bf16_dev(self.host_layers[0]["x"])
        # every layer has its own outputs (kept for the checks) and its own input buffer
        self.buf = [L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, self.policy[l][1], cfg.n_shared, cfg.F_shared)
                    for l in range(n_layers)]
        self.x = [self.x0] + [torch.empty_like(self.x0) for _ in range(n_layers)]
        torch.cuda.synchronize()

    def run(self):
        """Enqueues the whole chain on the current stream; allocates nothing."""
        c = self.cfg
        for l, (Wr, bias, Wgu, Wdp, Sgu, Sdp) in enumerate(self.dev_layers):
            alpha, beta, enable = self.policy[l]
            if self.weights != "bf16":
                layer = self.L.lynx_moe_layer_fp8 if self.weights == "fp8" else self.L.lynx_moe_layer_fp4
                b = layer(self.x[l], Wr, bias, Wgu, c.F, c.k, alpha, beta, enable, Sgu, c.n_shared, c.F_shared,
                          buffers=self.buf[l])
            else:
                b = self.L.lynx_moe_layer(self.x[l], Wr, bias, Wgu, Wdp, c.F, c.k, alpha, beta, enable, Sgu, Sdp,
                                          c.n_shared, c.F_shared, buffers=self.buf[l])
            self.L.lynx_residual_add(self.x[l], b.y, out=self.x[l + 1])

    def snapshot(self):
        torch.cuda.synchronize()
        out = [bf16_bits(x) for x in self.x]
        for b in self.buf:
            out += [host(b.y), host(b.new_idx), host(b.perm), host(b.num_active)]
        return out


def test_residual_add_is_one_rounded_fp32_addition(L):
    rng = np.random.default_rng(5)
    for shape in ((3, 64), (1, 2), (37, 4096)):
        xb = wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32) * 3)
        y = (rng.standard_normal(shape) * np.exp(rng.uniform(-8, 3, shape))).astype(np.float32)
        want = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(xb) + y)          # numpy fp32 add, then round to nearest even
        x = to_bf16_dev(xb)
        got = L.lynx_residual_add(x, dev(y))
        torch.cuda.synchronize()
        assert np.array_equal(bf16_bits(got), want)
        L.lynx_residual_add(x, dev(y), out=x)                            # in place
        torch.cuda.synchronize()
        assert np.array_equal(bf16_bits(x), want)


# one setting for every layer, and a layer-adaptive table: off, moderate, aggressive, and a wide three-bin setting
POLICIES = {"uniform": None, "per-layer": [(2.0, 2, 0), (2.0, 2, 1), (4.0, 1, 1), (1.0, 3, 1)]}


@pytest.mark.parametrize("policy", list(POLICIES))
@pytest.mark.parametrize("T,shared", [(8, 0), (24, 1)])
def test_stack_parity_layer_by_layer(L, T, shared, policy):
    print(f"stack of 4 layers, T={T}, shared={shared}, policy={policy}", flush=True)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], name="stack", H=256, F=384, N=24, k=3, n_shared=shared,
                              F_shared=128 if shared else 0, seed=11)
    st = Stack(L, cfg, T, 4, 2.0, 2, POLICIES[policy])
    st.run()
    torch.cuda.synchronize()
    remapped = 0
    for l, d in enumerate(st.host_layers):
        alpha, beta, enable = st.policy[l]
        xb = bf16_bits(st.x[l])                     # the GPU's own input of this layer
        b = st.buf[l]
        z = host(b.logits)
        r = oracle.route(xb, d["Wr"], d["bias"], cfg.k)
        assert np.all(np.abs(z - r["logits"]) <= 1e-5 * np.maximum(1.0, np.abs(r["logits"])))
        tk = oracle.topk(z, cfg.k)
        a = oracle.affinity_bin(z, tk["idx"], alpha, beta, enable)
        assert np.array_equal(host(b.new_idx), a["new_idx"])
        assert np.array_equal(host(b.num_active), a["num_active"])
        if not enable:
            assert np.array_equal(a["new_idx"], tk["idx"])
        p = oracle.permute(a["new_idx"], cfg.N)
        assert np.array_equal(host(b.perm), p["perm"]) and np.array_equal(host(b.offsets), p["offsets"])
        y_ref = oracle.moe_ffn(xb, d["Wg"], d["Wu"], d["Wd"], a["new_idx"], a["new_gate"], d.get("Sg"), d.get("Su"),
                               d.get("Sd"))
        y = host(b.y)
        assert row_rel_err(y, y_ref).max() <= Y_TOL
        assert np.array_equal(bf16_bits(st.x[l + 1]), wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(xb) + y))
        remapped += int(a["num_active"][0] - a["num_active"][1])
    print(f"  experts saved over the stack: {remapped}", flush=True)


@pytest.mark.parametrize("weights", ["bf16", "fp8", "fp4"])
@pytest.mark.parametrize("T", [8, 40])
def test_graph_replays_reproduce_the_eager_stack(L, T, weights):
    print(f"graph capture of a 3-layer stack, T={T}, expert weights {weights}", flush=True)
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], name="graph", H=256, F=384, N=24, k=3, n_shared=1, F_shared=128, seed=12)
    st = Stack(L, cfg, T, 3, 4.0, 1, weights=weights)
    st.run()
    eager = st.snapshot()
    other = to_bf16_dev(wl.make_tokens(cfg, T, st.host_layers[0]["Wr"], st.host_layers[0]["bias"], seed=99))
    first = st.x0.clone()
    st.x0.copy_(other)
    st.run()
    eager_other = st.snapshot()
    assert not np.array_equal(eager[-4], eager_other[-4])       # the second input really gives another result

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st.run()                                                # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        st.run()
    for rep, (inp, want) in enumerate([(first, eager), (other, eager_other), (first, eager), (first, eager)]):
        for x in st.x[1:]:
            x.zero_()                                           # eager work between the replays
        for b in st.buf:
            b.y.fill_(float("nan"))
        st.x0.copy_(inp)
        torch.cuda.synchronize()
        g.replay()
        got = st.snapshot()
        for i, (u, v) in enumerate(zip(got, want)):
            assert np.array_equal(u, v), f"replay {rep}: array {i} differs from the eager run"


@pytest.mark.timeout(400)
@pytest.mark.parametrize("T,preset", [(128, "aggressive")])
def test_full_qwen3_stack_layers_0_24_47(L, T, preset):
    """The 48-layer Qwen3-shaped stack that bench.py times (58 GB of packed expert weights resident), run once as a
    chain; layers 0, 24 and 47 are checked like a single full-size layer: routing outputs in full, the layer output
    on sampled tokens, each with the GPU's own input of that layer fed to the oracle."""
    cfg = wl.CONFIGS["qwen3"]
    check = (0, 24, 47)
    alpha, beta = wl.PRESETS[preset]
    n_layers = 48
    print(f"qwen3-shaped stack, {n_layers} layers, T={T}, preset {preset}", flush=True)
    layers, kept = [], {}
    for l in range(n_layers):
        d = wl.make_layer_device(cfg, 1, "cuda", layer=l)
        Wgu, Wdp = L.lynx_pack_weights(d["Wg"], d["Wu"], d["Wd"])
        torch.cuda.synchronize()
        layers.append((d["Wr"], d["bias"], Wgu, Wdp))
        if l in check:
            kept[l] = d
        del d
        if l % 12 == 11:
            print(f"  {l + 1} layers resident", flush=True)
    Wr0, b0 = host(layers[0][0]), host(layers[0][1])
    xs = [to_bf16_dev(wl.make_tokens(cfg, T, Wr0, b0))]
    bufs = {}
    for l, (Wr, bias, Wgu, Wdp) in enumerate(layers):
        buf = L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, beta, 0, 0) if l in check else bufs.setdefault("scratch", L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, beta, 0, 0))
        b = L.lynx_moe_layer(xs[l], Wr, bias, Wgu, Wdp, cfg.F, cfg.k, alpha, beta, 1, None, None, 0, 0, buffers=buf)
        if l in check:
            bufs[l] = b
        xs.append(L.lynx_residual_add(xs[l], b.y))
    torch.cuda.synchronize()
    for l in check:
        d, b = kept[l], bufs[l]
        xb = bf16_bits(xs[l])
        Wr, bias = host(d["Wr"]), host(d["bias"])
        z = host(b.logits)
        r = oracle.route(xb, Wr, bias, cfg.k)
        # deeper layers see the un-normalised chain's larger token norms: the bound scales with the logit
        assert np.all(np.abs(z - r["logits"]) <= 1e-5 * np.maximum(1.0, np.abs(r["logits"]))), f"layer {l}: logits"
        tk = oracle.topk(z, cfg.k)
        assert np.array_equal(host(b.topk_idx), tk["idx"]), f"layer {l}: top-k"
        a = oracle.affinity_bin(z, tk["idx"], alpha, beta, 1)
        for key, got in (("new_idx", b.new_idx), ("cnt_before", b.cnt_before), ("cnt_after", b.cnt_after),
                         ("bin_hist", b.bin_hist), ("num_active", b.num_active)):
            assert np.array_equal(host(got), a[key]), f"layer {l}: {key}"
        np.testing.assert_allclose(host(b.new_gate), a["new_gate"], rtol=1e-5, atol=1e-7)
        p = oracle.permute(a["new_idx"], cfg.N)
        for key, got in (("offsets", b.offsets), ("perm", b.perm), ("active", b.active), ("num_active", b.num_active_perm)):
            assert np.array_equal(host(got), p[key]), f"layer {l}: {key}"
        assert int(host(b.status)[0]) == 0
        y = host(b.y)
        assert np.all(np.isfinite(y))
        toks = sorted(set([0, T - 1] + tile_covering_tokens(p["offsets"], p["perm"], cfg.k)[:6]))
        sel = a["new_idx"][toks]
        used = np.unique(sel)
        remap = {int(e): i for i, e in enumerate(used)}
        sel_c = np.vectorize(remap.get)(sel).astype(np.int32)
        ue = torch.from_numpy(used.astype(np.int64)).cuda()
        Wg, Wu, Wd = (bf16_bits(d[k_].index_select(0, ue)) for k_ in ("Wg", "Wu", "Wd"))
        y_ref = oracle.moe_ffn(xb[toks], Wg, Wu, Wd, sel_c, a["new_gate"][toks])
        err = row_rel_err(y[toks], y_ref).max()
        assert err <= Y_TOL, f"layer {l}: max row error {err:.3e} on tokens {toks}"
        assert np.array_equal(bf16_bits(xs[l + 1]), wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(xb) + y)), f"layer {l}: residual"
        print(f"  layer {l}: experts {a['num_active'].tolist()}, max row error {err:.2e} on tokens {toks}", flush=True)
    del layers, kept, bufs, xs
    torch.cuda.empty_cache()
