#!/usr/bin/env python3
"""Benchmark of the Lynx MoE decode layer on one MI355X.

A step = one pass of the whole hot path (lynx_moe_layer = route -> affinity_bin -> permute ->
moe_ffn) over one decode batch of a synthetic Mixtral-8x7B-shaped layer (hidden 4096, FFN 14336,
8 experts, top-2, bf16 weights), inputs already resident in HBM.  Prints ONE JSON line: the headline
us/batch, the HBM roofline of the dominant kernel (gate/up weight stream) measured with HIP events
around that kernel inside the timed steps, a sweep over the configuration's batch sizes with the
remap off / on, and the CPU oracle timed on the host cores as a reported baseline.

Successive steps cycle over several resident copies of the layer's expert weights (distinct buffers, same
router and tokens), as the layers of a model would: a step that re-read the very buffers of the step before
would find a small configuration's experts in the 256 MB last-level cache and report a rate above HBM's.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config mixtral] [--tokens 8] [--preset aggressive]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="mixtral", choices=["tiny", "mixtral", "qwen15moe", "dsv2lite", "qwen3", "dsv3"])
    ap.add_argument("--router", default="softmax", choices=["softmax", "sigmoid"],
                    help="gate function of the router; sigmoid: the layer runs through lynx_moe_layer_sigmoid (the "
                         "quantised-weight variants, the score-biased variant and the CPU baseline, which are "
                         "softmax-gated, are then left out)")
    ap.add_argument("--groups", default="", metavar="G,TG",
                    help="group-limited router: G groups of consecutive experts, a token uses the experts of its TG "
                         "best groups; the layer runs through lynx_moe_layer_grouped (with --router's gate function; "
                         "the same variants are left out as for --router sigmoid)")
    ap.add_argument("--tokens", type=int, default=8)
    ap.add_argument("--preset", default="aggressive", choices=["moderate", "aggressive", "off"])
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fp8", action="store_true", help="skip the FP8-weight variant of the same workload")
    ap.add_argument("--sweep-iters", type=int, default=10)
    ap.add_argument("--layers", type=int, default=0,
                    help="resident copies of the expert weights that successive steps cycle over (0 = enough for 4 GiB)")
    ap.add_argument("--biased-gamma", type=float, default=4.0,
                    help="bias strength of the score-biased selection variant in the sweep (0 = leave it out)")
    ap.add_argument("--layer-policy", default="",
                    help="with --stack: a layer-adaptive remapping table such as '0-3:off,4-43:aggressive,44-47:moderate' "
                         "(layers not named keep --preset); timed beside the uniform settings")
    ap.add_argument("--stack", type=int, default=0,
                    help="time a chained stack of this many layers (own router and weights each, x <- bf16(x + y) between "
                         "them) as a whole, eagerly and as one HIP graph, instead of the single-layer benchmark")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="before the steps, run a plain 1 GiB read + 1 GiB write elementwise kernel three times: under "
                         "rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings give the counters' scale")
    return ap.parse_args()


def expert_bytes(cfg, n_routed):
    """Algorithmic expert-weight bytes of one layer pass: gate/up part and down part."""
    gu = n_routed * 2 * cfg.H * cfg.F * 2 + cfg.n_shared * 2 * cfg.H * cfg.F_shared * 2
    dn = n_routed * cfg.H * cfg.F * 2 + cfg.n_shared * cfg.H * cfg.F_shared * 2
    return gu, dn


class Layer:
    """Device-resident inputs and packed weights of one synthetic layer, plus per-T buffers."""

    def __init__(self, cfg, T_gen, keep_row_major=False, n_layers=1):
        import torch

        import paper_2411_08982_amd as L
        import workloads as wl
        self.L, self.cfg, self.torch, self.wl = L, cfg, torch, wl
        self.weights = []          # per resident layer: packed routed gate/up, down, shared gate/up, down
        self.calls = 0
        self.sigmoid_router = False
        self.groups = None   # (n_group, topk_group) for a group-limited router
        for l in range(n_layers):
            d = wl.make_layer_device(cfg, T_gen if l == 0 else 1, "cuda", layer=l)
            Wgu, Wdp = L.lynx_pack_weights(d["Wg"], d["Wu"], d["Wd"])
            Sgu = Sdp = None
            if cfg.n_shared:
                Sgu, Sdp = L.lynx_pack_weights(d["Sg"], d["Su"], d["Sd"])
            torch.cuda.synchronize()
            self.weights.append((Wgu, Wdp, Sgu, Sdp))
            if l == 0:             # router, tokens and the oracle's row-major weights are those of layer 0
                self.Wr, self.bias = d["Wr"], d["bias"]
                self.row_major = {k: d[k] for k in ("Wg", "Wu", "Wd", "Sg", "Su", "Sd")} if keep_row_major else None
                self.x = {T_gen: d["x"]}
            del d
        self.buf = {}

    def tokens(self, T):
        if T not in self.x:
            import numpy as np
            xb = self.wl.make_tokens(self.cfg, T, self.Wr.cpu().numpy(), self.bias.cpu().numpy())
            self.x[T] = self.torch.from_numpy(xb.view(np.int16)).cuda().view(self.torch.bfloat16)
        return self.x[T]

    def buffers(self, T, beta):
        key = (T, beta)
        if key not in self.buf:
            c = self.cfg
            self.buf[key] = self.L.LayerBuffers(T, c.H, c.F, c.N, c.k, beta, c.n_shared, c.F_shared)
        return self.buf[key]

    def step(self, T, alpha, beta, enable, events=None, layer=None, sigmoid=None):
        """One decode step (the whole hot path) through the fused C-ABI entry point, on the current stream.
        Successive calls take the resident layers' expert weights in turn."""
        c = self.cfg
        if layer is None:
            layer = self.calls % len(self.weights)
            self.calls += 1
        Wgu, Wdp, Sgu, Sdp = self.weights[layer]
        if sigmoid is None:
            sigmoid = self.sigmoid_router
        if self.groups is not None:
            return self.L.lynx_moe_layer_grouped(self.tokens(T), self.Wr, self.bias, Wgu, Wdp, c.F, c.k, self.groups[0],
                                                 self.groups[1], alpha, beta, int(bool(sigmoid)), enable, Sgu, Sdp, c.n_shared,
                                                 c.F_shared, buffers=self.buffers(T, beta), stage_events=events)
        entry = self.L.lynx_moe_layer_sigmoid if sigmoid else self.L.lynx_moe_layer
        return entry(self.tokens(T), self.Wr, self.bias, Wgu, Wdp, c.F, c.k, alpha, beta, enable, Sgu, Sdp, c.n_shared,
                     c.F_shared, buffers=self.buffers(T, beta), stage_events=events)


def preset_args(wl, preset):
    if preset == "off":
        return 2.0, 2, 0
    a, b = wl.PRESETS[preset]
    return a, b, 1


def layer_policy(spec, n_layers, default_preset):
    """'0-3:off,4-43:aggressive,44:moderate' -> one preset name per layer (paper Sec. 3.2.1: sensitivity to the
    remap differs between layers, so the policy may; the paper gives no rule, the table is the caller's)."""
    names = [default_preset] * n_layers
    for part in filter(None, (q.strip() for q in spec.split(","))):
        rng, _, preset = part.partition(":")
        if preset not in ("off", "moderate", "aggressive"):
            raise ValueError(f"--layer-policy: unknown preset in '{part}'")
        lo, _, hi = rng.partition("-")
        lo, hi = int(lo), int(hi) if hi else int(lo)
        if not 0 <= lo <= hi < n_layers:
            raise ValueError(f"--layer-policy: layers '{rng}' outside 0..{n_layers - 1}")
        names[lo:hi + 1] = [preset] * (hi - lo + 1)
    return names


def run_stack(args, cfg, wl, torch):
    """A stack of layers on one stream with a true dependency from each layer to the next, timed as a whole."""
    import numpy as np

    import paper_2411_08982_amd as L
    T, n_layers = args.tokens, args.stack
    alpha, beta, enable = preset_args(wl, args.preset)
    table = layer_policy(args.layer_policy, n_layers, args.preset) if args.layer_policy else None
    betas = sorted({beta} | {preset_args(wl, n)[1] for n in (table or []) if n != "off"})
    layers, bufs = [], []
    x0 = None
    for l in range(n_layers):
        d = wl.make_layer_device(cfg, T if l == 0 else 1, "cuda", layer=l)
        Wgu, Wdp = L.lynx_pack_weights(d["Wg"], d["Wu"], d["Wd"])
        Sgu = Sdp = None
        if cfg.n_shared:
            Sgu, Sdp = L.lynx_pack_weights(d["Sg"], d["Su"], d["Sd"])
        torch.cuda.synchronize()
        layers.append((d["Wr"], d["bias"], Wgu, Wdp, Sgu, Sdp))
        bufs.append({bt: L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, bt, cfg.n_shared, cfg.F_shared) for bt in betas})
        if l == 0:
            x0 = d["x"]
        del d
    xs = [x0] + [torch.empty_like(x0) for _ in range(n_layers)]

    used = [None] * n_layers   # the buffers the last chain wrote, per layer

    def chain(en):
        """en: 0 / 1 = remap off / the preset in every layer; "table" = the per-layer table."""
        for l, (Wr, bias, Wgu, Wdp, Sgu, Sdp) in enumerate(layers):
            a_l, b_l, e_l = (alpha, beta, en)
            if en == "table":   # a layer that is switched off keeps the default preset's bins (they are not used)
                a_l, b_l, e_l = preset_args(wl, table[l]) if table[l] != "off" else (alpha, beta, 0)
            b = L.lynx_moe_layer(xs[l], Wr, bias, Wgu, Wdp, cfg.F, cfg.k, a_l, b_l, e_l, Sgu, Sdp, cfg.n_shared,
                                 cfg.F_shared, buffers=bufs[l][b_l])
            used[l] = b
            L.lynx_residual_add(xs[l], b.y, out=xs[l + 1])

    def timed(fn, reps):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        return us[len(us) // 2], us[0]

    res = {}
    for name, en in (("off", 0), (args.preset, enable)) + ((("layer_policy", "table"),) if table else ()):
        if name in res:
            continue
        for _ in range(max(1, args.warmup)):
            chain(en)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            chain(en)
        torch.cuda.synchronize()
        wall_us = (time.perf_counter() - t0) * 1e6 / args.steps
        eager_med, eager_min = timed(lambda: chain(en), args.steps)
        na = np.array([b.num_active.cpu().numpy() for b in used])
        routed = float(na[:, 1].sum()) * 3 * cfg.H * cfg.F * 2 + n_layers * cfg.n_shared * 3 * cfg.H * cfg.F_shared * 2
        # the same chain as one HIP graph (the library enqueues kernels only: no allocation, memset or host read)
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            chain(en)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            chain(en)
        for _ in range(2):
            g.replay()
        graph_med, graph_min = timed(g.replay, args.steps)
        res[name] = {"us_wall_eager": round(wall_us, 1), "us_eager_median": round(eager_med, 1), "us_eager_min": round(eager_min, 1),
                     "us_graph_median": round(graph_med, 1), "us_graph_min": round(graph_min, 1),
                     "invoked_before_mean": round(float(na[:, 0].mean()), 2), "invoked_after_mean": round(float(na[:, 1].mean()), 2),
                     "expert_weight_GBps_graph": round(routed / (graph_med * 1e-6) / 1e9, 1)}
        del g
    best = res[args.preset]
    out = {"metric": f"MoE-stack decode us/batch ({n_layers} chained layers)", "value": best["us_graph_median"], "unit": "us/batch",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(best["us_graph_median"] * 1e-3, 5),
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{n_layers} chained {cfg.name}-shaped MoE layers (own router and expert weights each): hidden "
                                  f"{cfg.H}, FFN {cfg.F}, {cfg.N} experts top-{cfg.k}, {cfg.n_shared} shared, bf16 weights, {T} "
                                  f"decode tokens, remap {args.preset}; x <- bf16(x + y) between layers",
                      "tokens": T, "alpha": alpha, "beta": beta, "layers": n_layers},
           "us_per_layer": round(best["us_graph_median"] / n_layers, 2),
           "tokens_per_s": round(T / (best["us_graph_median"] * 1e-6), 1),
           "stack": res, "layer_policy": args.layer_policy or None,
           "roofline": {"bound": "hbm", "kernel": "whole stack (all kernels of all layers)", "achieved": best["expert_weight_GBps_graph"],
                        "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(best["expert_weight_GBps_graph"] / HBM_PEAK_GBPS, 4),
                        "traffic": None}}
    print(json.dumps(out))


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (no collectives, no sharding); --gpus {args.gpus} is not "
              "supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch

    import workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.config]
    if args.stack > 0:
        run_stack(args, cfg, wl, torch)
        return
    T = args.tokens
    if args.router == "sigmoid" or args.groups:
        args.no_fp8, args.no_cpu_baseline, args.biased_gamma = True, True, 0.0
    alpha, beta, enable = preset_args(wl, args.preset)
    routed_bytes = 3 * cfg.N * cfg.H * cfg.F * 2
    n_layers = args.layers if args.layers > 0 else max(1, min(8, -(-(4 << 30) // routed_bytes)))
    layer = Layer(cfg, T, keep_row_major=not args.no_cpu_baseline, n_layers=n_layers)
    layer.sigmoid_router = args.router == "sigmoid"
    if args.groups:
        layer.groups = tuple(int(v) for v in args.groups.split(","))

    if args.pmc_calibration:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")   # 1 GiB
        c = torch.empty_like(a)
        for _ in range(3):
            torch.mul(a, 1.0, out=c)                                    # plain copy kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, c
    K, W = args.steps, args.warmup
    for _ in range(W):
        layer.step(T, alpha, beta, enable)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        b = layer.step(T, alpha, beta, enable)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / K
    # Second pass over the same K steps with HIP events recorded (by the library, on the stream the kernels
    # run on) at the FFN stage boundaries.  It is kept apart from the timed region above because every event
    # costs a few microseconds of idle GPU between two kernels.
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
    for evs in events:           # a first record creates the underlying hipEvent_t handles
        for e in evs:
            e.record()
    torch.cuda.synchronize()
    for i in range(K):
        events[i][4].record()    # start of the step: routing = from here to the event before the gate/up kernel
        layer.step(T, alpha, beta, enable, events[i][:4])
    torch.cuda.synchronize()
    rt_ms = sum(e[4].elapsed_time(e[0]) for e in events) / K
    ffn_ms = sum(e[0].elapsed_time(e[1]) for e in events) / K      # the one kernel that streams all expert weights
    cb_ms = sum(e[2].elapsed_time(e[3]) for e in events) / K
    n_before, n_after = (int(v) for v in b.num_active.cpu().tolist())
    gu_bytes, dn_bytes = expert_bytes(cfg, n_after)
    ffn_bytes = gu_bytes + dn_bytes
    ffn_gbps = ffn_bytes / (ffn_ms * 1e-3) / 1e9
    n_launch = layer.L.lynx_moe_ffn_launches(T, cfg.F)

    # The practical ceiling beside it: a plain read-only streaming kernel over 2 GiB, same load width and hint.
    probe = torch.zeros(1 << 29, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    plain = {}
    for name, nt in (("non_temporal", True), ("default", False)):
        for _ in range(2):
            layer.L.lynx_read_probe(probe, sink, nt)
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        for _ in range(5):
            layer.L.lynx_read_probe(probe, sink, nt)
        p1.record()
        torch.cuda.synchronize()
        plain[name] = round(5 * probe.numel() * 4 / (p0.elapsed_time(p1) * 1e-3) / 1e9, 1)
    del probe

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(f"{args.config}_T{T}_{args.preset}")
        except Exception:
            traffic = None

    out = {
        "metric": "MoE-layer decode us/batch",
        "value": round(ms_per_step * 1e3, 2),
        "unit": "us/batch",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}-shaped MoE layer: hidden {cfg.H}, FFN {cfg.F}, {cfg.N} experts top-{cfg.k}, "
                               f"{cfg.n_shared} shared, bf16 weights, {T} decode tokens, remap {args.preset}"
                               + (", sigmoid-gated router" if args.router == "sigmoid" else "")
                               + (f", group-limited router ({layer.groups[1]} of {layer.groups[0]} groups)" if layer.groups else ""),
                   "tokens": T, "alpha": alpha, "beta": beta, "remap": bool(enable), "resident_layers": n_layers},
        "tokens_per_s": round(T / (ms_per_step * 1e-3), 1),
        "experts_invoked": {"before": n_before, "after": n_after},
        "expert_weight_hbm_GBps": round(ffn_gbps, 1),
        # from the pass with events (each event adds a few us of idle GPU, so the stages sum to more than `value`)
        "stage_us": {"routing_a1_to_a7": round(rt_ms * 1e3, 2), "expert_ffn_a8": round(ffn_ms * 1e3, 2),
                     "combine_a9": round(cb_ms * 1e3, 2)},
        "roofline": {"bound": "hbm", "kernel": "ffn_kernel (gate/up and down weight streams of all invoked experts)",
                     "achieved": round(ffn_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(ffn_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
                     "launches_per_step": n_launch, "bytes_per_launch": ffn_bytes // n_launch,
                     "avg_launch_us": round(ffn_ms * 1e3 / n_launch, 2),
                     "plain_read_GBps": plain},
    }

    if not args.no_sweep:
        sweep = []
        for Ts in cfg.batches:
            for preset in ("off", "moderate", "aggressive"):
                a_, b_, en_ = preset_args(wl, preset)
                for _ in range(3):
                    layer.step(Ts, a_, b_, en_)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for _ in range(args.sweep_iters):
                    bb = layer.step(Ts, a_, b_, en_)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / args.sweep_iters
                nb, na = (int(v) for v in bb.num_active.cpu().tolist())
                g, d_ = expert_bytes(cfg, na)
                sweep.append({"tokens": Ts, "remap": preset, "us": round(us, 1), "invoked_before": nb, "invoked_after": na,
                              "expert_weight_GBps": round((g + d_) / (us * 1e-6) / 1e9, 1),
                              "hbm_frac": round((g + d_) / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)})
        out["sweep"] = sweep
        if args.biased_gamma > 0:
            # the score-biased selection variant (logit + gamma * normalised batch score), through the separate calls
            # lynx_route -> lynx_affinity_bin_biased -> lynx_permute -> lynx_moe_ffn (more launches than the fused layer)
            L = layer.L
            a_, b_ = wl.PRESETS["moderate"]
            var = []
            for Ts in cfg.batches:
                x = layer.tokens(Ts)
                r = L.lynx_route(x, layer.Wr, layer.bias, cfg.k)
                ab = L.lynx_affinity_bin_biased(r["logits"], r["idx"], a_, b_, args.biased_gamma, 1)
                pm = L.lynx_permute(ab["new_idx"], cfg.N)
                ws = L.new_workspace(Ts, cfg.H, cfg.F, cfg.N, cfg.k, cfg.n_shared, cfg.F_shared)
                y = torch.empty((Ts, cfg.H), dtype=torch.float32, device="cuda")

                def step_biased(i):
                    Wgu, Wdp, Sgu, Sdp = layer.weights[i % len(layer.weights)]
                    L.lynx_route(x, layer.Wr, layer.bias, cfg.k, out=r)
                    L.lynx_affinity_bin_biased(r["logits"], r["idx"], a_, b_, args.biased_gamma, 1, workspace=ws, out=ab)
                    L.lynx_permute(ab["new_idx"], cfg.N, out=pm)
                    L.lynx_moe_ffn(x, Wgu, Wdp, ab["new_idx"], ab["new_gate"], pm, cfg.N, cfg.F, Sgu, Sdp, cfg.n_shared,
                                   cfg.F_shared, workspace=ws, y=y)
                for i in range(3):
                    step_biased(i)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for i in range(args.sweep_iters):
                    step_biased(i)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / args.sweep_iters
                nb, na = (int(v) for v in ab["num_active"].cpu().tolist())
                var.append({"tokens": Ts, "gamma": args.biased_gamma, "alpha": a_, "beta": b_, "us": round(us, 1),
                            "invoked_before": nb, "invoked_after": na})
            out["sweep_score_biased_variant"] = var

    if not args.no_sweep and not args.groups:
        # The same workload behind a sigmoid-gated router (gates = selected sigmoid scores over their sum; bins,
        # scores and the remap are the softmax path's): a widening, reported beside the metric above.
        for _ in range(3):
            layer.step(T, alpha, beta, enable, sigmoid=True)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.sweep_iters):
            bb = layer.step(T, alpha, beta, enable, sigmoid=True)
        e1.record()
        torch.cuda.synchronize()
        nb, na = (int(v) for v in bb.num_active.cpu().tolist())
        out["sigmoid_router"] = {"us_per_batch": round(e0.elapsed_time(e1) * 1e3 / args.sweep_iters, 2),
                                 "invoked_before": nb, "invoked_after": na}

    if not args.no_fp8:
        # The same workload with the expert weights in FP8 E4M3 (row scales) and in MXFP4 (block scales), both
        # weight-only: widenings beyond the bf16 metric above, reported beside it and never as `value`.
        L = layer.L
        import workloads as wl2

        def quantised_variant(quantize, run_layer, bytes_num, bytes_den):
            qs = []
            for l in range(n_layers):
                d = wl2.make_layer_device(cfg, 1, "cuda", layer=l)
                q = quantize(d["Wg"], d["Wu"], d["Wd"])
                sh = quantize(d["Sg"], d["Su"], d["Sd"]) if cfg.n_shared else None
                torch.cuda.synchronize()
                qs.append((q, sh))
                del d
            buf = layer.buffers(T, beta)

            def step_q(i, ev=None):
                q, sh = qs[i % n_layers]
                return run_layer(layer.tokens(T), layer.Wr, layer.bias, q, cfg.F, cfg.k, alpha, beta, enable, sh,
                                 cfg.n_shared, cfg.F_shared, buffers=buf, stage_events=ev)
            for i in range(W):
                step_q(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(K):
                step_q(i)
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) * 1e6 / K
            for i in range(K):
                step_q(i, events[i][:4])
            torch.cuda.synchronize()
            ffn_ms = sum(e[0].elapsed_time(e[1]) for e in events) / K
            nbytes = ffn_bytes * bytes_num // bytes_den
            return {"us_per_batch": round(us, 2), "expert_ffn_us": round(ffn_ms * 1e3, 2), "weight_bytes": nbytes,
                    "expert_weight_GBps": round(nbytes / (ffn_ms * 1e-3) / 1e9, 1),
                    "hbm_frac": round(nbytes / (ffn_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                    "speedup_vs_bf16": round(ms_per_step * 1e3 / us, 3)}

        out["fp8_weights"] = quantised_variant(L.lynx_quantize_weights_fp8, L.lynx_moe_layer_fp8, 1, 2)
        out["fp8_weights"]["format"] = "OCP FP8 E4M3 codes + one fp32 scale per weight row; activations bf16"
        if cfg.H % 128 == 0 and cfg.F % 128 == 0 and (cfg.n_shared == 0 or cfg.F_shared % 128 == 0):
            # 4 bits per weight + 8 bits per block of 32 = 17/64 of the bf16 bytes
            out["mxfp4_weights"] = quantised_variant(L.lynx_quantize_weights_fp4, L.lynx_moe_layer_fp4, 17, 64)
            out["mxfp4_weights"]["format"] = ("OCP MXFP4: FP4 E2M1 codes + one E8M0 scale per block of 32 columns; "
                                              "activations bf16")

    if not args.no_cpu_baseline:
        import numpy as np

        import oracle
        bits = lambda t: None if t is None else t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        rm = {k_: bits(v) for k_, v in layer.row_major.items()}
        xh = bits(layer.tokens(T))
        Wr, bias = layer.Wr.cpu().numpy(), layer.bias.cpu().numpy()
        times = []
        for _ in range(5):
            t0 = time.perf_counter()
            o = oracle.moe_layer(xh, Wr, bias, rm["Wg"], rm["Wu"], rm["Wd"], cfg.k, alpha, beta, enable, rm["Sg"], rm["Su"],
                                 rm["Sd"])
            times.append(time.perf_counter() - t0)
        cpu_s = sorted(times)[len(times) // 2]
        out["cpu_baseline"] = {"value": round(cpu_s * 1e6, 1), "unit": "us/batch", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"one full layer pass of the same workload ({T} tokens, all invoked experts), "
                                         "median of 5 repetitions, plain C fp64 oracle with an OpenMP split over weight rows",
                               "experts_invoked": [int(v) for v in o["bin"]["num_active"]]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
