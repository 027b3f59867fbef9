#!/usr/bin/env python3
"""Benchmark of the Lynx MoE decode step on one MI355X.

A step = one pass of the whole hot path (lynx_moe_layer = route -> affinity_bin -> permute -> moe_ffn, once per layer)
over one decode batch, inputs already resident in HBM.  Prints ONE JSON line.

Without --config (what the driver runs) the line covers every benchmark configuration:
  * headline (`value`, `config`, `roofline`, `cpu_baseline`): the largest configuration that fits one GPU, the chained
    stack of 48 Qwen3-30B-A3B-shaped MoE layers (58 GB of bf16 expert weights resident, own router and weights per
    layer, x <- bf16(x + y) between layers), 512 decode tokens, remap aggressive, replayed as one HIP graph;
    `stack` holds the same for 32 / 128 / 256 / 512 tokens with the remap off / moderate / aggressive;
  * `configs`: the Mixtral-8x7B-, Qwen1.5-MoE- and DeepSeek-V2-Lite-shaped single layers, every batch size of the
    configuration, remap off / moderate / aggressive: us per layer, tokens/s, experts invoked before / after, the
    weight-streaming kernel's and the whole layer's fraction of the HBM peak, the routing side's time and share, and what
    the remap costs (mean ratio of the selected softmax mass after / before, share of tokens that keep their top-1);
  * `mixtral_T8`: the Mixtral-shaped layer at 8 tokens in detail (stage times, plain-read ceiling, FP8 / MXFP4 weights).
With --config NAME it measures that one configuration (single layer, or --stack L layers): what the rocprofv3 summaries
under profiles/ were taken from.

Successive steps of a single-layer measurement cycle over several resident copies of the layer's expert weights
(distinct buffers, same router and tokens), as the layers of a model would: a step that re-read the very buffers of the
step before would find a small configuration's experts in the 256 MB last-level cache and report a rate above HBM's.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config NAME --tokens T --preset P | --stack L]
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
PRESET_NAMES = ("off", "moderate", "aggressive")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="", choices=["", "tiny", "mixtral", "qwen15moe", "dsv2lite", "qwen3", "dsv3"],
                    help="measure this one configuration instead of the full report")
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
    ap.add_argument("--no-fp8", action="store_true", help="skip the FP8 / MXFP4 weight variants of the same workload")
    ap.add_argument("--sweep-iters", type=int, default=10)
    ap.add_argument("--layers", type=int, default=0,
                    help="resident copies of the expert weights that successive steps cycle over (0 = enough for 4 GiB)")
    ap.add_argument("--biased-gamma", type=float, default=4.0,
                    help="bias strength of the score-biased selection variant in the sweep (0 = leave it out)")
    ap.add_argument("--layer-policy", default="",
                    help="with --stack: a layer-adaptive remapping table such as '0-3:off,4-43:aggressive,44-47:moderate' "
                         "(layers not named keep --preset); timed beside the uniform settings")
    ap.add_argument("--stack", type=int, default=0,
                    help="with --config: time a chained stack of this many layers (own router and weights each, "
                         "x <- bf16(x + y) between them) as a whole, eagerly and as one HIP graph")
    ap.add_argument("--stack-layers", type=int, default=48, help="layers of the stack in the full report")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="before the steps, run a plain 1 GiB read + 1 GiB write elementwise kernel three times: under "
                         "rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings give the counters' scale")
    ap.add_argument("--down-item-cap", type=int, default=0, help="tuning: down-projection work items the plan aims at")
    ap.add_argument("--down-item-units", type=int, default=0, help="tuning: most 64-row units per down work item")
    ap.add_argument("--down-k-waves", type=int, default=0, help="tuning: K slices of a down workgroup's waves")
    return ap.parse_args()


def expert_bytes(cfg, n_routed):
    """Algorithmic expert-weight bytes of one layer pass: gate/up part and down part."""
    gu = n_routed * 2 * cfg.H * cfg.F * 2 + cfg.n_shared * 2 * cfg.H * cfg.F_shared * 2
    dn = n_routed * cfg.H * cfg.F * 2 + cfg.n_shared * cfg.H * cfg.F_shared * 2
    return gu, dn


def traffic_of(key):
    """HBM bytes per launch of the weight-streaming kernel measured with rocprofv3 --pmc for this workload key, if a
    measurement is filed under profiles/ (else None: nothing is assumed)."""
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(tpath):
        return None
    try:
        return json.load(open(tpath)).get(key)
    except Exception:
        return None


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


def remap_cost(b):
    """What the remap gave up, from the layer's own outputs: the mean over the tokens of (softmax mass of the new
    selection) / (mass of the router's top-k), and the share of tokens whose top-ranked expert is still selected.
    Also checks the call's status word (a failed wait inside the expert kernel turns y into NaNs)."""
    import torch
    ratio = float((b.new_psum / b.topk_psum).mean().item())
    kept = float((b.new_idx == b.topk_idx[:, :1]).any(dim=1).float().mean().item())
    assert int(b.status.item()) == 0, "a bounded wait inside the expert kernel ran out: the outputs are NaN"
    assert bool(torch.isfinite(b.y).all().item())
    return round(ratio, 4), round(kept, 4)


def new_events(torch, n, per=5):
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(per)] for _ in range(n)]
    for e5 in evs:                # a first record creates the underlying hipEvent_t handles
        for e in e5:
            e.record()
    torch.cuda.synchronize()
    return evs


def measure_layer(layer, T, preset, iters, warmup, torch, wl, events=None):
    """One (configuration, batch size, remap setting): `iters` steps timed as a whole (no events inside), then the same
    steps again with the library recording HIP events at the FFN stage boundaries on the stream the kernels run on."""
    cfg = layer.cfg
    a_, b_, en_ = preset_args(wl, preset)
    for _ in range(warmup):
        layer.step(T, a_, b_, en_)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        bb = layer.step(T, a_, b_, en_)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / iters
    events = events if events is not None and len(events) >= iters else new_events(torch, iters)
    for i in range(iters):
        events[i][4].record()
        layer.step(T, a_, b_, en_, events[i][:4])
    torch.cuda.synchronize()
    rt = sum(e[4].elapsed_time(e[0]) for e in events[:iters]) * 1e3 / iters
    ffn = sum(e[0].elapsed_time(e[1]) for e in events[:iters]) * 1e3 / iters
    cb = sum(e[2].elapsed_time(e[3]) for e in events[:iters]) * 1e3 / iters
    nb, na = (int(v) for v in bb.num_active.cpu().tolist())
    g, d_ = expert_bytes(cfg, na)
    ratio, kept = remap_cost(bb)
    side = rt + cb      # everything that is not the weight stream: a1-a7 and the combine
    return {"config": cfg.name, "tokens": T, "remap": preset, "us": round(us, 1), "tokens_per_s": round(T / (us * 1e-6), 1),
            "invoked_before": nb, "invoked_after": na, "expert_weight_bytes": g + d_,
            "expert_weight_GBps": round((g + d_) / (us * 1e-6) / 1e9, 1),
            "layer_hbm_frac": round((g + d_) / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
            "ffn_kernel_us": round(ffn, 1), "ffn_kernel_hbm_frac": round((g + d_) / (ffn * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
            "routing_us": round(rt, 1), "combine_us": round(cb, 1),
            # from the pass with events (each adds a few us of idle GPU): share of routing + combine in the staged sum
            "routing_share": round(side / (side + ffn), 4),
            "psum_ratio": ratio, "top1_kept": kept}


def layer_policy(spec, n_layers, default_preset):
    """'0-3:off,4-43:aggressive,44:moderate' -> one preset name per layer (paper Sec. 3.2.1: sensitivity to the
    remap differs between layers, so the policy may; the paper gives no rule, the table is the caller's)."""
    names = [default_preset] * n_layers
    for part in filter(None, (q.strip() for q in spec.split(","))):
        rng, _, preset = part.partition(":")
        if preset not in PRESET_NAMES:
            raise ValueError(f"--layer-policy: unknown preset in '{part}'")
        lo, _, hi = rng.partition("-")
        lo, hi = int(lo), int(hi) if hi else int(lo)
        if not 0 <= lo <= hi < n_layers:
            raise ValueError(f"--layer-policy: layers '{rng}' outside 0..{n_layers - 1}")
        names[lo:hi + 1] = [preset] * (hi - lo + 1)
    return names


class Stack:
    """n_layers chained layers (own router and expert weights each) resident on the GPU."""

    def __init__(self, cfg, n_layers, torch, wl, keep_row_major_layers=0):
        import paper_2411_08982_amd as L
        self.cfg, self.n, self.torch, self.wl, self.L = cfg, n_layers, torch, wl, L
        self.layers, self.row_major = [], []
        for l in range(n_layers):
            d = wl.make_layer_device(cfg, 1, "cuda", layer=l)
            Wgu, Wdp = L.lynx_pack_weights(d["Wg"], d["Wu"], d["Wd"])
            Sgu = Sdp = None
            if cfg.n_shared:
                Sgu, Sdp = L.lynx_pack_weights(d["Sg"], d["Su"], d["Sd"])
            torch.cuda.synchronize()
            self.layers.append((d["Wr"], d["bias"], Wgu, Wdp, Sgu, Sdp))
            if l < keep_row_major_layers:     # for the CPU baseline: the oracle reads row-major weights
                self.row_major.append({k: (None if d[k] is None else d[k].cpu()) for k in ("Wg", "Wu", "Wd", "Sg", "Su", "Sd")})
            del d
        self.T = None

    def prepare(self, T, betas):
        import numpy as np
        cfg, torch, L = self.cfg, self.torch, self.L
        self.T = T
        Wr0, b0 = self.layers[0][0], self.layers[0][1]
        xb = self.wl.make_tokens(cfg, T, Wr0.cpu().numpy(), b0.cpu().numpy())
        x0 = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
        self.xs = [x0] + [torch.empty_like(x0) for _ in range(self.n)]
        self.bufs = [{bt: L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, bt, cfg.n_shared, cfg.F_shared) for bt in betas}
                     for _ in range(self.n)]
        self.used = [None] * self.n

    def chain(self, per_layer, events=None):
        """per_layer: (alpha, beta, enable) for every layer.  events: per layer five events; [4] is recorded before the
        layer, [0..3] by the library at the FFN stage boundaries."""
        cfg, L = self.cfg, self.L
        for l, (Wr, bias, Wgu, Wdp, Sgu, Sdp) in enumerate(self.layers):
            a_l, b_l, e_l = per_layer[l]
            if events is not None:
                events[l][4].record()
            b = L.lynx_moe_layer(self.xs[l], Wr, bias, Wgu, Wdp, cfg.F, cfg.k, a_l, b_l, e_l, Sgu, Sdp, cfg.n_shared,
                                 cfg.F_shared, buffers=self.bufs[l][b_l], stage_events=None if events is None else events[l][:4])
            self.used[l] = b
            L.lynx_residual_add(self.xs[l], b.y, out=self.xs[l + 1])

    def measure(self, per_layer, steps, warmup):
        import numpy as np
        torch, cfg, n = self.torch, self.cfg, self.n

        def timed(fn, reps):
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, b in evs:
                a.record()
                fn()
                b.record()
            torch.cuda.synchronize()
            us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
            return us[len(us) // 2], us[0]

        for _ in range(max(1, warmup)):
            self.chain(per_layer)
        torch.cuda.synchronize()
        eager_med, eager_min = timed(lambda: self.chain(per_layer), steps)
        na = np.array([b.num_active.cpu().numpy() for b in self.used])
        ratios = [remap_cost(b) for b in self.used]
        routed = float(na[:, 1].sum()) * 3 * cfg.H * cfg.F * 2 + n * cfg.n_shared * 3 * cfg.H * cfg.F_shared * 2
        # the same chain as one HIP graph (the library enqueues kernels only: no allocation, memset or host read)
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.chain(per_layer)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            self.chain(per_layer)
        for _ in range(max(1, warmup)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):          # the K timed steps: graph replays back to back, bracketed by synchronisations
            g.replay()
        torch.cuda.synchronize()
        graph_wall = (time.perf_counter() - t0) * 1e6 / steps
        graph_med, graph_min = timed(g.replay, steps)
        del g
        # eager passes with the library's stage events in every layer: the weight-streaming kernel's own time
        evs = new_events(torch, n)
        reps = max(2, min(steps, 4))
        ffn_us = side_us = 0.0
        for _ in range(reps):
            self.chain(per_layer, evs)
            torch.cuda.synchronize()
            ffn_us += sum(e[0].elapsed_time(e[1]) for e in evs) * 1e3 / reps
            side_us += sum(e[4].elapsed_time(e[0]) + e[2].elapsed_time(e[3]) for e in evs) * 1e3 / reps
        return {"us_eager_median": round(eager_med, 1), "us_eager_min": round(eager_min, 1),
                "us_graph_wall": round(graph_wall, 1), "us_graph_median": round(graph_med, 1), "us_graph_min": round(graph_min, 1),
                "invoked_before_mean": round(float(na[:, 0].mean()), 2), "invoked_after_mean": round(float(na[:, 1].mean()), 2),
                "expert_weight_bytes": int(routed),
                "expert_weight_GBps_graph": round(routed / (graph_wall * 1e-6) / 1e9, 1),
                "stack_hbm_frac": round(routed / (graph_wall * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                "us_per_layer": round(graph_wall / n, 2), "tokens_per_s": round(self.T / (graph_wall * 1e-6), 1),
                "ffn_kernel_us": round(ffn_us, 1),
                "ffn_kernel_hbm_frac": round(routed / (ffn_us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                "routing_and_combine_us": round(side_us, 1), "routing_share": round(side_us / (side_us + ffn_us), 4),
                "psum_ratio": round(float(np.mean([q[0] for q in ratios])), 4),
                "top1_kept": round(float(np.mean([q[1] for q in ratios])), 4)}


def cpu_baseline_stack(stack, T, preset, torch, wl, n_cpu_layers):
    """The oracle (plain C, fp64, as it stands) on the first n_cpu_layers layers of the stack, chained like the GPU's
    (x <- bf16(x + y)), timed on the host cores; the whole stack is that times n_layers / n_cpu_layers."""
    import numpy as np

    import oracle
    cfg = stack.cfg
    alpha, beta, enable = preset_args(wl, preset)
    bits = lambda t: None if t is None else t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    Wr0, b0 = stack.layers[0][0].cpu().numpy(), stack.layers[0][1].cpu().numpy()
    x = wl.make_tokens(cfg, T, Wr0, b0)
    host_layers = []
    for l in range(n_cpu_layers):
        rm = {k_: bits(v) for k_, v in stack.row_major[l].items()}
        host_layers.append((stack.layers[l][0].cpu().numpy(), stack.layers[l][1].cpu().numpy(), rm))
    t0 = time.perf_counter()
    invoked = []
    for Wr, bias, rm in host_layers:
        o = oracle.moe_layer(x, Wr, bias, rm["Wg"], rm["Wu"], rm["Wd"], cfg.k, alpha, beta, enable, rm["Sg"], rm["Su"], rm["Sd"])
        invoked.append(int(o["bin"]["num_active"][1]))
        x = wl.f32_to_bf16_bits((wl.bf16_bits_to_f32(x).astype(np.float64) + o["y"]).astype(np.float32))
    cpu_s = time.perf_counter() - t0
    scale = stack.n / n_cpu_layers
    return {"value": round(cpu_s * scale * 1e6, 1), "unit": "us/batch", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"the first {n_cpu_layers} of the {stack.n} layers of the same stack ({T} tokens, remap {preset}, chained), one "
                      f"repetition, {cpu_s:.2f} s measured, times {scale:g} for the whole stack; plain C fp64 oracle with an "
                      "OpenMP split over weight rows",
            "measured_s": round(cpu_s, 3), "extrapolation_factor": scale, "experts_invoked_per_layer": invoked}


def stack_line(args, cfg, wl, torch, n_layers, T_list, presets, headline, table=None, cpu_layers=0):
    """Builds the stack, measures every (T, preset) and returns the fields of the bench line that come from it."""
    stack = Stack(cfg, n_layers, torch, wl, keep_row_major_layers=cpu_layers)
    betas = sorted({preset_args(wl, p)[1] for p in PRESET_NAMES})
    res = {}
    for T in T_list:
        stack.prepare(T, betas)
        for preset in presets:
            per_layer = [preset_args(wl, preset)] * n_layers
            res[f"T{T}_{preset}"] = dict(tokens=T, remap=preset, **stack.measure(per_layer, args.steps, args.warmup))
        if table is not None and T == headline[0]:
            alpha, beta, _ = preset_args(wl, headline[1])
            per_layer = [preset_args(wl, n) if n != "off" else (alpha, beta, 0) for n in table]
            res["layer_policy"] = dict(tokens=T, remap="layer_policy", **stack.measure(per_layer, args.steps, args.warmup))
    T, preset = headline
    best = res[f"T{T}_{preset}"]
    alpha, beta, _ = preset_args(wl, preset)
    launches = n_layers * stack.L.lynx_moe_ffn_launches(T, cfg.F)
    out = {"metric": f"MoE-stack decode us/batch ({n_layers} chained layers)", "value": best["us_graph_wall"], "unit": "us/batch",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(best["us_graph_wall"] * 1e-3, 5),
           "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"{n_layers} chained {cfg.name}-shaped MoE layers (own router and expert weights each, "
                                  f"{n_layers * 3 * cfg.N * cfg.H * cfg.F * 2 / 1e9:.1f} GB of bf16 expert weights resident): hidden "
                                  f"{cfg.H}, FFN {cfg.F}, {cfg.N} experts top-{cfg.k}, {cfg.n_shared} shared, {T} decode tokens, "
                                  f"remap {preset}; x <- bf16(x + y) between layers, no normalisation (an un-normalised chain: "
                                  "token norms grow with depth and deeper layers route more sharply than layer 0); one "
                                  "HIP-graph replay per step",
                      "tokens": T, "alpha": alpha, "beta": beta, "layers": n_layers, "remap": preset},
           "us_per_layer": best["us_per_layer"], "tokens_per_s": best["tokens_per_s"],
           "experts_invoked": {"before_mean": best["invoked_before_mean"], "after_mean": best["invoked_after_mean"]},
           "remap_cost": {"psum_ratio": best["psum_ratio"], "top1_kept": best["top1_kept"]},
           "remap_gain_vs_off": (round(res[f"T{T}_off"]["us_graph_wall"] / best["us_graph_wall"], 3)
                                 if f"T{T}_off" in res else None),
           "stack": res, "layer_policy": args.layer_policy or None,
           "roofline": {"bound": "hbm", "kernel": "ffn_kernel (gate/up and down weight streams of all invoked experts), summed "
                                                  "over the layers of one pass of the stack, from the library's stage events",
                        "achieved": round(best["expert_weight_bytes"] / (best["ffn_kernel_us"] * 1e-6) / 1e9, 1),
                        "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": best["ffn_kernel_hbm_frac"],
                        "traffic": traffic_of(f"{cfg.name}_stack{n_layers}_T{T}_{preset}"),
                        "launches_per_step": launches, "bytes_per_launch": best["expert_weight_bytes"] // launches,
                        "avg_launch_us": round(best["ffn_kernel_us"] / launches, 2),
                        "whole_stack_frac": best["stack_hbm_frac"], "whole_stack_GBps": best["expert_weight_GBps_graph"]}}
    if cpu_layers:
        out["cpu_baseline"] = cpu_baseline_stack(stack, T, preset, torch, wl, cpu_layers)
    del stack
    torch.cuda.empty_cache()
    return out


def plain_read_ceiling(L, torch):
    """What a plain read-only streaming kernel reaches on this machine (2 GiB, same load width, with and without the hint)."""
    probe = torch.zeros(1 << 29, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    plain = {}
    for name, nt in (("non_temporal", True), ("default", False)):
        for _ in range(2):
            L.lynx_read_probe(probe, sink, nt)
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        for _ in range(5):
            L.lynx_read_probe(probe, sink, nt)
        p1.record()
        torch.cuda.synchronize()
        plain[name] = round(5 * probe.numel() * 4 / (p0.elapsed_time(p1) * 1e-3) / 1e9, 1)
    del probe
    return plain


def resident_copies(cfg, want=0):
    routed_bytes = 3 * cfg.N * cfg.H * cfg.F * 2
    return want if want > 0 else max(1, min(8, -(-(4 << 30) // routed_bytes)))


def single_layer_line(args, cfg, wl, torch, full=True):
    """The single-layer measurement of one configuration at args.tokens / args.preset with everything around it (sweep
    over the configuration's batch sizes, variants, CPU baseline): the line of `--config NAME`."""
    T = args.tokens
    if args.router == "sigmoid" or args.groups:
        args.no_fp8, args.no_cpu_baseline, args.biased_gamma = True, True, 0.0
    alpha, beta, enable = preset_args(wl, args.preset)
    n_layers = resident_copies(cfg, args.layers)
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
    events = new_events(torch, max(K, args.sweep_iters))
    for i in range(K):
        events[i][4].record()    # start of the step: routing = from here to the event before the gate/up kernel
        layer.step(T, alpha, beta, enable, events[i][:4])
    torch.cuda.synchronize()
    rt_ms = sum(e[4].elapsed_time(e[0]) for e in events[:K]) / K
    ffn_ms = sum(e[0].elapsed_time(e[1]) for e in events[:K]) / K      # the one kernel that streams all expert weights
    cb_ms = sum(e[2].elapsed_time(e[3]) for e in events[:K]) / K
    n_before, n_after = (int(v) for v in b.num_active.cpu().tolist())
    ratio, kept = remap_cost(b)
    gu_bytes, dn_bytes = expert_bytes(cfg, n_after)
    ffn_bytes = gu_bytes + dn_bytes
    ffn_gbps = ffn_bytes / (ffn_ms * 1e-3) / 1e9
    n_launch = layer.L.lynx_moe_ffn_launches(T, cfg.F)
    plain = plain_read_ceiling(layer.L, torch)

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
        "remap_cost": {"psum_ratio": ratio, "top1_kept": kept},
        "expert_weight_hbm_GBps": round(ffn_gbps, 1),
        # from the pass with events (each event adds a few us of idle GPU, so the stages sum to more than `value`)
        "stage_us": {"routing_a1_to_a7": round(rt_ms * 1e3, 2), "expert_ffn_a8": round(ffn_ms * 1e3, 2),
                     "combine_a9": round(cb_ms * 1e3, 2)},
        "roofline": {"bound": "hbm", "kernel": "ffn_kernel (gate/up and down weight streams of all invoked experts)",
                     "achieved": round(ffn_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(ffn_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": traffic_of(f"{cfg.name}_T{T}_{args.preset}"),
                     "launches_per_step": n_launch, "bytes_per_launch": ffn_bytes // n_launch,
                     "avg_launch_us": round(ffn_ms * 1e3 / n_launch, 2),
                     "plain_read_GBps": plain},
    }

    if not args.no_sweep:
        out["sweep"] = [measure_layer(layer, Ts, preset, args.sweep_iters, 3, torch, wl, events)
                        for Ts in cfg.batches for preset in PRESET_NAMES]
        if args.biased_gamma > 0 and full:
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
                            "invoked_before": nb, "invoked_after": na,
                            "psum_ratio": round(float((ab["new_psum"] / r["psum"]).mean().item()), 4)})
            out["sweep_score_biased_variant"] = var

    if not args.no_sweep and not args.groups and full:
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

        def quantised_variant(quantize, run_layer, bytes_num, bytes_den):
            qs = []
            for l in range(n_layers):
                d = wl.make_layer_device(cfg, 1, "cuda", layer=l)
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
            ffn_ms = sum(e[0].elapsed_time(e[1]) for e in events[:K]) / K
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
        for _ in range(3):
            t0 = time.perf_counter()
            o = oracle.moe_layer(xh, Wr, bias, rm["Wg"], rm["Wu"], rm["Wd"], cfg.k, alpha, beta, enable, rm["Sg"], rm["Su"],
                                 rm["Sd"])
            times.append(time.perf_counter() - t0)
        cpu_s = sorted(times)[len(times) // 2]
        out["cpu_baseline"] = {"value": round(cpu_s * 1e6, 1), "unit": "us/batch", "cores": oracle.num_threads(),
                               "kind": "oracle",
                               "sample": f"one full layer pass of the same workload ({T} tokens, all invoked experts), "
                                         "median of 3 repetitions, plain C fp64 oracle with an OpenMP split over weight rows",
                               "experts_invoked": [int(v) for v in o["bin"]["num_active"]]}
    del layer
    torch.cuda.empty_cache()
    return out


def full_report(args, wl, torch):
    """Every benchmark configuration in one line; the stack is the headline."""
    t_start = time.perf_counter()
    cfg4 = wl.CONFIGS["qwen3"]
    out = stack_line(args, cfg4, wl, torch, args.stack_layers, list(cfg4.batches), PRESET_NAMES,
                     headline=(max(cfg4.batches), "aggressive"),
                     cpu_layers=0 if args.no_cpu_baseline else min(4, args.stack_layers))
    out["seconds"] = {"stack": round(time.perf_counter() - t_start, 1)}
    entries = []
    for name in ("mixtral", "qwen15moe", "dsv2lite"):
        t0 = time.perf_counter()
        cfg = wl.CONFIGS[name]
        if name == "mixtral":
            # the Mixtral-shaped layer at 8 tokens in detail; its sweep is this configuration's part of `configs`
            a2 = argparse.Namespace(**vars(args))
            a2.config, a2.tokens, a2.preset, a2.no_cpu_baseline, a2.biased_gamma = name, 8, "aggressive", True, 0.0
            d = single_layer_line(a2, cfg, wl, torch, full=False)
            entries += d.pop("sweep")
            out["mixtral_T8"] = {k: d[k] for k in ("value", "config", "tokens_per_s", "experts_invoked", "remap_cost", "stage_us",
                                                   "roofline", "fp8_weights", "mxfp4_weights") if k in d}
        else:
            layer = Layer(cfg, cfg.batches[0], n_layers=resident_copies(cfg))
            evs = new_events(torch, args.sweep_iters)
            entries += [measure_layer(layer, Ts, preset, args.sweep_iters, 3, torch, wl, evs)
                        for Ts in cfg.batches for preset in PRESET_NAMES]
            del layer
            torch.cuda.empty_cache()
        out["seconds"][name] = round(time.perf_counter() - t0, 1)
    out["configs"] = entries
    return out


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
    if args.down_item_cap or args.down_item_units or args.down_k_waves:
        import paper_2411_08982_amd as L_
        from paper_2411_08982_amd import binding as B_
        L_.lynx_debug_set(B_.DEBUG_DOWN_ITEM_CAP, args.down_item_cap)
        L_.lynx_debug_set(B_.DEBUG_DOWN_ITEM_UNITS, args.down_item_units)
        L_.lynx_debug_set(B_.DEBUG_DOWN_K_WAVES, args.down_k_waves)
    if not args.config:
        out = full_report(args, wl, torch)
    elif args.stack > 0:
        cfg = wl.CONFIGS[args.config]
        table = layer_policy(args.layer_policy, args.stack, args.preset) if args.layer_policy else None
        presets = ["off"] + ([args.preset] if args.preset != "off" else [])
        out = stack_line(args, cfg, wl, torch, args.stack, [args.tokens], presets, headline=(args.tokens, args.preset),
                         table=table)
        out["stack"] = {v["remap"]: v for v in out["stack"].values()}   # one batch size: keyed by the remap setting
    else:
        out = single_layer_line(args, wl.CONFIGS[args.config], wl, torch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
