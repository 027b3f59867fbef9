"""Seeded synthetic inputs for the Lynx MoE decode layer (arXiv 2411.08982).

This module only draws random numbers and lays them out; it holds none of the method's arithmetic
and is the one module that both the CPU oracle's tests and the HIP path's tests / benchmark use.

Shapes follow the model families the paper evaluates (Sec. 5.1, Table 1): a Mixtral-8x7B-shaped
layer, a Qwen1.5-MoE-shaped layer with one shared expert, a DeepSeek-V2-Lite-shaped layer with two
shared experts, and a Qwen3-30B-A3B-shaped layer, plus a tiny functional case.  No trained weights
or datasets are used: hidden states are N(0,1) rounded to bf16, expert weights N(0, 0.02^2) rounded
to bf16, the router is N(0, 1/H) in fp32, and a per-expert logit bias with a Zipf-shaped popularity
prior reproduces the batch-level activation skew the paper reports (Sec. 2.2, Fig. 3).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class MoEConfig:
    name: str
    H: int          # hidden size
    F: int          # routed-expert FFN width
    N: int          # routed experts
    k: int          # experts per token
    n_shared: int   # shared experts (always active, weight 1)
    F_shared: int   # shared-expert FFN width
    zipf_s: float   # exponent of the popularity prior on the router bias
    bias_scale: float
    tail_frac: float  # fraction of tokens forced to near-uniform logits
    batches: tuple
    seed: int
    layers: int = 1


CONFIGS = {
    "tiny": MoEConfig("tiny", 512, 1024, 8, 2, 0, 0, 1.1, 0.5, 0.0, (16,), 0),
    "mixtral": MoEConfig("mixtral", 4096, 14336, 8, 2, 0, 0, 1.1, 0.5, 0.0, (1, 8, 32, 64, 128), 1),
    "qwen15moe": MoEConfig("qwen15moe", 2048, 1408, 60, 4, 1, 5632, 1.0, 0.5, 0.0, (8, 32, 64, 128, 256), 2),
    "dsv2lite": MoEConfig("dsv2lite", 2048, 1408, 64, 6, 2, 1408, 0.9, 0.5, 0.05, (16, 64, 128, 256), 3),
    "qwen3": MoEConfig("qwen3", 2048, 768, 128, 8, 0, 0, 1.0, 0.5, 0.0, (32, 128, 256, 512), 4, layers=48),
    # not one of the benchmark's configurations: a DeepSeek-V3-shaped layer (256 routed experts, top-8, one shared
    # expert, sigmoid-gated router) for the sigmoid-router widening; 22.5 GB of routed expert weights per layer
    "dsv3": MoEConfig("dsv3", 7168, 2048, 256, 8, 1, 2048, 1.0, 0.5, 0.0, (8, 32, 64, 128), 5),
}

# (alpha, beta) presets of the binning resolution; the paper prints no values (Sec. 3.2.1).
PRESETS = {"moderate": (2.0, 2), "aggressive": (4.0, 1)}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_normal(rng: np.random.Generator, shape, std: float, chunk: int = 1 << 24) -> np.ndarray:
    """N(0, std^2) rounded to bf16 bits, drawn in chunks to bound peak memory."""
    n = int(np.prod(shape))
    out = np.empty(n, np.uint16)
    for s in range(0, n, chunk):
        m = min(chunk, n - s)
        v = rng.standard_normal(m, dtype=np.float32)
        v *= np.float32(std)
        out[s:s + m] = f32_to_bf16_bits(v)
    return out.reshape(shape)


def zipf_bias(N: int, s: float, scale: float, rng: np.random.Generator) -> np.ndarray:
    """Per-expert logit bias: a random permutation gives each expert a popularity rank r in 1..N,
    w = r^-s, bias = scale * (ln w - mean ln w)."""
    ranks = rng.permutation(N) + 1
    lw = -s * np.log(ranks.astype(np.float64))
    return (scale * (lw - lw.mean())).astype(np.float32)


def make_router(cfg: MoEConfig, seed: int | None = None, layer: int = 0):
    rng = np.random.default_rng([cfg.seed if seed is None else seed, layer, 11])
    Wr = (rng.standard_normal((cfg.N, cfg.H), dtype=np.float32) / np.float32(np.sqrt(cfg.H))).astype(np.float32)
    bias = zipf_bias(cfg.N, cfg.zipf_s, cfg.bias_scale, rng)
    return Wr, bias


def make_tokens(cfg: MoEConfig, T: int, Wr=None, bias=None, seed: int | None = None, layer: int = 0) -> np.ndarray:
    """Hidden states [T,H] as bf16 bits.  For configs with a low-affinity tail, a seeded fraction of the
    tokens is shifted inside the row space of the router so that their logits come out near-uniform
    (N(0, 0.02^2) around 0).  This shapes an input: it solves a linear system in Wr for a prescribed router response
    (numpy's matmul and solve); no expected value of any test comes from it, and neither the oracle nor the kernels
    use it."""
    rng = np.random.default_rng([cfg.seed if seed is None else seed, layer, 22, T])
    x = rng.standard_normal((T, cfg.H), dtype=np.float32)
    if cfg.tail_frac > 0 and T > 0 and Wr is not None:
        n_tail = max(1, int(round(cfg.tail_frac * T)))
        tail = np.sort(rng.choice(T, size=n_tail, replace=False))
        W = Wr.astype(np.float64)
        b = np.zeros(cfg.N) if bias is None else bias.astype(np.float64)
        target = rng.standard_normal((n_tail, cfg.N)) * 0.02
        resid = target - (x[tail].astype(np.float64) @ W.T + b)          # [n_tail, N]
        corr = np.linalg.solve(W @ W.T, resid.T).T @ W                     # minimum-norm shift
        x[tail] = (x[tail].astype(np.float64) + corr).astype(np.float32)
    return f32_to_bf16_bits(x)


def make_expert_weights(cfg: MoEConfig, seed: int | None = None, layer: int = 0, n_experts: int | None = None):
    """Routed (Wg, Wu [N,F,H], Wd [N,H,F]) and shared (Sg, Su [S,Fs,H], Sd [S,H,Fs]) weights, bf16 bits."""
    rng = np.random.default_rng([cfg.seed if seed is None else seed, layer, 33])
    N = cfg.N if n_experts is None else n_experts
    Wg = bf16_normal(rng, (N, cfg.F, cfg.H), 0.02)
    Wu = bf16_normal(rng, (N, cfg.F, cfg.H), 0.02)
    Wd = bf16_normal(rng, (N, cfg.H, cfg.F), 0.02)
    if cfg.n_shared > 0:
        Sg = bf16_normal(rng, (cfg.n_shared, cfg.F_shared, cfg.H), 0.02)
        Su = bf16_normal(rng, (cfg.n_shared, cfg.F_shared, cfg.H), 0.02)
        Sd = bf16_normal(rng, (cfg.n_shared, cfg.H, cfg.F_shared), 0.02)
    else:
        Sg = Su = Sd = None
    return dict(Wg=Wg, Wu=Wu, Wd=Wd, Sg=Sg, Su=Su, Sd=Sd)


def make_layer(cfg: MoEConfig, T: int, seed: int | None = None, layer: int = 0, weights: bool = True):
    Wr, bias = make_router(cfg, seed, layer)
    x = make_tokens(cfg, T, Wr, bias, seed, layer)
    d = dict(cfg=cfg, T=T, x=x, Wr=Wr, bias=bias)
    if weights:
        d.update(make_expert_weights(cfg, seed, layer))
    return d


def make_logits(T: int, N: int, seed: int, zipf_s: float = 1.0, bias_scale: float = 0.5, tail_frac: float = 0.0,
                quantum: float | None = None) -> np.ndarray:
    """Router-like logits drawn directly: N(0,1) + Zipf bias, optional near-uniform tail.  With `quantum`
    the values are rounded to multiples of it, which makes exact ties and bin-boundary hits common."""
    rng = np.random.default_rng([seed, T, N, 44])
    z = rng.standard_normal((T, N)).astype(np.float32) + zipf_bias(N, zipf_s, bias_scale, rng)[None, :]
    if tail_frac > 0 and T > 0:
        n_tail = max(1, int(round(tail_frac * T)))
        tail = rng.choice(T, size=n_tail, replace=False)
        z[tail] = (rng.standard_normal((n_tail, N)) * 0.02).astype(np.float32)
    if quantum:
        z = (np.round(z / quantum) * quantum).astype(np.float32)
    return np.ascontiguousarray(z, dtype=np.float32)


# ---- device-side generation for the large configurations (benchmark, full-size GPU tests) --------

def make_layer_device(cfg: MoEConfig, T: int, device, seed: int | None = None, layer: int = 0):
    """Same recipe drawn with torch's generator on `device` (used where the weights are too large to
    draw on the host in reasonable time).  Router and tokens still come from the numpy recipe so that
    the low-affinity tail is identical; only the expert weights are drawn on the device.  Returns torch
    tensors: x, weights as bfloat16; Wr, bias as float32."""
    import torch

    Wr, bias = make_router(cfg, seed, layer)
    x = make_tokens(cfg, T, Wr, bias, seed, layer)
    g = torch.Generator(device=device)
    g.manual_seed(((cfg.seed if seed is None else seed) * 1000003 + layer) * 7 + 33)

    def draw(shape):
        out = torch.empty(shape, dtype=torch.bfloat16, device=device)
        flat = out.view(shape[0], -1)
        for i in range(shape[0]):  # one expert at a time keeps the fp32 temporary small
            flat[i].copy_(torch.randn(flat.shape[1], generator=g, device=device, dtype=torch.float32).mul_(0.02))
        return out

    d = dict(cfg=cfg, T=T,
             x=torch.from_numpy(x.view(np.int16)).to(device).view(torch.bfloat16),
             Wr=torch.from_numpy(Wr).to(device), bias=torch.from_numpy(bias).to(device),
             Wg=draw((cfg.N, cfg.F, cfg.H)), Wu=draw((cfg.N, cfg.F, cfg.H)), Wd=draw((cfg.N, cfg.H, cfg.F)))
    if cfg.n_shared > 0:
        d.update(Sg=draw((cfg.n_shared, cfg.F_shared, cfg.H)), Su=draw((cfg.n_shared, cfg.F_shared, cfg.H)),
                 Sd=draw((cfg.n_shared, cfg.H, cfg.F_shared)))
    else:
        d.update(Sg=None, Su=None, Sd=None)
    return d
