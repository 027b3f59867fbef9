"""The whole-layer entry point on the library's built-in scratch array (for callers that cannot allocate) against
lynx_moe_layer with a caller-provided workspace: same kernels, so every output must be bit-identical.  Two calls in a
row share the one array; the second is smaller, so it runs over what the first left behind."""
import numpy as np
import pytest
import torch

import paper_2411_08982_amd as L
import workloads as wl
from gpu_util import dev, host, to_bf16_dev

pytestmark = pytest.mark.gpu

FIELDS = ("logits", "topk_idx", "topk_gate", "topk_psum", "new_idx", "new_gate", "cnt_before", "cnt_after", "bin_hist",
          "num_active", "offsets", "perm", "active", "num_active_perm", "y")


def _layer(cfg_name, T):
    cfg = wl.CONFIGS[cfg_name]
    d = wl.make_layer(cfg, T)
    Wgu, Wdp = L.lynx_pack_weights(to_bf16_dev(d["Wg"]), to_bf16_dev(d["Wu"]), to_bf16_dev(d["Wd"]))
    return cfg, to_bf16_dev(d["x"]), dev(d["Wr"]), dev(d["bias"]), Wgu, Wdp


def _poisoned(cfg, T, beta):
    b = L.LayerBuffers(T, cfg.H, cfg.F, cfg.N, cfg.k, beta)
    for name in FIELDS:
        getattr(b, name).view(torch.uint8).fill_(0xFF)
    b.workspace.fill_(0xFF)
    return b


@pytest.mark.parametrize("sizes", [(48, 16), (16, 5), (40, 1)])
def test_static_scratch_layer_matches_workspace_layer_twice_in_a_row(sizes):
    alpha, beta = wl.PRESETS["moderate"]
    for T in sizes:   # the second call is the smaller one
        cfg, x, Wr, bias, Wgu, Wdp = _layer("tiny", T)
        ref = L.lynx_moe_layer(x, Wr, bias, Wgu, Wdp, cfg.F, cfg.k, alpha, beta, 1, buffers=_poisoned(cfg, T, beta))
        got = L.lynx_moe_layer_static(x, Wr, bias, Wgu, Wdp, cfg.F, cfg.k, alpha, beta, 1, buffers=_poisoned(cfg, T, beta))
        torch.cuda.synchronize()
        for name in FIELDS:
            a, b = host(getattr(ref, name)), host(getattr(got, name))
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), f"T={T}: {name} differs"
        assert np.isfinite(host(got.y)).all()
        assert int(host(ref.workspace.view(torch.int32))[L.binding.WAIT_FLAG_WORD]) == 0


def test_static_scratch_layer_refuses_what_does_not_fit():
    cfg = wl.CONFIGS["mixtral"]
    assert L.workspace_bytes(1024, cfg.H, cfg.F, cfg.N, cfg.k) > L.binding.STATIC_SCRATCH_BYTES
    one = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(L.LynxError) as ei:
        b = L.LayerBuffers(1024, cfg.H, cfg.F, cfg.N, cfg.k, 2)
        x = torch.zeros((1024, cfg.H), dtype=torch.bfloat16, device="cuda")
        Wr = torch.zeros((cfg.N, cfg.H), dtype=torch.float32, device="cuda")
        L.lynx_moe_layer_static(x, Wr, None, one, one, cfg.F, cfg.k, 2.0, 2, 1, buffers=b)
    assert ei.value.code == L.binding.ERR_UNSUPPORTED
