"""ctypes binding of liblynx.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used for device memory and
streams, nothing else), checks dtype / contiguity / device, and passes raw device pointers and the
current HIP stream to the C ABI declared in include/lynx.h.  No step of the path runs in Python or
torch, and there is no CPU fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_float, c_int, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblynx.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_HIP = 0, -1, -2, -3
MAX_T, MAX_N, MAX_K, MAX_BETA = 1024, 256, 16, 6

SYMBOLS = ["lynx_last_error", "lynx_workspace_bytes", "lynx_route", "lynx_affinity_bin", "lynx_affinity_bin_biased", "lynx_permute",
           "lynx_pack_weights", "lynx_moe_ffn", "lynx_moe_ffn_timed", "lynx_moe_layer", "lynx_moe_layer_static", "lynx_moe_ffn_launches", "lynx_residual_add", "lynx_read_probe",
           "lynx_quantize_weights_fp8", "lynx_moe_ffn_fp8", "lynx_moe_layer_fp8",
           "lynx_fp4_scale_words", "lynx_quantize_weights_fp4", "lynx_moe_ffn_fp4", "lynx_moe_layer_fp4",
           "lynx_route_sigmoid", "lynx_affinity_bin_sigmoid", "lynx_moe_layer_sigmoid",
           "lynx_route_grouped", "lynx_affinity_bin_grouped", "lynx_moe_layer_grouped", "lynx_debug_set"]


class LynxError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"liblynx error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Loads liblynx.so (built in-tree by paper_2411_08982_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built: run `python -m paper_2411_08982_amd.build` "
                                    "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        P, I, F = c_void_p, c_int, c_float
        L.lynx_last_error.restype = ctypes.c_char_p
        L.lynx_last_error.argtypes = []
        L.lynx_workspace_bytes.restype = c_size_t
        L.lynx_workspace_bytes.argtypes = [I] * 7
        L.lynx_route.argtypes = [P, P, P, I, I, I, I, P, P, P, P, P]
        L.lynx_affinity_bin.argtypes = [P, P, I, I, I, F, I, I, P, P, P, P, P, P, P, P, P]
        L.lynx_affinity_bin_biased.argtypes = [P, P, I, I, I, F, I, F, I, P, P, P, P, P, P, P, P, P]
        L.lynx_permute.argtypes = [P, I, I, I, P, P, P, P, P]
        L.lynx_pack_weights.argtypes = [P, P, P, I, I, I, P, P, P]
        L.lynx_moe_ffn.argtypes = [P, P, P, P, P, I, I, P, P, P, P, P, P, I, I, I, I, I, P, P, P, P]
        L.lynx_moe_ffn_timed.argtypes = L.lynx_moe_ffn.argtypes + [ctypes.POINTER(c_void_p)]
        L.lynx_moe_layer.argtypes = [P, P, P, P, P, P, P, I, I, I, I, I, I, I, F, I, I] + [P] * 19 + [ctypes.POINTER(c_void_p)]
        L.lynx_moe_layer_static.argtypes = [P, P, P, P, P, P, P, I, I, I, I, I, I, I, F, I, I] + [P] * 18
        L.lynx_read_probe.argtypes = [P, c_size_t, I, P, P]
        L.lynx_quantize_weights_fp8.argtypes = [P, P, P, I, I, I, P, P, P, P, P]
        L.lynx_moe_ffn_fp8.argtypes = [P] * 9 + [I, I] + [P] * 6 + [I] * 5 + [P, P, P, P, ctypes.POINTER(c_void_p)]
        L.lynx_moe_layer_fp8.argtypes = [P] * 11 + [I] * 7 + [F, I, I] + [P] * 19 + [ctypes.POINTER(c_void_p)]
        L.lynx_fp4_scale_words.argtypes = [I, I, I, I]
        L.lynx_quantize_weights_fp4.argtypes = L.lynx_quantize_weights_fp8.argtypes
        L.lynx_moe_ffn_fp4.argtypes = L.lynx_moe_ffn_fp8.argtypes
        L.lynx_moe_layer_fp4.argtypes = L.lynx_moe_layer_fp8.argtypes
        L.lynx_moe_ffn_launches.argtypes = [I, I]
        L.lynx_residual_add.argtypes = [P, P, c_size_t, P, P]
        L.lynx_debug_set.argtypes = [I, I]
        L.lynx_route_sigmoid.argtypes = L.lynx_route.argtypes
        L.lynx_affinity_bin_sigmoid.argtypes = L.lynx_affinity_bin.argtypes
        L.lynx_moe_layer_sigmoid.argtypes = L.lynx_moe_layer.argtypes
        L.lynx_route_grouped.argtypes = [P, P, P, I, I, I, I, I, I, I, P, P, P, P, P]
        L.lynx_affinity_bin_grouped.argtypes = [P, I, I, I, I, I, I, F, I, I] + [P] * 12
        L.lynx_moe_layer_grouped.argtypes = ([P, P, P, P, P, P, P, I, I, I, I, I, I, I, I, I, I, F, I, I] + [P] * 19 +
                                             [ctypes.POINTER(c_void_p)])
        for name in SYMBOLS:
            # without declared argument types ctypes passes Python ints as 32-bit C ints: a device pointer would be cut
            if getattr(L, name).argtypes is None:
                raise RuntimeError(f"binding: no argument types declared for {name}")
        for name in SYMBOLS[2:]:
            getattr(L, name).restype = c_int
        L.lynx_fp4_scale_words.restype = c_size_t
        _lib = L
    return _lib


def _check(rc: int):
    if rc != OK:
        raise LynxError(rc, lib().lynx_last_error().decode())


def _ptr(t, dtype, what):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{what}: expected a CUDA/HIP tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: must be contiguous")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


BF16, F32, I32 = torch.bfloat16, torch.float32, torch.int32


WAIT_FLAG_WORD = 9744   # int32 word of the workspace: non-zero if a bounded wait inside the FFN kernel ran out


def workspace_bytes(T, H, F, N, k, n_shared=0, F_shared=0) -> int:
    return int(lib().lynx_workspace_bytes(T, H, F, N, k, n_shared, F_shared))


def new_workspace(T, H, F, N, k, n_shared=0, F_shared=0, device="cuda"):
    return torch.empty(max(workspace_bytes(T, H, F, N, k, n_shared, F_shared), 256), dtype=torch.uint8, device=device)


def lynx_route(x, Wr, bias, k, out=None, _entry="lynx_route"):
    """x [T,H] bf16, Wr [N,H] f32, bias [N] f32 or None -> dict(logits, idx, gate, psum)."""
    T, H = x.shape
    N = Wr.shape[0]
    dev = x.device
    o = out or dict(logits=torch.empty((T, N), dtype=F32, device=dev), idx=torch.empty((T, k), dtype=I32, device=dev),
                    gate=torch.empty((T, k), dtype=F32, device=dev), psum=torch.empty((T,), dtype=F32, device=dev))
    _check(getattr(lib(), _entry)(_ptr(x, BF16, "x"), _ptr(Wr, F32, "Wr"), _ptr(bias, F32, "bias"), T, H, N, k,
                                  _ptr(o["logits"], F32, "logits"), _ptr(o["idx"], I32, "idx"),
                                  _ptr(o["gate"], F32, "gate"), _ptr(o["psum"], F32, "psum"), _stream()))
    return o


def lynx_route_sigmoid(x, Wr, bias, k, out=None):
    """lynx_route for a sigmoid-gated router; the entry "psum" holds the sum of the selected scores."""
    return lynx_route(x, Wr, bias, k, out, _entry="lynx_route_sigmoid")


def lynx_route_grouped(x, Wr, bias, k, n_group, topk_group, gate_fn=0, out=None):
    """lynx_route for a group-limited router (gate_fn 0 softmax, 1 sigmoid); "psum" holds the third output."""
    T, H = x.shape
    N = Wr.shape[0]
    dev = x.device
    o = out or dict(logits=torch.empty((T, N), dtype=F32, device=dev), idx=torch.empty((T, k), dtype=I32, device=dev),
                    gate=torch.empty((T, k), dtype=F32, device=dev), psum=torch.empty((T,), dtype=F32, device=dev))
    _check(lib().lynx_route_grouped(_ptr(x, BF16, "x"), _ptr(Wr, F32, "Wr"), _ptr(bias, F32, "bias"), T, H, N, k,
                                    int(n_group), int(topk_group), int(gate_fn), _ptr(o["logits"], F32, "logits"),
                                    _ptr(o["idx"], I32, "idx"), _ptr(o["gate"], F32, "gate"), _ptr(o["psum"], F32, "psum"),
                                    _stream()))
    return o


def lynx_affinity_bin_grouped(logits, k, n_group, topk_group, alpha, beta, gate_fn=0, enable=1, workspace=None, out=None):
    """Group-limited top-k and remap from logits [T,N] f32 -> dict(idx, gate, psum, new_idx, new_gate, cnt_before,
    cnt_after, bin_hist, num_active)."""
    T, N = logits.shape
    dev = logits.device
    nb = max(int(beta), 1)
    o = out or dict(idx=torch.empty((T, k), dtype=I32, device=dev), gate=torch.empty((T, k), dtype=F32, device=dev),
                    psum=torch.empty((T,), dtype=F32, device=dev),
                    new_idx=torch.empty((T, k), dtype=I32, device=dev), new_gate=torch.empty((T, k), dtype=F32, device=dev),
                    new_psum=torch.empty((T,), dtype=F32, device=dev),
                    cnt_before=torch.empty((N,), dtype=I32, device=dev), cnt_after=torch.empty((N,), dtype=I32, device=dev),
                    bin_hist=torch.empty((N, nb), dtype=I32, device=dev), num_active=torch.empty((2,), dtype=I32, device=dev))
    if workspace is None:
        workspace = torch.empty(65536, dtype=torch.uint8, device=dev)
    _check(lib().lynx_affinity_bin_grouped(_ptr(logits, F32, "logits"), T, N, int(k), int(n_group), int(topk_group),
                                           int(gate_fn), float(alpha), int(beta), int(enable), _ptr(o["idx"], I32, "idx"),
                                           _ptr(o["gate"], F32, "gate"), _ptr(o["psum"], F32, "psum"),
                                           _ptr(o["new_idx"], I32, "new_idx"), _ptr(o["new_gate"], F32, "new_gate"),
                                           _ptr(o.get("new_psum"), F32, "new_psum"),
                                           _ptr(o["cnt_before"], I32, "cnt_before"), _ptr(o["cnt_after"], I32, "cnt_after"),
                                           _ptr(o["bin_hist"], I32, "bin_hist"), _ptr(o["num_active"], I32, "num_active"),
                                           workspace.data_ptr(), _stream()))
    return o


def lynx_affinity_bin(logits, topk_idx, alpha, beta, enable=1, workspace=None, out=None, _entry="lynx_affinity_bin"):
    """logits [T,N] f32, topk_idx [T,k] i32 -> dict(new_idx, new_gate, cnt_before, cnt_after, bin_hist, num_active)."""
    T, N = logits.shape
    k = topk_idx.shape[1]
    dev = logits.device
    nb = max(int(beta), 1)
    o = out or dict(new_idx=torch.empty((T, k), dtype=I32, device=dev), new_gate=torch.empty((T, k), dtype=F32, device=dev),
                    new_psum=torch.empty((T,), dtype=F32, device=dev),
                    cnt_before=torch.empty((N,), dtype=I32, device=dev), cnt_after=torch.empty((N,), dtype=I32, device=dev),
                    bin_hist=torch.empty((N, nb), dtype=I32, device=dev), num_active=torch.empty((2,), dtype=I32, device=dev))
    if workspace is None:
        workspace = torch.empty(65536, dtype=torch.uint8, device=dev)
    ws = workspace.data_ptr()
    _check(getattr(lib(), _entry)(_ptr(logits, F32, "logits"), _ptr(topk_idx, I32, "topk_idx"), T, N, k, float(alpha),
                                  int(beta), int(enable), _ptr(o["new_idx"], I32, "new_idx"),
                                  _ptr(o["new_gate"], F32, "new_gate"), _ptr(o.get("new_psum"), F32, "new_psum"),
                                  _ptr(o["cnt_before"], I32, "cnt_before"),
                                  _ptr(o["cnt_after"], I32, "cnt_after"), _ptr(o["bin_hist"], I32, "bin_hist"),
                                  _ptr(o["num_active"], I32, "num_active"), ws, _stream()))
    return o


def lynx_affinity_bin_sigmoid(logits, topk_idx, alpha, beta, enable=1, workspace=None, out=None):
    """lynx_affinity_bin with the gates of a sigmoid-gated router."""
    return lynx_affinity_bin(logits, topk_idx, alpha, beta, enable, workspace, out, _entry="lynx_affinity_bin_sigmoid")


def lynx_affinity_bin_biased(logits, topk_idx, alpha, beta, gamma, enable=1, workspace=None, out=None):
    """Score-biased selection variant; arguments and result as lynx_affinity_bin plus the bias strength gamma."""
    T, N = logits.shape
    k = topk_idx.shape[1]
    dev = logits.device
    nb = max(int(beta), 1)
    o = out or dict(new_idx=torch.empty((T, k), dtype=I32, device=dev), new_gate=torch.empty((T, k), dtype=F32, device=dev),
                    new_psum=torch.empty((T,), dtype=F32, device=dev),
                    cnt_before=torch.empty((N,), dtype=I32, device=dev), cnt_after=torch.empty((N,), dtype=I32, device=dev),
                    bin_hist=torch.empty((N, nb), dtype=I32, device=dev), num_active=torch.empty((2,), dtype=I32, device=dev))
    if workspace is None:
        workspace = torch.empty(65536, dtype=torch.uint8, device=dev)
    _check(lib().lynx_affinity_bin_biased(_ptr(logits, F32, "logits"), _ptr(topk_idx, I32, "topk_idx"), T, N, k,
                                          float(alpha), int(beta), float(gamma), int(enable),
                                          _ptr(o["new_idx"], I32, "new_idx"), _ptr(o["new_gate"], F32, "new_gate"),
                                          _ptr(o.get("new_psum"), F32, "new_psum"),
                                          _ptr(o["cnt_before"], I32, "cnt_before"), _ptr(o["cnt_after"], I32, "cnt_after"),
                                          _ptr(o["bin_hist"], I32, "bin_hist"), _ptr(o["num_active"], I32, "num_active"),
                                          workspace.data_ptr(), _stream()))
    return o


def lynx_permute(idx, N, out=None):
    """idx [T,k] i32 -> dict(offsets [N+1], perm [T*k], active [N], num_active [1])."""
    T, k = idx.shape
    dev = idx.device
    o = out or dict(offsets=torch.empty((N + 1,), dtype=I32, device=dev), perm=torch.empty((T * k,), dtype=I32, device=dev),
                    active=torch.empty((N,), dtype=I32, device=dev), num_active=torch.empty((1,), dtype=I32, device=dev))
    _check(lib().lynx_permute(_ptr(idx, I32, "idx"), T, N, k, _ptr(o["offsets"], I32, "offsets"),
                              _ptr(o["perm"], I32, "perm"), _ptr(o["active"], I32, "active"),
                              _ptr(o["num_active"], I32, "num_active"), _stream()))
    return o


def lynx_pack_weights(Wg, Wu, Wd):
    """Wg, Wu [E,F,H], Wd [E,H,F] bf16 row-major -> (Wgu_packed, Wd_packed) in the streaming layout."""
    E, F, H = Wg.shape
    if Wu.shape != (E, F, H) or Wd.shape != (E, H, F):
        raise ValueError("weight shapes do not match")
    Wgu = torch.empty((E, F // 16, H // 32, 2, 64, 8), dtype=BF16, device=Wg.device)
    Wdp = torch.empty((E, H // 16, F // 32, 64, 8), dtype=BF16, device=Wg.device)
    _check(lib().lynx_pack_weights(_ptr(Wg, BF16, "Wg"), _ptr(Wu, BF16, "Wu"), _ptr(Wd, BF16, "Wd"), E, H, F,
                                   _ptr(Wgu, BF16, "Wgu"), _ptr(Wdp, BF16, "Wdp"), _stream()))
    return Wgu, Wdp


def lynx_moe_ffn(x, Wgu, Wdp, idx, gate, perm_out, N, F, Sgu=None, Sdp=None, n_shared=0, F_shared=0, workspace=None,
                 y=None, stage_events=None, status=None):
    """x [T,H] bf16, packed weights, idx/gate [T,k], perm_out = result of lynx_permute -> y [T,H] f32.
    stage_events: optional list of four torch.cuda.Event(enable_timing=True) that have been recorded at
    least once (so that their handles exist); they are re-recorded at the stage boundaries."""
    T, H = x.shape
    k = idx.shape[1]
    if workspace is None:
        workspace = new_workspace(T, H, F, N, k, n_shared, F_shared, x.device)
    need = workspace_bytes(T, H, F, N, k, n_shared, F_shared)
    if workspace.numel() * workspace.element_size() < need:
        raise ValueError(f"workspace too small: {workspace.numel()} < {need}")
    if y is None:
        y = torch.empty((T, H), dtype=F32, device=x.device)
    args = (_ptr(x, BF16, "x"), _ptr(Wgu, BF16, "Wgu"), _ptr(Wdp, BF16, "Wdp"), _ptr(Sgu, BF16, "Sgu"),
            _ptr(Sdp, BF16, "Sdp"), n_shared, F_shared, _ptr(idx, I32, "idx"), _ptr(gate, F32, "gate"),
            _ptr(perm_out["offsets"], I32, "offsets"), _ptr(perm_out["perm"], I32, "perm"),
            _ptr(perm_out["active"], I32, "active"), _ptr(perm_out["num_active"], I32, "num_active"),
            T, H, F, N, k, _ptr(y, F32, "y"), _ptr(status, I32, "status"), workspace.data_ptr(), _stream())
    if stage_events is None:
        _check(lib().lynx_moe_ffn(*args))
    else:
        ev = (c_void_p * 4)(*[e.cuda_event for e in stage_events])
        _check(lib().lynx_moe_ffn_timed(*args, ev))
    return y


class LayerBuffers:
    """All outputs and scratch of lynx_moe_layer for fixed sizes, allocated once."""

    def __init__(self, T, H, F, N, k, beta, n_shared=0, F_shared=0, device="cuda"):
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=device)
        self.sizes = (T, H, F, N, k, n_shared, F_shared)
        self.beta = beta
        self.logits, self.topk_idx, self.topk_gate, self.topk_psum = e((T, N), F32), e((T, k), I32), e((T, k), F32), e((T,), F32)
        self.new_idx, self.new_gate, self.new_psum = e((T, k), I32), e((T, k), F32), e((T,), F32)
        self.status = e((1,), I32)
        self.cnt_before, self.cnt_after, self.bin_hist, self.num_active = e((N,), I32), e((N,), I32), e((N, beta), I32), e((2,), I32)
        self.offsets, self.perm, self.active, self.num_active_perm = e((N + 1,), I32), e((max(T * k, 1),), I32), e((N,), I32), e((1,), I32)
        self.y = e((T, H), F32)
        self.workspace = new_workspace(T, H, F, N, k, n_shared, F_shared, device)


def lynx_moe_layer(x, Wr, bias, Wgu, Wdp, F, k, alpha, beta, enable=1, Sgu=None, Sdp=None, n_shared=0, F_shared=0,
                   buffers: LayerBuffers | None = None, stage_events=None, _entry="lynx_moe_layer"):
    """route -> affinity_bin -> permute -> FFN + combine on the current stream.  Returns the LayerBuffers."""
    T, H = x.shape
    N = Wr.shape[0]
    b = buffers or LayerBuffers(T, H, F, N, k, beta, n_shared, F_shared, x.device)
    if b.sizes != (T, H, F, N, k, n_shared, F_shared) or b.beta != beta:
        raise ValueError("buffers were allocated for other sizes")
    _check(getattr(lib(), _entry)(
        _ptr(x, BF16, "x"), _ptr(Wr, F32, "Wr"), _ptr(bias, F32, "bias"), _ptr(Wgu, BF16, "Wgu"), _ptr(Wdp, BF16, "Wdp"),
        _ptr(Sgu, BF16, "Sgu"), _ptr(Sdp, BF16, "Sdp"), n_shared, F_shared, T, H, F, N, k, float(alpha), int(beta),
        int(enable), b.logits.data_ptr(), b.topk_idx.data_ptr(), b.topk_gate.data_ptr(), b.topk_psum.data_ptr(),
        b.new_idx.data_ptr(), b.new_gate.data_ptr(), b.new_psum.data_ptr(), b.cnt_before.data_ptr(), b.cnt_after.data_ptr(),
        b.bin_hist.data_ptr(), b.num_active.data_ptr(), b.offsets.data_ptr(), b.perm.data_ptr(), b.active.data_ptr(),
        b.num_active_perm.data_ptr(), b.y.data_ptr(), b.status.data_ptr(), b.workspace.data_ptr(), _stream(),
        None if stage_events is None else (c_void_p * 4)(*[e.cuda_event for e in stage_events])))
    return b


STATIC_SCRATCH_BYTES = 64 << 20   # LYNX_STATIC_SCRATCH_BYTES


def lynx_moe_layer_static(x, Wr, bias, Wgu, Wdp, F, k, alpha, beta, enable=1, Sgu=None, Sdp=None, n_shared=0, F_shared=0,
                          buffers: LayerBuffers | None = None):
    """lynx_moe_layer on the library's built-in scratch array (the call allocates nothing; b.workspace is not used)."""
    T, H = x.shape
    N = Wr.shape[0]
    b = buffers or LayerBuffers(T, H, F, N, k, beta, n_shared, F_shared, x.device)
    if b.sizes != (T, H, F, N, k, n_shared, F_shared) or b.beta != beta:
        raise ValueError("buffers were allocated for other sizes")
    _check(lib().lynx_moe_layer_static(
        _ptr(x, BF16, "x"), _ptr(Wr, F32, "Wr"), _ptr(bias, F32, "bias"), _ptr(Wgu, BF16, "Wgu"), _ptr(Wdp, BF16, "Wdp"),
        _ptr(Sgu, BF16, "Sgu"), _ptr(Sdp, BF16, "Sdp"), n_shared, F_shared, T, H, F, N, k, float(alpha), int(beta),
        int(enable), b.logits.data_ptr(), b.topk_idx.data_ptr(), b.topk_gate.data_ptr(), b.topk_psum.data_ptr(),
        b.new_idx.data_ptr(), b.new_gate.data_ptr(), b.new_psum.data_ptr(), b.cnt_before.data_ptr(), b.cnt_after.data_ptr(),
        b.bin_hist.data_ptr(), b.num_active.data_ptr(), b.offsets.data_ptr(), b.perm.data_ptr(), b.active.data_ptr(),
        b.num_active_perm.data_ptr(), b.y.data_ptr(), b.status.data_ptr(), _stream()))
    return b


def lynx_moe_layer_sigmoid(x, Wr, bias, Wgu, Wdp, F, k, alpha, beta, enable=1, Sgu=None, Sdp=None, n_shared=0, F_shared=0,
                           buffers: LayerBuffers | None = None, stage_events=None):
    """lynx_moe_layer for a sigmoid-gated router (topk_psum holds the sum of the selected scores)."""
    return lynx_moe_layer(x, Wr, bias, Wgu, Wdp, F, k, alpha, beta, enable, Sgu, Sdp, n_shared, F_shared, buffers,
                          stage_events, _entry="lynx_moe_layer_sigmoid")


def lynx_moe_layer_grouped(x, Wr, bias, Wgu, Wdp, F, k, n_group, topk_group, alpha, beta, gate_fn=0, enable=1, Sgu=None,
                           Sdp=None, n_shared=0, F_shared=0, buffers: LayerBuffers | None = None, stage_events=None):
    """lynx_moe_layer for a group-limited router (gate_fn 0 softmax, 1 sigmoid)."""
    T, H = x.shape
    N = Wr.shape[0]
    b = buffers or LayerBuffers(T, H, F, N, k, beta, n_shared, F_shared, x.device)
    if b.sizes != (T, H, F, N, k, n_shared, F_shared) or b.beta != beta:
        raise ValueError("buffers were allocated for other sizes")
    _check(lib().lynx_moe_layer_grouped(
        _ptr(x, BF16, "x"), _ptr(Wr, F32, "Wr"), _ptr(bias, F32, "bias"), _ptr(Wgu, BF16, "Wgu"), _ptr(Wdp, BF16, "Wdp"),
        _ptr(Sgu, BF16, "Sgu"), _ptr(Sdp, BF16, "Sdp"), n_shared, F_shared, T, H, F, N, k, int(n_group), int(topk_group),
        int(gate_fn), float(alpha), int(beta), int(enable), b.logits.data_ptr(), b.topk_idx.data_ptr(),
        b.topk_gate.data_ptr(), b.topk_psum.data_ptr(), b.new_idx.data_ptr(), b.new_gate.data_ptr(), b.new_psum.data_ptr(),
        b.cnt_before.data_ptr(), b.cnt_after.data_ptr(), b.bin_hist.data_ptr(), b.num_active.data_ptr(),
        b.offsets.data_ptr(), b.perm.data_ptr(), b.active.data_ptr(), b.num_active_perm.data_ptr(), b.y.data_ptr(), b.status.data_ptr(),
        b.workspace.data_ptr(), _stream(),
        None if stage_events is None else (c_void_p * 4)(*[e.cuda_event for e in stage_events])))
    return b


def lynx_read_probe(buf, sink, non_temporal=True):
    """Enqueues the plain read-only streaming kernel over `buf` (any contiguous device tensor whose byte size is a
    multiple of 16); `sink` is a one-element int32/uint32 device tensor.  The caller times it."""
    assert buf.is_cuda and buf.is_contiguous() and sink.is_cuda and sink.numel() >= 1 and sink.element_size() == 4
    _check(lib().lynx_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), int(bool(non_temporal)), sink.data_ptr(),
                                 _stream()))


def lynx_residual_add(x, y, out=None):
    """out = bf16(x + y) (x, out bf16; y fp32, same shape), the update that chains layers of a stack."""
    out = torch.empty_like(x) if out is None else out
    assert x.shape == y.shape == out.shape
    _check(lib().lynx_residual_add(_ptr(x, BF16, "x"), _ptr(y, F32, "y"), x.numel(), _ptr(out, BF16, "out"), _stream()))
    return out


DEBUG_SPIN_LIMIT, DEBUG_TARGET_BIAS, DEBUG_DOWN_ITEM_CAP, DEBUG_DOWN_ITEM_UNITS, DEBUG_DOWN_K_WAVES = 1, 2, 3, 4, 5


def lynx_debug_set(what: int, value: int):
    """Process-wide knob of the library (include/lynx_bench.h): tuning runs and the test of the give-up path."""
    _check(lib().lynx_debug_set(int(what), int(value)))


def lynx_moe_ffn_launches(T, F) -> int:
    """Launches of the weight-streaming kernel per lynx_moe_ffn call (1 or 2) for this batch size and expert width."""
    return int(lib().lynx_moe_ffn_launches(int(T), int(F)))


# ---- FP8 (E4M3) expert weights, weight-only ---------------------------------------------------------------------------

U8 = torch.uint8


class Fp8Weights:
    """Quantised, packed expert weights of one set of experts: codes (uint8) and row scales (fp32)."""

    def __init__(self, Wgu_q, Wd_q, scales_gu, scales_d):
        self.Wgu_q, self.Wd_q, self.scales_gu, self.scales_d = Wgu_q, Wd_q, scales_gu, scales_d


def lynx_quantize_weights_fp8(Wg, Wu, Wd) -> Fp8Weights:
    """Wg, Wu [E,F,H], Wd [E,H,F] bf16 row-major -> Fp8Weights in the streaming layout."""
    E, Fdim, H = Wg.shape
    dev = Wg.device
    Wgu_q = torch.empty((E, Fdim // 16, H // 64, 2, 64, 16), dtype=U8, device=dev)
    Wd_q = torch.empty((E, H // 16, Fdim // 64, 64, 16), dtype=U8, device=dev)
    sgu = torch.empty((E, 2, Fdim), dtype=F32, device=dev)
    sd = torch.empty((E, H), dtype=F32, device=dev)
    _check(lib().lynx_quantize_weights_fp8(_ptr(Wg, BF16, "Wg"), _ptr(Wu, BF16, "Wu"), _ptr(Wd, BF16, "Wd"), E, H, Fdim,
                                           Wgu_q.data_ptr(), Wd_q.data_ptr(), sgu.data_ptr(), sd.data_ptr(), _stream()))
    return Fp8Weights(Wgu_q, Wd_q, sgu, sd)


def _fp8_ptrs(q):
    if q is None:
        return (None, None, None, None)
    return (_ptr(q.Wgu_q, U8, "Wgu_q"), _ptr(q.Wd_q, U8, "Wd_q"), _ptr(q.scales_gu, F32, "scales_gu"),
            _ptr(q.scales_d, F32, "scales_d"))


def lynx_moe_ffn_fp8(x, q, idx, gate, perm_out, N, F, shared=None, n_shared=0, F_shared=0, workspace=None, y=None,
                     stage_events=None, status=None):
    """lynx_moe_ffn with FP8 weights: q, shared = Fp8Weights of the routed / shared experts."""
    T, H = x.shape
    k = idx.shape[1]
    if workspace is None:
        workspace = new_workspace(T, H, F, N, k, n_shared, F_shared, x.device)
    if y is None:
        y = torch.empty((T, H), dtype=F32, device=x.device)
    a, b, c, d = _fp8_ptrs(q)
    sa, sb, sc, sd = _fp8_ptrs(shared)
    ev = None if stage_events is None else (c_void_p * 4)(*[e.cuda_event for e in stage_events])
    _check(lib().lynx_moe_ffn_fp8(_ptr(x, BF16, "x"), a, b, c, d, sa, sb, sc, sd, n_shared, F_shared, _ptr(idx, I32, "idx"),
                                  _ptr(gate, F32, "gate"), _ptr(perm_out["offsets"], I32, "offsets"),
                                  _ptr(perm_out["perm"], I32, "perm"), _ptr(perm_out["active"], I32, "active"),
                                  _ptr(perm_out["num_active"], I32, "num_active"), T, H, F, N, k, _ptr(y, F32, "y"),
                                  _ptr(status, I32, "status"), workspace.data_ptr(), _stream(), ev))
    return y


def lynx_moe_layer_fp8(x, Wr, bias, q, F, k, alpha, beta, enable=1, shared=None, n_shared=0, F_shared=0,
                       buffers: LayerBuffers | None = None, stage_events=None):
    """lynx_moe_layer with FP8 expert weights.  Returns the LayerBuffers."""
    T, H = x.shape
    N = Wr.shape[0]
    b = buffers or LayerBuffers(T, H, F, N, k, beta, n_shared, F_shared, x.device)
    if b.sizes != (T, H, F, N, k, n_shared, F_shared) or b.beta != beta:
        raise ValueError("buffers were allocated for other sizes")
    a_, b_, c_, d_ = _fp8_ptrs(q)
    sa, sb, sc, sd = _fp8_ptrs(shared)
    _check(lib().lynx_moe_layer_fp8(
        _ptr(x, BF16, "x"), _ptr(Wr, F32, "Wr"), _ptr(bias, F32, "bias"), a_, b_, c_, d_, sa, sb, sc, sd, n_shared, F_shared,
        T, H, F, N, k, float(alpha), int(beta), int(enable), b.logits.data_ptr(), b.topk_idx.data_ptr(),
        b.topk_gate.data_ptr(), b.topk_psum.data_ptr(), b.new_idx.data_ptr(), b.new_gate.data_ptr(), b.new_psum.data_ptr(),
        b.cnt_before.data_ptr(), b.cnt_after.data_ptr(), b.bin_hist.data_ptr(), b.num_active.data_ptr(),
        b.offsets.data_ptr(), b.perm.data_ptr(), b.active.data_ptr(), b.num_active_perm.data_ptr(), b.y.data_ptr(), b.status.data_ptr(),
        b.workspace.data_ptr(), _stream(),
        None if stage_events is None else (c_void_p * 4)(*[e.cuda_event for e in stage_events])))
    return b


class Fp4Weights:
    """MXFP4 expert weights of one set of experts in the streaming layout: packed E2M1 codes (uint8) and the
    block-scale exponents (int32 words of four E8M0 bytes)."""

    def __init__(self, Wgu_q, Wd_q, scales_gu, scales_d):
        self.Wgu_q, self.Wd_q, self.scales_gu, self.scales_d = Wgu_q, Wd_q, scales_gu, scales_d


def lynx_quantize_weights_fp4(Wg, Wu, Wd) -> Fp4Weights:
    """Wg, Wu [E,F,H], Wd [E,H,F] bf16 row-major (H, F multiples of 128) -> Fp4Weights."""
    E, Fdim, H = Wg.shape
    dev = Wg.device
    kt4 = lambda K: (K // 128 + 3) // 4
    Wgu_q = torch.empty((E, Fdim // 16, H // 128, 2, 64, 16), dtype=U8, device=dev)
    Wd_q = torch.empty((E, H // 16, Fdim // 128, 64, 16), dtype=U8, device=dev)
    sgu = torch.zeros((E, Fdim // 16, kt4(H), 64, 2), dtype=I32, device=dev)
    sd = torch.zeros((E, H // 32, kt4(Fdim), 64, 2), dtype=I32, device=dev)
    if E and (H % 128 == 0) and (Fdim % 128 == 0):
        assert lib().lynx_fp4_scale_words(E, Fdim, H, 1) == sgu.numel() and lib().lynx_fp4_scale_words(E, H, Fdim, 0) == sd.numel()
    _check(lib().lynx_quantize_weights_fp4(_ptr(Wg, BF16, "Wg"), _ptr(Wu, BF16, "Wu"), _ptr(Wd, BF16, "Wd"), E, H, Fdim,
                                           Wgu_q.data_ptr(), Wd_q.data_ptr(), sgu.data_ptr(), sd.data_ptr(), _stream()))
    return Fp4Weights(Wgu_q, Wd_q, sgu, sd)


def _fp4_ptrs(q):
    if q is None:
        return (None, None, None, None)
    return (_ptr(q.Wgu_q, U8, "Wgu_q"), _ptr(q.Wd_q, U8, "Wd_q"), _ptr(q.scales_gu, I32, "scales_gu"),
            _ptr(q.scales_d, I32, "scales_d"))


def lynx_moe_ffn_fp4(x, q, idx, gate, perm_out, N, F, shared=None, n_shared=0, F_shared=0, workspace=None, y=None,
                     stage_events=None, status=None):
    """lynx_moe_ffn with MXFP4 weights: q, shared = Fp4Weights of the routed / shared experts."""
    T, H = x.shape
    k = idx.shape[1]
    if workspace is None:
        workspace = new_workspace(T, H, F, N, k, n_shared, F_shared, x.device)
    if y is None:
        y = torch.empty((T, H), dtype=F32, device=x.device)
    a, b, c, d = _fp4_ptrs(q)
    sa, sb, sc, sd = _fp4_ptrs(shared)
    ev = None if stage_events is None else (c_void_p * 4)(*[e.cuda_event for e in stage_events])
    _check(lib().lynx_moe_ffn_fp4(_ptr(x, BF16, "x"), a, b, c, d, sa, sb, sc, sd, n_shared, F_shared, _ptr(idx, I32, "idx"),
                                  _ptr(gate, F32, "gate"), _ptr(perm_out["offsets"], I32, "offsets"),
                                  _ptr(perm_out["perm"], I32, "perm"), _ptr(perm_out["active"], I32, "active"),
                                  _ptr(perm_out["num_active"], I32, "num_active"), T, H, F, N, k, _ptr(y, F32, "y"),
                                  _ptr(status, I32, "status"), workspace.data_ptr(), _stream(), ev))
    return y


def lynx_moe_layer_fp4(x, Wr, bias, q, F, k, alpha, beta, enable=1, shared=None, n_shared=0, F_shared=0,
                       buffers: LayerBuffers | None = None, stage_events=None):
    """lynx_moe_layer with MXFP4 expert weights.  Returns the LayerBuffers."""
    T, H = x.shape
    N = Wr.shape[0]
    b = buffers or LayerBuffers(T, H, F, N, k, beta, n_shared, F_shared, x.device)
    if b.sizes != (T, H, F, N, k, n_shared, F_shared) or b.beta != beta:
        raise ValueError("buffers were allocated for other sizes")
    a_, b_, c_, d_ = _fp4_ptrs(q)
    sa, sb, sc, sd = _fp4_ptrs(shared)
    _check(lib().lynx_moe_layer_fp4(
        _ptr(x, BF16, "x"), _ptr(Wr, F32, "Wr"), _ptr(bias, F32, "bias"), a_, b_, c_, d_, sa, sb, sc, sd, n_shared, F_shared,
        T, H, F, N, k, float(alpha), int(beta), int(enable), b.logits.data_ptr(), b.topk_idx.data_ptr(),
        b.topk_gate.data_ptr(), b.topk_psum.data_ptr(), b.new_idx.data_ptr(), b.new_gate.data_ptr(), b.new_psum.data_ptr(),
        b.cnt_before.data_ptr(), b.cnt_after.data_ptr(), b.bin_hist.data_ptr(), b.num_active.data_ptr(),
        b.offsets.data_ptr(), b.perm.data_ptr(), b.active.data_ptr(), b.num_active_perm.data_ptr(), b.y.data_ptr(), b.status.data_ptr(),
        b.workspace.data_ptr(), _stream(),
        None if stage_events is None else (c_void_p * 4)(*[e.cuda_event for e in stage_events])))
    return b
