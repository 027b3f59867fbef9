"""CPU oracle of the Lynx MoE decode layer -- TEST INFRASTRUCTURE, not the product.

Thin ctypes wrapper around ``lynx_oracle.c`` (plain C, fp64).  Only the tests, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this package; the HIP path never does, and this
package never imports the HIP path.  What each function computes, and which passage of the paper
(arXiv 2411.08982) it follows, is stated in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_float, c_int, c_int32, c_uint16, c_uint64

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lynx_oracle.c")
_LIB = os.path.join(_HERE, "liblynx_oracle.so")

OK = 0
ERR_INVALID_ARG = -1
ERR_UNSUPPORTED = -2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-shared",
               "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p, f32p, f64p, i32p, u64p = (POINTER(c_uint16), POINTER(c_float), POINTER(c_double), POINTER(c_int32),
                                        POINTER(c_uint64))
        u8p = POINTER(ctypes.c_uint8)
        lib.orc_num_threads.restype = c_int
        lib.orc_route.argtypes = [u16p, f32p, f32p, c_int, c_int, c_int, c_int, f32p, i32p, f64p, f64p]
        lib.orc_topk.argtypes = [f32p, c_int, c_int, c_int, i32p, f64p, f64p]
        lib.orc_topk_sigmoid.argtypes = [f32p, c_int, c_int, c_int, i32p, f64p, f64p]
        lib.orc_sigmoid_gates.argtypes = [f32p, i32p, c_int, c_int, c_int, f64p, f64p]
        lib.orc_selection_mass.argtypes = [f32p, i32p, c_int, c_int, c_int, f64p]
        lib.orc_selection_mass.restype = c_int
        lib.orc_group_allowed.argtypes = [f32p, c_int, c_int, c_int, c_int, u8p]
        lib.orc_topk_grouped.argtypes = [f32p, c_int, c_int, c_int, c_int, c_int, c_int, i32p, f64p, f64p]
        lib.orc_affinity_bin_grouped.argtypes = [f32p, i32p, c_int, c_int, c_int, c_int, c_int, c_float, c_int, c_int, i32p,
                                                 f64p, i32p, i32p, i32p, i32p, i32p]
        lib.orc_affinity_bin.argtypes = [f32p, i32p, c_int, c_int, c_int, c_float, c_int, c_int, i32p, f64p, i32p,
                                         i32p, i32p, i32p, i32p, u64p, i32p]
        lib.orc_affinity_bin_biased.argtypes = [f32p, i32p, c_int, c_int, c_int, c_float, c_int, c_float, c_int, i32p,
                                                f64p, i32p, i32p, i32p, i32p, f32p]
        lib.orc_permute.argtypes = [i32p, c_int, c_int, c_int, i32p, i32p, i32p, i32p]
        lib.orc_moe_ffn.argtypes = [u16p, u16p, u16p, u16p, u16p, u16p, u16p, c_int, c_int, i32p, f64p, c_int, c_int,
                                    c_int, c_int, c_int, f64p]
        lib.orc_e4m3_decode.argtypes = [ctypes.c_uint8]
        lib.orc_e4m3_decode.restype = c_double
        lib.orc_e4m3_encode.argtypes = [c_float]
        lib.orc_e4m3_encode.restype = ctypes.c_uint8
        lib.orc_quantize_rows_e4m3.argtypes = [u16p, ctypes.c_long, c_int, u8p, f32p]
        lib.orc_e2m1_decode.argtypes = [ctypes.c_uint8]
        lib.orc_e2m1_decode.restype = c_double
        lib.orc_e2m1_encode.argtypes = [c_float]
        lib.orc_e2m1_encode.restype = ctypes.c_uint8
        lib.orc_quantize_mxfp4.argtypes = [u16p, ctypes.c_long, c_int, u8p, u8p]
        lib.orc_dequantize_mxfp4.argtypes = [u8p, u8p, ctypes.c_long, c_int, u16p]
        lib.orc_quantize_rows_e4m3.restype = c_int
        lib.orc_moe_ffn_q8.argtypes = [u16p, u8p, u8p, u8p, f32p, f32p, f32p, u8p, u8p, u8p, f32p, f32p, f32p, c_int, c_int,
                                       i32p, f64p, c_int, c_int, c_int, c_int, c_int, f64p]
        lib.orc_moe_ffn_q8.restype = c_int
        for f in (lib.orc_route, lib.orc_topk, lib.orc_topk_sigmoid, lib.orc_sigmoid_gates, lib.orc_affinity_bin,
                  lib.orc_affinity_bin_biased, lib.orc_permute, lib.orc_moe_ffn):
            f.restype = c_int
        _lib = lib
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where} returned {code}")
        self.code = code


def _p(a, ctype):
    if a is None:
        return ctypes.cast(None, POINTER(ctype))
    return a.ctypes.data_as(POINTER(ctype))


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().orc_num_threads())


def route(x_bf16, Wr, bias, k):
    """x_bf16 [T,H] uint16 (bf16 bits), Wr [N,H] f32, bias [N] f32 or None.
    Returns dict(logits f32 [T,N], idx i32 [T,k], gate f64 [T,k], psum f64 [T])."""
    x = _arr(x_bf16, np.uint16)
    Wr = _arr(Wr, np.float32)
    T, H = x.shape
    N = Wr.shape[0]
    assert Wr.shape[1] == H
    b = None if bias is None else _arr(bias, np.float32)
    logits = np.zeros((T, N), np.float32)
    idx = np.zeros((T, k), np.int32)
    gate = np.zeros((T, k), np.float64)
    psum = np.zeros((T,), np.float64)
    rc = _load().orc_route(_p(x, c_uint16), _p(Wr, c_float), _p(b, c_float), T, H, N, k, _p(logits, c_float),
                           _p(idx, c_int32), _p(gate, c_double), _p(psum, c_double))
    if rc != OK:
        raise OracleError(rc, "orc_route")
    return dict(logits=logits, idx=idx, gate=gate, psum=psum)


def topk(logits, k):
    """Softmax + top-k from given fp32 logits [T,N].  Returns dict(idx, gate f64, psum f64)."""
    z = _arr(logits, np.float32)
    T, N = z.shape
    idx = np.zeros((T, k), np.int32)
    gate = np.zeros((T, k), np.float64)
    psum = np.zeros((T,), np.float64)
    rc = _load().orc_topk(_p(z, c_float), T, N, k, _p(idx, c_int32), _p(gate, c_double), _p(psum, c_double))
    if rc != OK:
        raise OracleError(rc, "orc_topk")
    return dict(idx=idx, gate=gate, psum=psum)


def selection_mass(logits, idx):
    """Share of the softmax over all experts held by the selection idx [T,k] (entries outside [0,N) skipped): f64 [T]."""
    z = _arr(logits, np.float32)
    idx = _arr(idx, np.int32)
    T, N = z.shape
    psum = np.zeros((T,), np.float64)
    rc = _load().orc_selection_mass(_p(z, c_float), _p(idx, c_int32), T, N, idx.shape[1], _p(psum, c_double))
    if rc != OK:
        raise OracleError(rc, "orc_selection_mass")
    return psum


def topk_sigmoid(logits, k):
    """Sigmoid-gated router: top-k by logit, gates = selected sigmoid scores / their sum.
    Returns dict(idx, gate f64, ssum f64 = sum of the selected scores)."""
    z = _arr(logits, np.float32)
    T, N = z.shape
    idx = np.zeros((T, k), np.int32)
    gate = np.zeros((T, k), np.float64)
    ssum = np.zeros((T,), np.float64)
    rc = _load().orc_topk_sigmoid(_p(z, c_float), T, N, k, _p(idx, c_int32), _p(gate, c_double), _p(ssum, c_double))
    if rc != OK:
        raise OracleError(rc, "orc_topk_sigmoid")
    return dict(idx=idx, gate=gate, ssum=ssum)


def sigmoid_gates(logits, idx):
    """Gates of a given selection idx [T,k] under a sigmoid-gated router.  Returns (gate f64 [T,k], ssum f64 [T])."""
    z = _arr(logits, np.float32)
    idx = _arr(idx, np.int32)
    T, N = z.shape
    k = idx.shape[1]
    gate = np.zeros((T, k), np.float64)
    ssum = np.zeros((T,), np.float64)
    rc = _load().orc_sigmoid_gates(_p(z, c_float), _p(idx, c_int32), T, N, k, _p(gate, c_double), _p(ssum, c_double))
    if rc != OK:
        raise OracleError(rc, "orc_sigmoid_gates")
    return gate, ssum


def affinity_bin_sigmoid(logits, topk_idx, alpha, beta, enable=1):
    """AffinityBinning under a sigmoid-gated router: bins, scores, nominations and remap exactly as affinity_bin (they
    use logit differences only); the gates of the new selection are the sigmoid scores over their sum."""
    a = affinity_bin(logits, topk_idx, alpha, beta, enable)
    a["new_gate"], a["new_psum"] = sigmoid_gates(logits, a["new_idx"])   # the sum of the new selection's scores
    return a


def group_allowed(logits, n_group, topk_group):
    """Group-limited routers: allow [T,N] (0/1), the experts of each token's topk_group best groups (group score =
    largest logit in the group, ties to the lower group)."""
    z = _arr(logits, np.float32)
    T, N = z.shape
    allow = np.zeros((T, N), np.uint8)
    rc = _load().orc_group_allowed(_p(z, c_float), T, N, int(n_group), int(topk_group), _p(allow, ctypes.c_uint8))
    if rc != OK:
        raise OracleError(rc, "orc_group_allowed")
    return allow


def topk_grouped(logits, k, n_group, topk_group, gate_fn=0):
    """Group-limited top-k.  gate_fn 0: softmax gates, third = selected share of the softmax over all experts;
    1: sigmoid gates, third = sum of the selected scores.  Returns dict(idx, gate f64, third f64)."""
    z = _arr(logits, np.float32)
    T, N = z.shape
    idx = np.zeros((T, k), np.int32)
    gate = np.zeros((T, k), np.float64)
    third = np.zeros((T,), np.float64)
    rc = _load().orc_topk_grouped(_p(z, c_float), T, N, k, int(n_group), int(topk_group), int(gate_fn), _p(idx, c_int32),
                                  _p(gate, c_double), _p(third, c_double))
    if rc != OK:
        raise OracleError(rc, "orc_topk_grouped")
    return dict(idx=idx, gate=gate, third=third)


def affinity_bin_grouped(logits, topk_idx, n_group, topk_group, alpha, beta, enable=1, gate_fn=0):
    """AffinityBinning for a group-limited router: every token stays inside its own groups.  topk_idx is the selection
    of topk_grouped.  Returns dict with new_idx, new_gate (f64), cnt_before, cnt_after, bin_hist, num_active, active."""
    z = _arr(logits, np.float32)
    idx = _arr(topk_idx, np.int32)
    T, N = z.shape
    k = idx.shape[1]
    nb = max(int(beta), 1)
    new_idx = np.zeros((T, k), np.int32)
    new_gate = np.zeros((T, k), np.float64)
    cnt_before = np.zeros((N,), np.int32)
    cnt_after = np.zeros((N,), np.int32)
    bin_hist = np.zeros((N, nb), np.int32)
    num_active = np.zeros((2,), np.int32)
    active = np.zeros((N,), np.int32)
    rc = _load().orc_affinity_bin_grouped(_p(z, c_float), _p(idx, c_int32), T, N, k, int(n_group), int(topk_group),
                                          float(alpha), int(beta), int(enable), _p(new_idx, c_int32),
                                          _p(new_gate, c_double), _p(cnt_before, c_int32), _p(cnt_after, c_int32),
                                          _p(bin_hist, c_int32), _p(num_active, c_int32), _p(active, c_int32))
    if rc != OK:
        raise OracleError(rc, "orc_affinity_bin_grouped")
    new_third = selection_mass(z, new_idx)
    if gate_fn:
        new_gate, new_third = sigmoid_gates(z, new_idx)
    return dict(new_idx=new_idx, new_gate=new_gate, new_psum=new_third, cnt_before=cnt_before, cnt_after=cnt_after, bin_hist=bin_hist,
                num_active=num_active, active=active)


def affinity_bin(logits, topk_idx, alpha, beta, enable=1):
    """logits [T,N] f32, topk_idx [T,k] i32.  Returns dict with new_idx, new_gate (f64), cnt_before,
    cnt_after, bin_hist [N,beta], num_active [2], and the diagnostics q [T,N], score [N] (uint64),
    active [N] (0/1)."""
    z = _arr(logits, np.float32)
    idx = _arr(topk_idx, np.int32)
    T, N = z.shape
    k = idx.shape[1]
    assert idx.shape[0] == T
    nb = max(int(beta), 1)
    new_idx = np.zeros((T, k), np.int32)
    new_gate = np.zeros((T, k), np.float64)
    cnt_before = np.zeros((N,), np.int32)
    cnt_after = np.zeros((N,), np.int32)
    bin_hist = np.zeros((N, nb), np.int32)
    num_active = np.zeros((2,), np.int32)
    q = np.zeros((T, N), np.int32)
    score = np.zeros((N,), np.uint64)
    active = np.zeros((N,), np.int32)
    rc = _load().orc_affinity_bin(_p(z, c_float), _p(idx, c_int32), T, N, k, float(alpha), int(beta), int(enable),
                                  _p(new_idx, c_int32), _p(new_gate, c_double), _p(cnt_before, c_int32),
                                  _p(cnt_after, c_int32), _p(bin_hist, c_int32), _p(num_active, c_int32),
                                  _p(q, c_int32), _p(score, c_uint64), _p(active, c_int32))
    if rc != OK:
        raise OracleError(rc, "orc_affinity_bin")
    return dict(new_idx=new_idx, new_gate=new_gate, new_psum=selection_mass(z, new_idx), cnt_before=cnt_before,
                cnt_after=cnt_after, bin_hist=bin_hist, num_active=num_active, q=q, score=score, active=active)


def affinity_bin_biased(logits, topk_idx, alpha, beta, gamma, enable=1):
    """Score-biased selection (the variant of Sec. 3.3.1 that adds the batch score to the logits).  Returns dict
    with new_idx, new_gate (f64), cnt_before, cnt_after, bin_hist [N,beta], num_active [2], bias [N] (f32)."""
    z = _arr(logits, np.float32)
    idx = _arr(topk_idx, np.int32)
    T, N = z.shape
    k = idx.shape[1]
    assert idx.shape[0] == T
    nb = max(int(beta), 1)
    new_idx = np.zeros((T, k), np.int32)
    new_gate = np.zeros((T, k), np.float64)
    cnt_before = np.zeros((N,), np.int32)
    cnt_after = np.zeros((N,), np.int32)
    bin_hist = np.zeros((N, nb), np.int32)
    num_active = np.zeros((2,), np.int32)
    bias = np.zeros((N,), np.float32)
    rc = _load().orc_affinity_bin_biased(_p(z, c_float), _p(idx, c_int32), T, N, k, float(alpha), int(beta), float(gamma),
                                         int(enable), _p(new_idx, c_int32), _p(new_gate, c_double),
                                         _p(cnt_before, c_int32), _p(cnt_after, c_int32), _p(bin_hist, c_int32),
                                         _p(num_active, c_int32), _p(bias, c_float))
    if rc != OK:
        raise OracleError(rc, "orc_affinity_bin_biased")
    return dict(new_idx=new_idx, new_gate=new_gate, new_psum=selection_mass(z, new_idx), cnt_before=cnt_before,
                cnt_after=cnt_after, bin_hist=bin_hist, num_active=num_active, bias=bias)


def permute(idx, N):
    """idx [T,k] i32.  Returns dict(offsets [N+1], perm [T*k], active [N], num_active [1])."""
    idx = _arr(idx, np.int32)
    T, k = idx.shape
    offsets = np.zeros((N + 1,), np.int32)
    perm = np.zeros((T * k,), np.int32)
    active = np.zeros((N,), np.int32)
    num_active = np.zeros((1,), np.int32)
    rc = _load().orc_permute(_p(idx, c_int32), T, N, k, _p(offsets, c_int32), _p(perm, c_int32), _p(active, c_int32),
                             _p(num_active, c_int32))
    if rc != OK:
        raise OracleError(rc, "orc_permute")
    return dict(offsets=offsets, perm=perm, active=active, num_active=num_active)


def moe_ffn(x_bf16, Wg, Wu, Wd, idx, gate, Sg=None, Su=None, Sd=None):
    """x_bf16 [T,H]; Wg, Wu [N,F,H]; Wd [N,H,F]; optional shared Sg, Su [S,Fs,H], Sd [S,H,Fs] (all uint16
    bf16 bits); idx [T,k] i32; gate [T,k] f64.  Returns y [T,H] f64."""
    x = _arr(x_bf16, np.uint16)
    Wg, Wu, Wd = _arr(Wg, np.uint16), _arr(Wu, np.uint16), _arr(Wd, np.uint16)
    idx = _arr(idx, np.int32)
    gate = _arr(gate, np.float64)
    T, H = x.shape
    N, F, H2 = Wg.shape
    assert H2 == H and Wu.shape == (N, F, H) and Wd.shape == (N, H, F)
    k = idx.shape[1]
    assert idx.shape == (T, k) and gate.shape == (T, k)
    if Sg is not None and len(Sg) > 0:
        Sg, Su, Sd = _arr(Sg, np.uint16), _arr(Su, np.uint16), _arr(Sd, np.uint16)
        S, Fs, _ = Sg.shape
        assert Su.shape == (S, Fs, H) and Sd.shape == (S, H, Fs)
    else:
        Sg = Su = Sd = None
        S, Fs = 0, 0
    y = np.zeros((T, H), np.float64)
    rc = _load().orc_moe_ffn(_p(x, c_uint16), _p(Wg, c_uint16), _p(Wu, c_uint16), _p(Wd, c_uint16), _p(Sg, c_uint16),
                             _p(Su, c_uint16), _p(Sd, c_uint16), S, Fs, _p(idx, c_int32), _p(gate, c_double), T, H, F,
                             N, k, _p(y, c_double))
    if rc != OK:
        raise OracleError(rc, "orc_moe_ffn")
    return y


def moe_layer(x_bf16, Wr, bias, Wg, Wu, Wd, k, alpha, beta, enable=1, Sg=None, Su=None, Sd=None):
    """The whole decode step: route -> affinity_bin -> permute -> FFN + combine."""
    r = route(x_bf16, Wr, bias, k)
    a = affinity_bin(r["logits"], r["idx"], alpha, beta, enable)
    p = permute(a["new_idx"], Wr.shape[0])
    y = moe_ffn(x_bf16, Wg, Wu, Wd, a["new_idx"], a["new_gate"], Sg, Su, Sd)
    return dict(route=r, bin=a, permute=p, y=y)


# ---- expert weights in FP8 E4M3, weight-only ------------------------------------------------------------------------

def e4m3_decode(codes):
    """uint8 codes (any shape) -> float64 values (NaN for the two NaN codes)."""
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    lib = _load()
    return np.array([lib.orc_e4m3_decode(int(v)) for v in c.ravel()], np.float64).reshape(c.shape)


def e4m3_encode(values):
    """float32 values (any shape) -> nearest E4M3 codes (ties to even, saturating at +-448)."""
    v = np.ascontiguousarray(values, dtype=np.float32)
    lib = _load()
    return np.array([lib.orc_e4m3_encode(float(x)) for x in v.ravel()], np.uint8).reshape(v.shape)


def quantize_rows_e4m3(W_bf16):
    """bf16 bits [..., K] -> (codes uint8 [..., K], scales float32 [...]): one scale per row, scale = amax / 448."""
    W = _arr(W_bf16, np.uint16)
    K = W.shape[-1]
    rows = W.size // K
    codes = np.zeros(W.shape, np.uint8)
    scales = np.zeros(W.shape[:-1], np.float32)
    rc = _load().orc_quantize_rows_e4m3(_p(W, c_uint16), rows, K, codes.ctypes.data_as(POINTER(ctypes.c_uint8)),
                                        _p(scales, c_float))
    if rc != OK:
        raise OracleError(rc, "orc_quantize_rows_e4m3")
    return codes, scales


def moe_ffn_q8(x_bf16, Qg, Qu, Qd, sg, su, sd, idx, gate, SQg=None, SQu=None, SQd=None, ssg=None, ssu=None, ssd=None):
    """moe_ffn with E4M3 weights: codes Qg, Qu [N,F,H], Qd [N,H,F] and scales sg, su [N,F], sd [N,H] (shared likewise)."""
    x = _arr(x_bf16, np.uint16)
    T, H = x.shape
    N, F, _ = Qg.shape
    idx = _arr(idx, np.int32)
    k = idx.shape[1]
    gate = _arr(gate, np.float64)
    u8 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.uint8)
    f32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.float32)
    Qg, Qu, Qd, SQg, SQu, SQd = (u8(a) for a in (Qg, Qu, Qd, SQg, SQu, SQd))
    sg, su, sd, ssg, ssu, ssd = (f32(a) for a in (sg, su, sd, ssg, ssu, ssd))
    n_shared, F_shared = (0, 0) if SQg is None else (SQg.shape[0], SQg.shape[1])
    pu8 = lambda a: None if a is None else a.ctypes.data_as(POINTER(ctypes.c_uint8))
    pf = lambda a: None if a is None else _p(a, c_float)
    y = np.zeros((T, H), np.float64)
    rc = _load().orc_moe_ffn_q8(_p(x, c_uint16), pu8(Qg), pu8(Qu), pu8(Qd), pf(sg), pf(su), pf(sd), pu8(SQg), pu8(SQu),
                                pu8(SQd), pf(ssg), pf(ssu), pf(ssd), n_shared, F_shared, _p(idx, c_int32),
                                _p(gate, c_double), T, H, F, N, k, _p(y, c_double))
    if rc != OK:
        raise OracleError(rc, "orc_moe_ffn_q8")
    return y


def e2m1_decode(codes):
    """4-bit E2M1 codes (uint8, low nibble; any shape) -> float64 values."""
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    lib = _load()
    return np.array([lib.orc_e2m1_decode(int(v)) for v in c.ravel()], np.float64).reshape(c.shape)


def e2m1_encode(values):
    """float32 values (any shape) -> nearest E2M1 codes (ties to the even code, saturating at +-6)."""
    v = np.ascontiguousarray(values, dtype=np.float32)
    lib = _load()
    return np.array([lib.orc_e2m1_encode(float(x)) for x in v.ravel()], np.uint8).reshape(v.shape)


def quantize_mxfp4(W_bf16):
    """bf16 bits [..., K] (K a multiple of 32) -> (codes uint8 [..., K], one E2M1 code per byte; scale exponents
    uint8 [..., K/32], E8M0): per block of 32, E - 127 = floor(log2(amax)) - 2."""
    W = _arr(W_bf16, np.uint16)
    K = W.shape[-1]
    rows = W.size // K
    codes = np.zeros(W.shape, np.uint8)
    scales = np.zeros(W.shape[:-1] + (K // 32,), np.uint8)
    u8p = lambda a: a.ctypes.data_as(POINTER(ctypes.c_uint8))
    rc = _load().orc_quantize_mxfp4(_p(W, c_uint16), rows, K, u8p(codes), u8p(scales))
    if rc != OK:
        raise OracleError(rc, "orc_quantize_mxfp4")
    return codes, scales


def dequantize_mxfp4(codes, scales):
    """(codes [..., K], scale exponents [..., K/32]) -> the bf16 bits of decode(code) * 2^(E - 127), exactly."""
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    s = np.ascontiguousarray(scales, dtype=np.uint8)
    K = c.shape[-1]
    rows = c.size // K
    W = np.zeros(c.shape, np.uint16)
    u8p = lambda a: a.ctypes.data_as(POINTER(ctypes.c_uint8))
    rc = _load().orc_dequantize_mxfp4(u8p(c), u8p(s), rows, K, _p(W, c_uint16))
    if rc != OK:
        raise OracleError(rc, "orc_dequantize_mxfp4")
    return W


def moe_ffn_q4(x_bf16, Qg, Qu, Qd, eg, eu, ed, idx, gate, SQg=None, SQu=None, SQd=None, seg=None, seu=None, sed=None):
    """moe_ffn with MXFP4 weights (codes Q*, scale exponents e*; shared experts SQ*, se*): the dequantised weights
    are bf16 numbers, so this is moe_ffn over them."""
    dq = dequantize_mxfp4
    shared = (None, None, None) if SQg is None else (dq(SQg, seg), dq(SQu, seu), dq(SQd, sed))
    return moe_ffn(x_bf16, dq(Qg, eg), dq(Qu, eu), dq(Qd, ed), idx, gate, *shared)
