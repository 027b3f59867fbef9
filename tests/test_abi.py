"""The C-ABI library loads and exports every symbol that include/lynx.h declares; argument checks
that return before any kernel launch behave as documented.  No GPU is needed."""
import ctypes
import os
import re

import pytest

import paper_2411_08982_amd as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if h.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lynx_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = L.lib()
    names = _declared()
    assert set(names) == set(L.SYMBOLS) and len(names) == 28
    for n in names:
        assert getattr(lib, n) is not None


def test_header_limits_match_binding():
    text = open(os.path.join(ROOT, "include", "lynx.h")).read()
    vals = {m[0]: int(m[1]) for m in re.findall(r"#define (LYNX_MAX_[A-Z]+) (\d+)", text)}
    from paper_2411_08982_amd import binding as B
    assert (vals["LYNX_MAX_T"], vals["LYNX_MAX_N"], vals["LYNX_MAX_K"], vals["LYNX_MAX_BETA"]) == (
        B.MAX_T, B.MAX_N, B.MAX_K, B.MAX_BETA)


def test_workspace_bytes_monotone_and_nonnegative():
    a = L.workspace_bytes(16, 512, 1024, 8, 2)
    b = L.workspace_bytes(32, 512, 1024, 8, 2)
    c = L.workspace_bytes(32, 512, 1024, 8, 2, 1, 2048)
    assert 0 < a < b < c
    assert L.workspace_bytes(-1, 512, 1024, 8, 2) == 0
    # h scratch (bf16) + per-pair outputs (fp32) must fit
    assert a >= 16 * 2 * 1024 * 2 + 16 * 2 * 512 * 4


def test_argument_errors_are_reported_before_any_launch():
    lib = L.lib()
    one = ctypes.c_void_p(256)   # never dereferenced: every call below must fail on its size checks
    rc = lib.lynx_route(one, one, None, 4, 64, 4, 8, one, one, one, one, None)           # k > N
    assert rc == -2 and b"lynx_route" in lib.lynx_last_error()
    assert lib.lynx_route(one, one, None, 4, 48, 4, 2, one, one, one, one, None) == -2    # H % 32
    assert lib.lynx_route(one, one, None, -1, 64, 4, 2, one, one, one, one, None) == -1
    assert lib.lynx_route(None, one, None, 4, 64, 4, 2, one, one, one, one, None) == -1
    assert lib.lynx_route(one, one, None, 2000, 64, 4, 2, one, one, one, one, None) == -2  # T > LYNX_MAX_T
    ab = lambda T, N, k, alpha, beta: lib.lynx_affinity_bin(one, one, T, N, k, ctypes.c_float(alpha), beta, 1, one, one, None,
                                                             one, one, one, one, None, None)
    assert ab(4, 8, 2, 1.0, 0) == -1
    assert ab(4, 8, 2, -1.0, 2) == -1
    assert ab(4, 8, 2, float("nan"), 2) == -1
    assert ab(4, 8, 2, float("inf"), 2) == -1
    assert ab(4, 8, 2, 1.0, 7) == -2
    assert ab(4, 300, 2, 1.0, 2) == -2
    abb = lambda gamma: lib.lynx_affinity_bin_biased(one, one, 4, 8, 2, ctypes.c_float(2.0), 2, ctypes.c_float(gamma), 1,
                                                     one, one, None, one, one, one, one, None, None)
    assert abb(-1.0) == -1 and abb(float("nan")) == -1 and abb(float("inf")) == -1
    # group-limited router: n_group divides N, 1 <= topk_group <= n_group, enough experts in the groups, gate_fn 0 / 1
    rg = lambda N, k, G, tg, gf: lib.lynx_route_grouped(one, one, None, 4, 64, N, k, G, tg, gf, one, one, one, one, None)
    assert rg(12, 2, 5, 2, 0) == -1 and b"n_group" in lib.lynx_last_error()
    assert rg(12, 2, 4, 5, 0) == -1 and rg(12, 2, 0, 1, 0) == -1 and rg(12, 2, 4, 0, 0) == -1
    assert rg(12, 4, 4, 1, 0) == -1 and b"fewer than k" in lib.lynx_last_error()
    assert rg(12, 2, 4, 2, 2) == -1 and b"gate_fn" in lib.lynx_last_error()
    assert rg(256, 2, 128, 2, 0) == -2
    abg = lambda N, k, G, tg, beta: lib.lynx_affinity_bin_grouped(one, 4, N, k, G, tg, 0, ctypes.c_float(1.0), beta, 1, one,
                                                                  one, one, one, one, None, one, one, one, one, one, None)
    assert abg(12, 2, 5, 2, 2) == -1 and abg(12, 4, 4, 1, 2) == -1 and abg(12, 2, 4, 2, 0) == -1 and abg(12, 2, 4, 2, 7) == -2
    assert lib.lynx_affinity_bin_grouped(one, 4, 12, 2, 4, 2, 0, ctypes.c_float(1.0), 2, 1, one, one, one, one, one, None, one,
                                         one, one, one, None, None) == -1      # no workspace
    assert lib.lynx_permute(one, 4, 8, 9, one, one, one, one, None) == -2
    assert lib.lynx_permute(one, 4, 0, 1, one, one, one, one, None) == -1
    assert lib.lynx_pack_weights(one, one, one, 2, 48, 64, one, one, None) == -2
    rc = lib.lynx_moe_ffn(one, one, one, None, None, 1, 64, one, one, one, one, one, one, 4, 64, 64, 4, 2, one, None, one, None)
    assert rc == -1 and b"shared" in lib.lynx_last_error()
    assert lib.lynx_moe_ffn(one, one, one, None, None, 0, 0, one, one, one, one, one, one, 4, 64, 72, 4, 2, one, None, one,
                            None) == -2
    # the whole layer checks the FFN's limits before its routing kernels are enqueued: too many shared experts for
    # the completion counters at this batch size (256 + 400 * 8 token blocks > 1024)
    ly = lambda n_shared, T: lib.lynx_moe_layer(one, one, None, one, one, one, one, n_shared, 64, T, 64, 64, 4, 2,
                                                ctypes.c_float(2.0), 2, 1, *([one] * 16), None, one, None, None)
    assert ly(400, 1024) == -2 and b"shared experts" in lib.lynx_last_error()
    assert lib.lynx_debug_set(99, 1) == -1 and lib.lynx_debug_set(1, -1) == 0
    # the entry point on the built-in scratch array refuses sizes that do not fit it, before anything is enqueued
    st = lambda T, H, F, N, k: lib.lynx_moe_layer_static(one, one, None, one, one, None, None, 0, 0, T, H, F, N, k,
                                                         ctypes.c_float(2.0), 2, 1, *([one] * 17), None)
    assert st(1024, 4096, 14336, 8, 2) == -2 and b"scratch" in lib.lynx_last_error()
    assert L.workspace_bytes(512, 2048, 768, 128, 8) <= 64 << 20 < L.workspace_bytes(1024, 4096, 14336, 8, 2)
    assert st(4, 64, 64, 4, 8) == -2 and st(-1, 64, 64, 4, 2) == -1
    assert lib.lynx_residual_add(one, one, 3, one, None) == -1       # odd length
    assert lib.lynx_residual_add(one, None, 4, one, None) == -1
    assert lib.lynx_moe_ffn_launches(8, 14336) == 2 and lib.lynx_moe_ffn_launches(64, 768) == 1
    assert lib.lynx_quantize_weights_fp8(one, one, one, 2, 96, 64, one, one, one, one, None) == -2    # H % 64
    assert lib.lynx_quantize_weights_fp8(one, one, None, 2, 64, 64, one, one, one, one, None) == -1
    assert lib.lynx_read_probe(None, 32, 1, one, None) == -1
    assert lib.lynx_read_probe(one, 24, 1, one, None) == -1          # size not a multiple of 16
    assert lib.lynx_read_probe(one, 0, 1, one, None) == 0            # nothing to read


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    from paper_2411_08982_amd import binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.lib()
