"""MI355X (gfx950) implementation of the batched MoE-layer decode step of Lynx (arXiv 2411.08982).

The product is liblynx.so (hand-written HIP, C ABI in include/lynx.h); this package is its thin
Python binding.  Build with `python -m paper_2411_08982_amd.build`.
"""
from .binding import (LIB_PATH, SYMBOLS, Fp4Weights, Fp8Weights, lynx_moe_ffn_fp4, lynx_moe_layer_fp4, lynx_quantize_weights_fp4, LayerBuffers, LynxError, lynx_moe_ffn_fp8, lynx_moe_layer_fp8,
                      lynx_quantize_weights_fp8, lib, lynx_affinity_bin, lynx_affinity_bin_biased, lynx_moe_ffn, lynx_moe_ffn_launches, lynx_moe_layer, lynx_moe_layer_static,
                      lynx_pack_weights, lynx_permute, lynx_read_probe, lynx_residual_add, lynx_route, new_workspace, workspace_bytes,
                      lynx_route_sigmoid, lynx_affinity_bin_sigmoid, lynx_moe_layer_sigmoid,
                      lynx_route_grouped, lynx_affinity_bin_grouped, lynx_moe_layer_grouped, lynx_debug_set)

__all__ = ["LIB_PATH", "SYMBOLS", "Fp4Weights", "Fp8Weights", "lynx_moe_ffn_fp4", "lynx_moe_layer_fp4", "lynx_quantize_weights_fp4", "LayerBuffers", "LynxError", "lynx_moe_ffn_fp8", "lynx_moe_layer_fp8",
           "lynx_quantize_weights_fp8", "lib", "lynx_affinity_bin", "lynx_affinity_bin_biased", "lynx_moe_ffn", "lynx_moe_ffn_launches",
           "lynx_moe_layer", "lynx_moe_layer_static", "lynx_pack_weights", "lynx_permute", "lynx_read_probe", "lynx_residual_add", "lynx_route", "new_workspace", "workspace_bytes",
           "lynx_route_sigmoid", "lynx_affinity_bin_sigmoid", "lynx_moe_layer_sigmoid",
           "lynx_route_grouped", "lynx_affinity_bin_grouped", "lynx_moe_layer_grouped", "lynx_debug_set"]
