"""MI355X-native MoE layer share: route -> dispatch -> expert FFN -> combine.

Thin Python binding over the C-ABI library `libmoe.so` (hand-written HIP for
gfx950).  PyTorch only provides device memory and streams; every step of the
path runs in the library's kernels.  Importing works without a GPU; calling an
entry point without the built library raises.
"""
from .binding import (MoEConfig, MoEError, lib_path, load_library, moe_combine, moe_dispatch,
                      moe_dispatch_noalloc, moe_dispatch_noalloc_max_bytes,
                      moe_combine_stage, moe_dispatch_shard, moe_expert_ffn, moe_expert_ffn_fp8act,
                      moe_fp8act_workspace_bytes, moe_quant_act, moe_dispatch_fp8q, moe_expert_ffn_fp8q,
                      moe_route, moe_workspace_bytes, moe_status_string,
                      moe_profile_enable, moe_profile_read, moe_profile_filter, moe_probe_mfma_rate,
                      MOE_F32, MOE_BF16, MOE_FP8_E4M3_B128, MOE_SCORE_SOFTMAX, MOE_SCORE_SIGMOID)
from .layer import MoELayerShare

__all__ = ["MoEConfig", "MoEError", "MoELayerShare", "lib_path", "load_library", "moe_route",
           "moe_dispatch", "moe_dispatch_noalloc", "moe_dispatch_noalloc_max_bytes", "moe_dispatch_shard", "moe_expert_ffn", "moe_combine",
           "moe_combine_stage", "moe_workspace_bytes", "moe_expert_ffn_fp8act",
           "moe_fp8act_workspace_bytes", "moe_quant_act", "moe_dispatch_fp8q", "moe_expert_ffn_fp8q",
           "moe_status_string", "moe_profile_enable", "moe_profile_read", "moe_profile_filter", "moe_probe_mfma_rate", "MOE_F32", "MOE_BF16", "MOE_FP8_E4M3_B128",
           "MOE_SCORE_SOFTMAX", "MOE_SCORE_SIGMOID"]
