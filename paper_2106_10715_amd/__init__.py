"""MI355X-native MoE feed-forward layer of CPM-2-MoE: thin Python binding over libmoe355.so.

Every step of the layer runs in the HIP kernels of the C-ABI library; this package only marshals
arguments (torch tensors -> device pointers).  Importing the package is cheap; the first call loads
the shared library and raises if it has not been built (there is no fallback path).
"""
from .binding import (  # noqa: F401
    MOE_BF16, MOE_F32, MoeCfg, MoeError, StreamCtx, lib, lib_path,
    moe_combine, moe_expert_bytes, moe_expert_ffn, moe_layer_forward, moe_pack_weights, moe_permute, moe_permute_static,
    moe_route, moe_workspace_bytes, moe_gate_bytes, moe_pack_gate, moe_layer_forward_timed, Timer, STAGES, TIME_STAGES,
    TIME_UP_KERNEL, moe_schedule_order, moe_plan_slots, moe_stream_slots_that_fit, ORDER_ASCENDING, ORDER_GREEDY, GATE_TOPK, GATE_HASH,
)
