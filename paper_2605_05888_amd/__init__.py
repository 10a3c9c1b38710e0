"""MI355X-native MoE-layer hot path: thin Python binding over the C-ABI HIP library.

The functions here only marshal arguments (tensor pointers, sizes, the current
HIP stream) into ``libmoe_hub.so``; every step of the path runs in the library's
kernels.  There is no CPU or PyTorch fallback: if the library is missing or a
call fails, an exception is raised.
"""
from .binding import (  # noqa: F401
    MoEHubError, lib_path, load_library, exported_symbols, last_error,
    BF16, F32, SCORE_SOFTMAX_TOPK, SCORE_SIGMOID_TOPK,
    OP_ROUTE, OP_DISPATCH_LAYOUT, OP_GROUPED_FFN,
    workspace_bytes, moe_route, moe_dispatch_layout, moe_dispatch_layout_arrival, moe_dispatch_layout_static,
    moe_route_resolve_arrival,
    moe_permute, moe_grouped_ffn, moe_combine,
    moe_ffn_schedule, moe_ffn_gate_up, moe_ffn_gate_up_gather, moe_ffn_down,
    moe_ffn_down_combine, moe_ffn_status, moe_ffn_gate_up_down,
)
