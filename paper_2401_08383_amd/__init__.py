"""MI355X (gfx950) implementation of the single-GPU hot path of context-coherent MoE inference
with inter-layer expert affinity: the expert layer (gate, dispatch, expert FFN, combine) and the
affinity statistic (co-routing counts, conditional probabilities, placement locality).

The work is done by hand-written HIP kernels in ``libexflow_moe.so`` (C ABI in
``include/exflow_moe.h``); this package is only the ctypes binding over it.
"""
from .binding import (  # noqa: F401
    EXF_ACT_GELU_ERF,
    EXF_ACT_GELU_TANH,
    EXF_BF16,
    EXF_F32,
    ExflowError,
    LIB_PATH,
    SIGNATURES,
    affinity_histogram,
    affinity_multihop,
    affinity_statistics,
    check_placement,
    comm_volume,
    last_error,
    lib,
    moe_combine,
    moe_dispatch,
    moe_dispatch_static,
    moe_expert_ffn,
    moe_expert_ffn_fused,
    moe_gate_topk,
    moe_topk_from_logits,
    placement_locality,
    placement_locality_from_counts,
    placement_search,
    routing_transfers,
    transfer_ratios,
)
