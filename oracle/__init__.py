"""CPU oracle of the SMILE bi-level MoE layer (forward pass and its derivative) (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the HIP library.
"""
from .oracle import (  # noqa: F401
    build,
    capacity,
    gate_logits,
    route,
    slots_two_stage,
    dispatch,
    dispatch_stage1,
    dispatch_stage2,
    expert_ffn,
    combine,
    aux_loss,
    layer_forward,
    combine_backward,
    route_backward,
    expert_ffn_backward,
    dispatch_backward,
    gate_weights_backward,
    layer_backward,
    threads,
    RouteResult,
)
