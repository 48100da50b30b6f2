"""MI355X-native forward path of SMILE's bi-level routed MoE layer (arXiv 2212.05191).

`binding` wraps the C-ABI library built from csrc/ (HIP, gfx950); `workloads`
holds the seeded synthetic inputs.  There is no CPU fallback: calling the
binding without the built library raises.
"""
from . import workloads  # noqa: F401
