"""smile_route_bilevel_static (the routing step with its scratch memory in a fixed device array inside the
library: no ctx, no allocation) against smile_route_bilevel, through the C-ABI, on two calls in a row, the second
with a smaller input, so that whatever the first call left in the shared array is still there."""
import os
import sys

import numpy as np
import pytest

import oracle
from paper_2212_05191_amd import binding as B
from paper_2212_05191_amd import workloads as wl

pytestmark = pytest.mark.gpu

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity  # noqa: E402

ROUTE_OUTPUTS = ("group_idx", "local_idx", "pos_in_group", "slot", "gate", "p_top", "q_top", "group_count",
                 "local_count", "expert_count", "kept_count", "p_sum", "q_sum")


def _route_both_ways(torch, cfg):
    from paper_2212_05191_amd.runner import GpuLayer, to_host
    print(f"[case] static routing {cfg.name}: T={cfg.T} n={cfg.n_groups} m={cfg.m_local} C={cfg.capacity} "
          f"Cg={cfg.group_capacity}", flush=True)
    layer = GpuLayer(cfg)
    try:
        b = layer.buf
        layer.gate_logits()
        for k in ROUTE_OUTPUTS:
            getattr(b, k).fill_(-77)
        layer.route()                                   # the existing entry point (ctx workspace)
        torch.cuda.synchronize()
        want = {k: to_host(getattr(b, k)).copy() for k in ROUTE_OUTPUTS}
        for k in ROUTE_OUTPUTS:
            getattr(b, k).fill_(-55)
        B.smile_route_bilevel_static(layer.desc, b.logits_inter, b.logits_intra, layer.bias_inter, layer.bias_intra,
                                     b.group_idx, b.local_idx, b.pos_in_group, b.slot, b.gate, b.p_top, b.q_top,
                                     b.group_count, b.local_count, b.expert_count, b.kept_count, b.p_sum, b.q_sum)
        torch.cuda.synchronize()
        got = {k: to_host(getattr(b, k)) for k in ROUTE_OUTPUTS}
        for k in ROUTE_OUTPUTS:   # same kernels, fixed summation order: identical bits, floats included
            np.testing.assert_array_equal(got[k], want[k], err_msg=k)
        # and against the oracle on the same logits
        bi, bq = wl.gen_routing_biases(cfg)
        r = oracle.route(to_host(b.logits_inter), to_host(b.logits_intra), cfg.capacity, bi, bq, cfg.group_capacity)
        for k in ("group_idx", "local_idx", "pos_in_group", "slot", "group_count", "local_count", "expert_count",
                  "kept_count"):
            np.testing.assert_array_equal(got[k], getattr(r, k), err_msg=k)
        for k in ("gate", "p_top", "q_top", "p_sum", "q_sum"):
            np.testing.assert_allclose(got[k], getattr(r, k), rtol=1e-5, err_msg=k)
    finally:
        layer.close()


def test_static_scratch_routing_two_calls_in_a_row():
    import torch
    assert torch.cuda.is_available(), "needs the MI355X"
    B.load()
    big = wl.small_config("static_big", 40000, 64, 64, 8, 8, 500, "bf16", "gelu", skew=True, seed=41)
    small = wl.small_config("static_small", 2900, 64, 64, 3, 4, 200, "bf16", "gelu", skew=True, seed=42)
    capped = wl.small_config("static_group_cap", 5000, 64, 64, 4, 8, 120, "bf16", "gelu", skew=True, seed=43,
                             group_capacity=900)
    _route_both_ways(torch, big)
    _route_both_ways(torch, small)      # smaller than the call before: stale histograms of 157 blocks lie behind its 12
    _route_both_ways(torch, capped)     # the group-capacity kernels use the same array
    # a shape whose routing scratch exceeds the fixed array is refused before anything is enqueued
    huge = B.make_desc(1 << 22, 64, 64, 32, 8, 20000, "bf16", "gelu")
    t = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    with pytest.raises(B.SmileError) as ei:
        B.smile_route_bilevel_static(huge, *([t] * 17))
    assert ei.value.status == B.WORKSPACE
