"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on the same seeded
inputs.  Small / medium shapes and the four full-size benchmark configurations are compared element by
element (every routing output, every kept row of xe, ye and y); the extra full-size workloads completely for
routing and dispatch and on sampled rows for the expert FFN / combine.
"""
import dataclasses
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


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.load()
    return torch


def _run(cfg, forward="steps", **kw):
    from paper_2212_05191_amd.runner import GpuLayer
    _say(f"[case] {cfg.name}: T={cfg.T} d={cfg.d_model} F={cfg.d_ff} n={cfg.n_groups} m={cfg.m_local} "
         f"C={cfg.capacity} {cfg.dtype}/{cfg.act} skew={cfg.skew} forward={forward}")
    layer = GpuLayer(cfg, **kw)
    # poison the outputs so that an unwritten element cannot pass by luck
    for k, v in layer.buf.__dict__.items():
        if k not in ("xe", "ye"):
            v.fill_(-77)
    layer.buf.xe.zero_()
    layer.buf.ye.zero_()
    if forward == "steps":
        layer.forward_steps()
    elif forward == "fused":
        layer.forward_fused()
    elif forward != "none":
        layer.forward()
    return layer


SMALL = [
    wl.CONFIGS["cfg1"],
    wl.small_config("ragged_f32_relu", 777, 72, 136, 3, 5, 37, "f32", "relu", seed=11),
    wl.small_config("ragged_f32_gelu", 1301, 64, 200, 5, 3, 100, "f32", "gelu", seed=12),
    wl.small_config("mid_bf16_gelu", 3000, 192, 320, 3, 4, 200, "bf16", "gelu", seed=13),
    wl.small_config("mid_bf16_relu_skew", 2500, 128, 448, 4, 8, 90, "bf16", "relu", skew=True, seed=14),
    wl.small_config("one_token", 1, 64, 64, 2, 2, 1, "bf16", "gelu", seed=15),
    wl.small_config("capacity_one", 300, 64, 128, 2, 3, 1, "bf16", "gelu", seed=16),
    wl.small_config("single_group", 600, 64, 128, 1, 6, 80, "bf16", "gelu", seed=17),
    wl.small_config("single_local", 600, 64, 128, 6, 1, 80, "f32", "gelu", seed=18),
    wl.small_config("one_expert_dense", 200, 128, 256, 1, 1, 200, "bf16", "gelu", seed=19),
    wl.small_config("many_groups", 5000, 64, 64, 40, 24, 9, "bf16", "relu", seed=20),
    # flat one-level routers (Section 2, Eq. 1-2 with k = 1): more than 128 logit columns -> two gate passes
    wl.small_config("flat_switch_200", 6000, 128, 128, 1, 200, 40, "bf16", "gelu", seed=24),
    wl.small_config("flat_switch_t_130", 3000, 64, 64, 130, 1, 30, "bf16", "relu", seed=25),
    # the largest expert count the library accepts (N = 4096), capacity far above the load, fp32 with wider layers
    wl.small_config("max_experts", 20000, 64, 64, 64, 64, 8, "bf16", "gelu", seed=27),
    wl.small_config("capacity_above_T", 700, 128, 192, 2, 2, 1000, "bf16", "gelu", seed=28),
    wl.small_config("f32_wider", 2100, 256, 512, 3, 3, 250, "f32", "gelu", seed=29),
    # a first-hop buffer per group as well (Section 3.2.3): tight, tight with skewed groups over many routing
    # blocks, and too loose to matter
    wl.small_config("group_cap_f32", 1500, 64, 128, 3, 4, 100, "f32", "relu", seed=30, group_capacity=300),
    wl.small_config("group_cap_bf16_skew", 6000, 128, 192, 4, 8, 150, "bf16", "gelu", skew=True, seed=31,
                    group_capacity=1100),
    wl.small_config("group_cap_loose", 900, 64, 64, 2, 3, 120, "bf16", "gelu", seed=32, group_capacity=900),
    wl.small_config("group_cap_one_row", 300, 64, 64, 5, 2, 4, "bf16", "relu", seed=33, group_capacity=1),
    # half precision, the precision the paper trains in (Section 4.1)
    wl.small_config("mid_f16_gelu", 3000, 192, 320, 3, 4, 200, "f16", "gelu", seed=34),
    wl.small_config("f16_relu_skew_group_cap", 2500, 128, 448, 4, 8, 90, "f16", "relu", skew=True, seed=35,
                    group_capacity=800),
    wl.small_config("f16_flat_200", 4000, 64, 128, 1, 200, 30, "f16", "gelu", seed=36),
    # 2928 counters per histogram copy: too many for one copy per wave beside the probability tile in 64 KB of LDS
    wl.small_config("wide_router_48x60", 12000, 64, 64, 48, 60, 9, "bf16", "gelu", seed=38),
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: c.name)
def test_small_shapes_full_parity(torch_cuda, cfg):
    layer = _run(cfg)
    try:
        info = parity.check_full(cfg, layer)
        _say(f"   {info}")
    finally:
        layer.close()


@pytest.mark.parametrize("cfg", [SMALL[3], SMALL[17]], ids=lambda c: c.name)
def test_chained_entry_point_equals_step_by_step(torch_cuda, cfg):
    a = _run(cfg, "steps")
    b = _run(cfg, "chained", own_workspace=True)
    try:
        oa, ob = parity.fetch(a), parity.fetch(b)
        for k in oa:
            if k in ("xe", "ye"):
                continue        # rows beyond kept_count are unspecified
            np.testing.assert_array_equal(oa[k], ob[k], err_msg=k)
        parity.check_full(cfg, b)
    finally:
        a.close()
        b.close()


FUSED_CASES = [SMALL[0], SMALL[1], SMALL[3], SMALL[4], SMALL[5], SMALL[6], SMALL[10], SMALL[16], SMALL[17], SMALL[19],
               SMALL[20], SMALL[21],
               wl.small_config("fused_ragged", 4099, 128, 256, 4, 8, 100, "bf16", "gelu", skew=True, seed=26)]


@pytest.mark.parametrize("cfg", FUSED_CASES, ids=lambda c: c.name)
def test_fused_entry_point_equals_step_by_step(torch_cuda, cfg):
    """smile_layer_forward without expert buffers (gather / scatter fused into the GEMMs) gives the same
    bits as the six separate calls, and its y matches the oracle."""
    a = _run(cfg, "steps")
    b = _run(cfg, "fused")
    try:
        oa, ob = parity.fetch(a), parity.fetch(b)
        for k in oa:
            if k in ("xe", "ye"):
                continue        # not produced by the fused path
            np.testing.assert_array_equal(oa[k], ob[k], err_msg=k)
        parity.check_full(cfg, a)
    finally:
        a.close()
        b.close()


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "cfg5"])
def test_full_size_configs_every_row_and_fused_path(torch_cuda, name):
    """The four full-size bf16 configurations: every routing output, every kept row of xe (bit-exact), ye and y
    of the chained forward pass against the oracle; then the buffer-free forward pass (the one bench.py times:
    gather and gate-weighted scatter inside the expert GEMMs) -- its y against the ORACLE's y to the same
    tolerance, its routing outputs and loss bit-identical to the chained pass."""
    from paper_2212_05191_amd.runner import to_host
    cfg = wl.get_config(name)
    a = _run(cfg, "chained", workers=16)
    try:
        info, y_ref, r = parity.check_full_streamed(cfg, a)
        _say(f"   chained: {info}")
        if name == "cfg5":
            assert info["dropped"] > cfg.T // 10, "the skewed configuration must drop many tokens"
        y_chained = a.buf.y.clone()
        loss_ref = a.buf.loss3.clone()
        slot_ref = a.buf.slot.clone()
        a.buf.y.fill_(-77)
        a.buf.slot.fill_(-77)
        a.buf.loss3.fill_(-77)
        a.forward_fused()
        torch_cuda.cuda.synchronize()
        y_fused = to_host(a.buf.y)
        err = parity.normwise(y_fused, y_ref)
        _say(f"   fused: err_y {err:.2e} against the oracle")
        assert err <= parity.TOL[cfg.dtype], f"fused forward y against the oracle: {err}"
        assert np.all(y_fused[r.slot < 0] == 0), "fused forward: dropped tokens must give zero rows"
        assert bool((a.buf.y == y_chained).all()), "fused and chained forward passes differ"
        assert bool((a.buf.slot == slot_ref).all()) and bool((a.buf.loss3 == loss_ref).all()), name
    finally:
        a.close()


@pytest.mark.parametrize("cfg", [SMALL[3], SMALL[16], SMALL[17]], ids=lambda c: c.name)
def test_two_hop_dispatch(torch_cuda, cfg):
    """The dispatch as the two hops of Section 3.2.3 through a materialised group buffer: hop 1 against the
    oracle's, hop 2 against the one-hop move (bit-exact copies)."""
    torch = torch_cuda
    layer = _run(cfg)
    try:
        out = parity.fetch(layer)
        x = parity.host_inputs(cfg)[0]
        rows = cfg.group_capacity if cfg.group_capacity else int(out["group_count"].max())
        b = layer.buf
        xg = torch.full((cfg.n_groups, rows, cfg.d_model), -5.0, dtype=layer.x.dtype, device=layer.x.device)
        xe2 = torch.full_like(b.xe, -9.0)
        B.smile_dispatch_hop1(layer.ctx, layer.x, b.group_idx, b.pos_in_group, rows, xg)
        B.smile_dispatch_hop2(layer.ctx, xg, b.group_idx, b.local_idx, b.pos_in_group, b.slot, rows, xe2)
        torch.cuda.synchronize()
        from paper_2212_05191_amd.runner import to_host
        want = oracle.dispatch_stage1(x, out["group_idx"], out["pos_in_group"], cfg.n_groups, rows, fill=-5.0)
        np.testing.assert_array_equal(to_host(xg), want)
        mask = np.arange(cfg.capacity)[None, :] < out["kept_count"][:, None]
        got = to_host(xe2)
        np.testing.assert_array_equal(got[mask], out["xe"][mask])
        assert np.all(got[~mask] == -9.0), "rows beyond kept_count must stay untouched"
        want2 = oracle.dispatch_stage2(want, out["group_idx"], out["local_idx"], out["pos_in_group"], out["slot"],
                                       cfg.m_local, cfg.capacity, fill=-9.0)
        np.testing.assert_array_equal(got, want2)
        # a group buffer that is too short drops the late tokens at hop 1 and never reads beyond it at hop 2
        short = max(1, rows // 2)
        xg_s = torch.full((cfg.n_groups, short, cfg.d_model), -5.0, dtype=layer.x.dtype, device=layer.x.device)
        B.smile_dispatch_hop1(layer.ctx, layer.x, b.group_idx, b.pos_in_group, short, xg_s)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(
            to_host(xg_s), oracle.dispatch_stage1(x, out["group_idx"], out["pos_in_group"], cfg.n_groups, short, fill=-5.0))
        with pytest.raises(B.SmileError):
            B.smile_dispatch_hop1(layer.ctx, layer.x, b.group_idx, b.pos_in_group, 0, xg)
    finally:
        layer.close()


def test_repeated_calls_are_bit_identical(torch_cuda):
    cfg = wl.small_config("determinism", 4099, 128, 256, 4, 8, 100, "bf16", "gelu", skew=True, seed=21)
    layer = _run(cfg)
    try:
        first = parity.fetch(layer)
        for _ in range(3):
            layer.forward()
            again = parity.fetch(layer)
            for k in first:
                np.testing.assert_array_equal(first[k], again[k], err_msg=k)
    finally:
        layer.close()


def test_work_runs_on_the_callers_stream(torch_cuda):
    """Every entry point enqueues on the stream it is given: a forward + backward pass issued on a side stream
    (default priority) behind a long-running kernel of that stream gives the same bits as on the default stream."""
    torch = torch_cuda
    cfg = wl.small_config("side_stream", 3000, 128, 256, 3, 4, 300, "bf16", "gelu", skew=True, seed=37)
    a = _run(cfg, "chained")
    a.prepare_backward(wl.gen_output_grad(cfg))
    a.backward()
    b = _run(cfg, "none")
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            # something long in front: if the library launched on another stream it would race with the fill below
            big = torch.empty(256 << 20, dtype=torch.uint8, device=b.x.device)
            for _ in range(4):
                big.fill_(1)
            b.buf.y.fill_(-77)
            b.forward_steps()
            b.prepare_backward(wl.gen_output_grad(cfg))
            b.backward_steps()
        side.synchronize()
        oa, ob = parity.fetch(a), parity.fetch(b)
        kept = oa["kept_count"]
        mask = np.arange(cfg.capacity)[None, :] < kept[:, None]
        for k in oa:
            if k in ("xe", "ye"):
                np.testing.assert_array_equal(oa[k][mask], ob[k][mask], err_msg=k)
            else:
                np.testing.assert_array_equal(oa[k], ob[k], err_msg=k)
        from paper_2212_05191_amd.runner import to_host
        for k in ("dx", "dw1", "dw2", "dw_inter", "dw_intra", "dgate"):
            np.testing.assert_array_equal(to_host(getattr(a.bwd, k)), to_host(getattr(b.bwd, k)), err_msg=k)
    finally:
        a.close()
        b.close()


def test_kernel_timing_leaves_results_unchanged(torch_cuda):
    """smile_kernel_timing: every kernel of a call takes a caller-owned event pair; the outputs keep their bits,
    the reported kernels are the call's launches in order, and each pair yields a positive duration."""
    import ctypes
    torch = torch_cuda
    cfg = wl.small_config("timing", 5000, 128, 256, 3, 4, 450, "bf16", "gelu", skew=True, seed=39)
    layer = _run(cfg, "fused")
    try:
        lib = B.load()
        hip = ctypes.CDLL("libamdhip64.so")
        hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        first = parity.fetch(layer)
        evs = []
        for _ in range(16):
            e = ctypes.c_void_p()
            assert hip.hipEventCreate(ctypes.byref(e)) == 0
            evs.append(e)
        arr = (ctypes.c_void_p * 16)(*[e.value for e in evs])
        assert lib.smile_kernel_timing(layer.ctx.handle, arr, 8) == 0
        layer.forward_fused()
        n = lib.smile_kernel_timing_count(layer.ctx.handle)
        names = [lib.smile_kernel_timing_name(layer.ctx.handle, i).decode() for i in range(n)]
        torch.cuda.synchronize()
        _say(f"   kernels: {names}")
        assert 4 <= n <= 6 and "gate_logits" in names[0] and sum("grouped_gemm" in k for k in names) == 2
        for i in range(n):
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), evs[2 * i], evs[2 * i + 1]) == 0
            assert 0.0 < ms.value < 50.0, (names[i], ms.value)
        again = parity.fetch(layer)
        for k in first:
            if k not in ("xe", "ye"):
                np.testing.assert_array_equal(first[k], again[k], err_msg=k)
        # detached: the next call takes no events and gives the same bits
        assert lib.smile_kernel_timing(layer.ctx.handle, None, 0) == 0
        layer.forward_fused()
        assert lib.smile_kernel_timing_count(layer.ctx.handle) == 0
        third = parity.fetch(layer)
        np.testing.assert_array_equal(first["y"], third["y"])
        for e in evs:
            hip.hipEventDestroy(e)
    finally:
        layer.close()


def test_expert_biases(torch_cuda):
    """Optional b1 / b2 of the expert FFN (NULL in the benchmark configurations)."""
    torch = torch_cuda
    from paper_2212_05191_amd.runner import GpuLayer, to_device, to_host
    for dtype in ("f32", "bf16"):
        cfg = wl.small_config(f"biases_{dtype}", 500, 64, 192, 2, 2, 150, dtype, "gelu", seed=22)
        _say(f"[case] {cfg.name}")
        layer = GpuLayer(cfg)
        rng = np.random.default_rng(5)
        b1 = wl.quantize(rng.standard_normal((cfg.N, cfg.d_ff)).astype(np.float32), dtype)
        b2 = wl.quantize(rng.standard_normal((cfg.N, cfg.d_model)).astype(np.float32), dtype)
        layer.b1, layer.b2 = to_device(b1, dtype), to_device(b2, dtype)
        layer.buf.ye.zero_()
        layer.forward_steps()
        out = parity.fetch(layer)
        x, wi, wq, bi, bq = parity.host_inputs(cfg)
        r, _ = parity.check_logits_and_routing(cfg, out, x, wi, wq, bi, bq)
        xe = parity.check_dispatch_exact(cfg, out, x, r)
        w1 = np.stack([wl.gen_expert_weights(cfg, e)[0] for e in range(cfg.N)])
        w2 = np.stack([wl.gen_expert_weights(cfg, e)[1] for e in range(cfg.N)])
        ye = oracle.expert_ffn(xe, r.kept_count, w1, w2, cfg.act, dtype, b1, b2)
        mask = np.arange(cfg.capacity)[None, :] < r.kept_count[:, None]
        assert parity.normwise(out["ye"][mask], ye[mask]) <= parity.TOL[dtype]
        layer.close()


@pytest.mark.parametrize("tile,dtype", [(t, "bf16") for t in range(7)] + [(0, "f16"), (2, "f16"), (6, "f16")])
def test_every_ffn_tile_shape(torch_cuda, tile, dtype, monkeypatch):
    """Each MFMA tile shape of the grouped GEMM, on a shape with ragged row and column tiles."""
    monkeypatch.setenv("SMILE_FFN_TILE", str(tile))
    cfg = wl.small_config(f"tile{tile}_{dtype}", 4000, 320, 448, 2, 3, 600, dtype, "gelu", seed=23)
    layer = _run(cfg)
    try:
        _say(f"   {parity.check_full(cfg, layer)}")
    finally:
        layer.close()


@pytest.mark.parametrize("name", ["t2_48b", "cfg5_group_cap", "cfg2_f16"])
def test_extra_full_size_workloads_sampled_parity(torch_cuda, name):
    """Workloads beyond the five benchmark configurations, at full size: routing and dispatch completely, the
    expert FFN / combine on sampled rows."""
    if name == "cfg5_group_cap":
        # cfg5 with a first-hop buffer of 1.25 x the mean group load: its Zipf-skewed groups overflow it
        cfg = dataclasses.replace(wl.get_config("cfg5"), name=name, group_capacity=2560)
    else:
        cfg = wl.get_config(name)
    layer = _run(cfg, "chained", workers=16)
    try:
        info = parity.check_sampled(cfg, layer)
        _say(f"   {info}")
    finally:
        layer.close()
