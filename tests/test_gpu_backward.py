"""GPU parity of the backward pass: every step through the C-ABI against the CPU oracle's step on the
same inputs (the oracle step is fed the GPU's outputs of the step before, so each comparison tests one
step), then the final gradients against the oracle's whole chain."""
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
from parity import normwise  # noqa: E402

ALPHA, BETA = 0.005, 0.005
# fp32 sums of up to T products against fp64 (measured: 3e-7 and below); bf16 tensors carry one or two roundings
TOL_F32_SUM = 1e-5


def _say(msg):
    print(msg, flush=True)


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.load()
    return torch


def _forward_backward(cfg, chained=False, dloss=1.0, **kw):
    from paper_2212_05191_amd.runner import GpuLayer
    _say(f"[case] backward {cfg.name}: T={cfg.T} d={cfg.d_model} F={cfg.d_ff} n={cfg.n_groups} m={cfg.m_local} "
         f"C={cfg.capacity} Cg={cfg.group_capacity} {cfg.dtype}/{cfg.act} chained={chained}")
    layer = GpuLayer(cfg, **kw)
    layer.buf.xe.zero_()
    layer.buf.ye.zero_()
    layer.forward()
    layer.prepare_backward(wl.gen_output_grad(cfg))
    for k, v in layer.bwd.__dict__.items():
        v.fill_(-77)
    layer.bwd.dye.zero_()
    layer.bwd.dxe.zero_()
    if chained:
        layer.backward(dloss)
    else:
        layer.backward_steps(dloss)
    return layer


class _LazyExperts:
    """A per-expert gradient tensor [N, ...] left on the device: indexing by expert copies that expert only (the
    weight gradients of a 256-expert configuration are 8 GB as host float32)."""

    def __init__(self, t):
        self.t = t

    def __getitem__(self, e):
        from paper_2212_05191_amd.runner import to_host
        return to_host(self.t[e])


def _fetch_backward(layer, lazy_weight_grads=False):
    import torch
    from paper_2212_05191_amd.runner import to_host
    torch.cuda.synchronize()
    return {k: (_LazyExperts(v) if lazy_weight_grads and k in ("dw1", "dw2") else to_host(v))
            for k, v in layer.bwd.__dict__.items()}


def _check_steps(cfg, layer, dloss=1.0, experts=None):
    """experts: None = compare the expert FFN step on every expert, else on the listed ones."""
    tol = parity.TOL[cfg.dtype]
    fwd = parity.fetch(layer)
    out = _fetch_backward(layer, lazy_weight_grads=experts is not None)
    x, wi, wq, bi, bq = parity.host_inputs(cfg)
    dy = wl.gen_output_grad(cfg)
    n, m, N, Cap = cfg.n_groups, cfg.m_local, cfg.N, cfg.capacity
    g, l, slot, kept = fwd["group_idx"], fwd["local_idx"], fwd["slot"], fwd["kept_count"]
    mask = np.arange(Cap)[None, :] < kept[:, None]
    info = {}

    # combine backward
    dye, dgate = oracle.combine_backward(dy, fwd["ye"], g, l, slot, fwd["gate"].astype(np.float64), m, cfg.dtype)
    info["dye"] = normwise(out["dye"][mask], dye[mask])
    assert info["dye"] <= tol, "dye"
    info["dgate"] = normwise(out["dgate"], dgate)
    assert info["dgate"] <= TOL_F32_SUM, "dgate"
    assert np.all(out["dgate"][slot < 0] == 0), "a dropped token has no gate gradient"

    # route backward
    dlp, dlq = oracle.route_backward(fwd["logits_inter"], fwd["logits_intra"], g, l, out["dgate"].astype(np.float64),
                                     fwd["group_count"], fwd["local_count"], ALPHA, BETA, dloss, bi, bq)
    info["dlp"], info["dlq"] = normwise(out["dlp"], dlp), normwise(out["dlq"], dlq)
    assert info["dlp"] <= TOL_F32_SUM and info["dlq"] <= TOL_F32_SUM, "router logit gradients"

    # expert FFN backward
    es = list(range(N)) if experts is None else list(experts)
    worst = dict(dxe=0.0, dw1=0.0, dw2=0.0)
    for e in es:
        w1, w2 = wl.gen_expert_weights(cfg, e)
        dxe, dw1, dw2 = oracle.expert_ffn_backward(fwd["xe"][e:e + 1], kept[e:e + 1], w1[None], w2[None],
                                                   out["dye"][e:e + 1], cfg.act, cfg.dtype)
        k = int(kept[e])
        if k:
            worst["dxe"] = max(worst["dxe"], normwise(out["dxe"][e, :k], dxe[0, :k]))
            worst["dw1"] = max(worst["dw1"], normwise(out["dw1"][e], dw1[0]))
            worst["dw2"] = max(worst["dw2"], normwise(out["dw2"][e], dw2[0]))
        else:
            assert np.all(out["dw1"][e] == 0) and np.all(out["dw2"][e] == 0), "empty expert: zero weight gradients"
    info.update(worst)
    assert worst["dxe"] <= tol and worst["dw1"] <= tol and worst["dw2"] <= tol, f"expert FFN backward {worst}"

    # dispatch backward
    dx = oracle.dispatch_backward(out["dxe"], g, l, slot, out["dlp"].astype(np.float64), out["dlq"].astype(np.float64),
                                  wi, wq, cfg.dtype)
    info["dx"] = normwise(out["dx"], dx)
    assert info["dx"] <= tol, "dx"

    # router weights backward
    dwi, dwq = oracle.gate_weights_backward(x, out["dlp"].astype(np.float64), out["dlq"].astype(np.float64))
    info["dw_inter"], info["dw_intra"] = normwise(out["dw_inter"], dwi), normwise(out["dw_intra"], dwq)
    assert info["dw_inter"] <= TOL_F32_SUM and info["dw_intra"] <= TOL_F32_SUM, "router weight gradients"
    return fwd, out, info


def _check_end_to_end(cfg, fwd, out, dloss=1.0):
    """The final gradients against the oracle's own chain (forward from the GPU's logits, so that the routing
    decisions are the same; everything after that is the oracle's)."""
    tol = parity.TOL[cfg.dtype]
    x, wi, wq, bi, bq = parity.host_inputs(cfg)
    w1 = np.stack([wl.gen_expert_weights(cfg, e)[0] for e in range(cfg.N)])
    w2 = np.stack([wl.gen_expert_weights(cfg, e)[1] for e in range(cfg.N)])
    f = oracle.layer_forward(x, wi, wq, w1, w2, cfg.capacity, cfg.act, cfg.dtype, ALPHA, BETA, bi, bq,
                             logits=(fwd["logits_inter"], fwd["logits_intra"]), group_capacity=cfg.group_capacity)
    b = oracle.layer_backward(f, x, wi, wq, w1, w2, wl.gen_output_grad(cfg), cfg.act, cfg.dtype, ALPHA, BETA, dloss,
                              bi, bq)
    errs = {k: normwise(out[k], np.asarray(b[k], np.float64)) for k in ("dx", "dw1", "dw2", "dw_inter", "dw_intra")}
    assert all(v <= tol for v in errs.values()), errs
    return errs


BACKWARD_CASES = [
    wl.CONFIGS["cfg1"],
    wl.small_config("bwd_ragged_f32_gelu", 1301, 64, 200, 5, 3, 100, "f32", "gelu", seed=41),
    wl.small_config("bwd_f32_relu_skew", 900, 72, 136, 3, 2, 120, "f32", "relu", skew=True, seed=42),
    wl.small_config("bwd_bf16_gelu", 3000, 192, 320, 3, 4, 200, "bf16", "gelu", seed=43),
    wl.small_config("bwd_bf16_relu_skew", 2500, 128, 448, 4, 8, 90, "bf16", "relu", skew=True, seed=44),
    wl.small_config("bwd_one_token", 1, 64, 64, 2, 2, 1, "bf16", "gelu", seed=45),
    wl.small_config("bwd_capacity_one", 300, 64, 128, 2, 3, 1, "bf16", "gelu", seed=46),
    wl.small_config("bwd_flat", 1500, 128, 128, 1, 12, 100, "bf16", "gelu", seed=47),
    wl.small_config("bwd_group_cap", 1500, 64, 128, 3, 4, 100, "bf16", "gelu", seed=48, group_capacity=300),
    wl.small_config("bwd_empty_experts", 40, 64, 64, 4, 4, 8, "f32", "gelu", seed=49),
    wl.small_config("bwd_bf16_empty_experts", 40, 64, 128, 4, 4, 8, "bf16", "gelu", seed=51),
    # contraction lengths of the weight-gradient GEMMs from 0 to several 64-row slabs with ragged ends
    wl.small_config("bwd_bf16_long_ragged", 4099, 128, 256, 2, 4, 700, "bf16", "gelu", skew=True, seed=52),
    wl.small_config("bwd_f16_gelu", 3000, 192, 320, 3, 4, 200, "f16", "gelu", seed=53),
    wl.small_config("bwd_f16_relu_skew", 2500, 128, 448, 4, 8, 90, "f16", "relu", skew=True, seed=54),
    # wide routers: the matrix-core kernels of the two router-weight products run with 5, 7 and 10 chunks of 16
    # logit columns and 2, 4 and 5 tiles of 32 (d not a multiple of 256, T not a multiple of 64), and the
    # widest case falls back to the vector-ALU kernels
    wl.small_config("bwd_router_40x24", 1100, 192, 128, 40, 24, 9, "bf16", "gelu", seed=56),
    wl.small_config("bwd_router_96x8", 1300, 320, 64, 96, 8, 6, "bf16", "relu", seed=57),
    wl.small_config("bwd_router_flat_129", 1000, 576, 64, 1, 129, 20, "bf16", "gelu", seed=58),
    wl.small_config("bwd_router_flat_200", 900, 64, 64, 1, 200, 12, "bf16", "gelu", seed=59),
]


@pytest.mark.parametrize("cfg", BACKWARD_CASES, ids=lambda c: c.name)
def test_backward_steps_parity(torch_cuda, cfg):
    layer = _forward_backward(cfg, dloss=1.5)
    try:
        fwd, out, info = _check_steps(cfg, layer, dloss=1.5)
        _say(f"   steps {({k: float(f'{v:.2e}') for k, v in info.items()})}")
        errs = _check_end_to_end(cfg, fwd, out, dloss=1.5)
        _say(f"   chain {({k: float(f'{v:.2e}') for k, v in errs.items()})}")
    finally:
        layer.close()


@pytest.mark.parametrize("cfg", [BACKWARD_CASES[1], BACKWARD_CASES[4]], ids=lambda c: c.name)
def test_chained_backward_equals_steps_and_repeats(torch_cuda, cfg):
    a = _forward_backward(cfg)
    b = _forward_backward(cfg, chained=True)
    try:
        oa, ob = _fetch_backward(a), _fetch_backward(b)
        kept = parity.fetch(a)["kept_count"]
        mask = np.arange(cfg.capacity)[None, :] < kept[:, None]
        for k in oa:
            if k in ("dye", "dxe"):
                np.testing.assert_array_equal(oa[k][mask], ob[k][mask], err_msg=k)
            else:
                np.testing.assert_array_equal(oa[k], ob[k], err_msg=k)
        b.backward()
        again = _fetch_backward(b)
        for k in ob:
            np.testing.assert_array_equal(ob[k], again[k], err_msg=f"{k} (repeat)")
    finally:
        a.close()
        b.close()


@pytest.mark.parametrize("cfg", [BACKWARD_CASES[3], BACKWARD_CASES[14], BACKWARD_CASES[16]], ids=lambda c: c.name)
def test_matrix_core_router_gradients_match_the_fma_kernels(torch_cuda, cfg, monkeypatch):
    """dx and the router-weight gradients from the matrix-core kernels (logit gradients as three bf16 planes) against
    the vector-ALU kernels (fp32 FMAs): the fp32 gradients agree to fp32 rounding of the sums, dx to one bf16
    rounding step of the largest element."""
    a = _forward_backward(cfg, chained=True)
    monkeypatch.setenv("SMILE_ROUTER_GRAD_MFMA", "0")
    b = _forward_backward(cfg, chained=True)
    try:
        oa, ob = _fetch_backward(a), _fetch_backward(b)
        for k in ("dw_inter", "dw_intra"):
            err = parity.normwise(oa[k], ob[k].astype(np.float64))
            _say(f"   {k}: {err:.2e}")
            assert err <= 2e-6, (k, err)
        scale = float(np.abs(ob["dx"]).max())
        diff = float(np.abs(oa["dx"].astype(np.float64) - ob["dx"]).max())
        _say(f"   dx: max diff {diff:.3e} (max |dx| {scale:.3e})")
        assert diff <= scale * 2.0 ** -8, (diff, scale)
    finally:
        a.close()
        b.close()


PERSISTENT_CASES = [
    # ragged row tiles, several column tiles
    wl.small_config("persist_ragged", 2600, 320, 448, 2, 3, 500, "bf16", "gelu", seed=61),
    # 130 experts (three 64-expert chunks of the tile walk), many of them empty or nearly so, buffers mostly empty
    wl.small_config("persist_130_experts_skew", 3000, 64, 128, 10, 13, 300, "bf16", "relu", skew=True, seed=62),
    wl.small_config("persist_f16", 1500, 128, 192, 3, 4, 260, "f16", "gelu", seed=63),
    # 520 experts: the walk's per-lane table spans nine chunks of 64 experts
    wl.small_config("persist_520_experts", 4000, 64, 64, 20, 26, 24, "bf16", "gelu", skew=True, seed=65),
    # fewer live tiles than workgroups in the grid
    wl.small_config("persist_few_tiles", 90, 64, 64, 2, 2, 140, "bf16", "gelu", seed=64),
]


@pytest.mark.parametrize("cfg", PERSISTENT_CASES, ids=lambda c: c.name)
def test_persistent_grid_forward_and_backward(torch_cuda, cfg, monkeypatch):
    """The expert GEMMs launched as persistent workgroups that walk the live tiles (normally chosen only for grids
    of many tiles), forced here on small ragged shapes: forward (both paths) and backward against the oracle."""
    monkeypatch.setenv("SMILE_FFN_PERSIST", "1")
    layer = _forward_backward(cfg, dloss=0.7)
    try:
        _say(f"   forward {parity.check_full(cfg, layer)}")
        y_ref = layer.buf.y.clone()
        layer.buf.y.fill_(-1)
        layer.forward_fused()
        torch_cuda.cuda.synchronize()
        assert bool((layer.buf.y == y_ref).all()), "fused forward differs from the materialised one"
        _, _, info = _check_steps(cfg, layer, dloss=0.7)
        _say(f"   steps {({k: float(f'{v:.2e}') for k, v in info.items()})}")
    finally:
        layer.close()


@pytest.mark.parametrize("tile", [0, 1, 2, 3])
def test_every_gradient_gemm_tile_shape(torch_cuda, tile, monkeypatch):
    """Each tile shape of the transposed-operand GEMM on a shape with ragged tiles in every direction."""
    monkeypatch.setenv("SMILE_TGEMM_TILE", str(tile))
    cfg = wl.small_config(f"bwd_tile{tile}", 2600, 320, 448, 2, 3, 500, "bf16", "gelu", seed=55)
    layer = _forward_backward(cfg)
    try:
        _, _, info = _check_steps(cfg, layer)
        _say(f"   {({k: float(f'{v:.2e}') for k, v in info.items()})}")
    finally:
        layer.close()


def test_many_tokens_forward_and_backward(torch_cuda):
    """A long batch (300 000 tokens, over a thousand routing blocks) through the fused forward, the materialised
    forward and the backward pass."""
    cfg = wl.small_config("many_tokens", 300000, 64, 64, 4, 4, 20000, "bf16", "relu", skew=True, seed=56)
    layer = _forward_backward(cfg, chained=True, workers=16)
    try:
        info = parity.check_full(cfg, layer)
        _say(f"   forward {info}")
        assert info["dropped"] > 0
        _, _, steps = _check_steps(cfg, layer)
        _say(f"   backward {({k: float(f'{v:.2e}') for k, v in steps.items()})}")
        y_ref = layer.buf.y.clone()
        layer.buf.y.fill_(-77)
        layer.forward_fused()
        torch_cuda.cuda.synchronize()
        assert bool((layer.buf.y == y_ref).all())
    finally:
        layer.close()


def test_backward_large_aux_coefficients(torch_cuda):
    """Eq. 4 terms large enough to dominate the router gradients (the default 0.005 hides them below the gate term)."""
    from paper_2212_05191_amd.runner import GpuLayer
    cfg = wl.small_config("bwd_aux", 700, 64, 64, 4, 3, 80, "f32", "relu", skew=True, seed=50)
    layer = GpuLayer(cfg, alpha=0.8, beta=0.6)
    try:
        layer.forward()
        dy = np.zeros((cfg.T, cfg.d_model), np.float32)      # no gradient through y: only the loss terms remain
        layer.prepare_backward(dy)
        layer.backward(2.0)
        fwd, out = parity.fetch(layer), _fetch_backward(layer)
        x, wi, wq, bi, bq = parity.host_inputs(cfg)
        assert np.all(out["dgate"] == 0)
        dlp, dlq = oracle.route_backward(fwd["logits_inter"], fwd["logits_intra"], fwd["group_idx"], fwd["local_idx"],
                                         np.zeros(cfg.T), fwd["group_count"], fwd["local_count"], 0.8, 0.6, 2.0, bi, bq)
        assert np.abs(dlp).max() > 0
        assert normwise(out["dlp"], dlp) <= TOL_F32_SUM and normwise(out["dlq"], dlq) <= TOL_F32_SUM
        dwi, dwq = oracle.gate_weights_backward(x, dlp, dlq)
        assert normwise(out["dw_inter"], dwi) <= 5e-5 and normwise(out["dw_intra"], dwq) <= 5e-5
        assert np.all(out["dw1"] == 0) and np.all(out["dw2"] == 0)
    finally:
        layer.close()


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4", "cfg5"])
def test_backward_full_size_sampled(torch_cuda, name):
    """Benchmark configurations at full size: every streaming / router step completely, the expert FFN step
    (every element of dxe, dw1 and dw2 of the expert) on the first, last, fullest and emptiest expert and on
    eight more drawn at random."""
    cfg = wl.CONFIGS[name]
    layer = _forward_backward(cfg, chained=True, workers=16)
    try:
        import torch
        torch.cuda.synchronize()
        kept = layer.buf.kept_count.cpu().numpy()
        picks = {0, cfg.N - 1, int(np.argmax(kept)), int(np.argmin(kept))}
        picks |= set(int(e) for e in np.random.default_rng(7).choice(cfg.N, size=min(8, cfg.N), replace=False))
        picks = sorted(picks)
        _, _, info = _check_steps(cfg, layer, experts=picks)
        _say(f"   {({k: float(f'{v:.2e}') for k, v in info.items()})}")
    finally:
        layer.close()


@pytest.mark.parametrize("cfg", [BACKWARD_CASES[1], BACKWARD_CASES[3], BACKWARD_CASES[4], BACKWARD_CASES[12]],
                         ids=lambda c: c.name)
def test_saved_activations_equal_recomputation(torch_cuda, cfg):
    """Forward pass that also stores h and the pre-activation, backward pass that reads them: the forward
    outputs and every gradient are bit-identical to the path that recomputes them."""
    torch = torch_cuda
    from paper_2212_05191_amd.runner import GpuLayer
    a = _forward_backward(cfg, chained=True)
    _say(f"[case] saved activations {cfg.name}")
    b = GpuLayer(cfg)
    try:
        b.enable_saved_activations()
        b.h_save.fill_(-3)
        b.pre_save.fill_(-3)
        b.buf.xe.zero_()
        b.buf.ye.zero_()
        b.forward()
        b.prepare_backward(wl.gen_output_grad(cfg))
        b.backward()
        fa, fb = parity.fetch(a), parity.fetch(b)
        kept = fa["kept_count"]
        mask = np.arange(cfg.capacity)[None, :] < kept[:, None]
        for k in fa:
            if k in ("xe", "ye"):
                np.testing.assert_array_equal(fa[k][mask], fb[k][mask], err_msg=k)
            else:
                np.testing.assert_array_equal(fa[k], fb[k], err_msg=k)
        ga, gb = _fetch_backward(a), _fetch_backward(b)
        for k in ga:
            if k in ("dye", "dxe"):
                np.testing.assert_array_equal(ga[k][mask], gb[k][mask], err_msg=k)
            else:
                np.testing.assert_array_equal(ga[k], gb[k], err_msg=k)
        # rows beyond kept_count of the saved tensors are not written
        from paper_2212_05191_amd.runner import to_host
        hs, ps = to_host(b.h_save), to_host(b.pre_save)
        assert np.all(hs[~mask] == -3) and np.all(ps[~mask] == -3)
        # h = act(pre) up to the rounding of pre
        ref = np.maximum(ps[mask], 0) if cfg.act == "relu" else None
        if ref is not None:
            np.testing.assert_array_equal(hs[mask], ref)
        # the fused forward (no expert buffers) saves the same tensors
        h_first = b.h_save.clone()
        y_first = b.buf.y.clone()
        b.h_save.fill_(-3)
        b.buf.y.fill_(-77)
        b.forward_fused()
        torch.cuda.synchronize()
        assert bool((b.buf.y == y_first).all())
        m = torch.from_numpy(mask).to(b.h_save.device)
        assert bool((b.h_save[m] == h_first[m]).all())
    finally:
        a.close()
        b.close()
