"""Stage-wise comparison of the HIP path with the CPU oracle on the same seeded inputs.

Protocol (handles tokens whose two best logits are nearly tied, where an ulp of difference in the
logits would legitimately flip the routing):
  (i)   GPU logits vs oracle logits, norm-wise tolerance;
  (ii)  oracle routing run on the GPU's logits: every integer output must be bit-identical, floats
        within tolerance;
  (iii) oracle dispatch / expert FFN / combine / loss from that routing vs the GPU's buffers
        (dispatch is a copy: bit-exact);
  (iv)  oracle run fully independently: tokens routed differently must all be near-ties.

Tolerances (norm-wise, max|a-b| / max|b| per tensor): 1e-5 in fp32, 2e-2 in bf16, 4e-3 in fp16 (8 units of
its 2^-11 rounding error: the same few roundings as bf16 with 8 times finer steps).  Gate logits: 1e-5 in every
storage type -- both sides multiply the same rounded inputs and differ only in the accumulation (fp32 on the
matrix cores, fp64 in the oracle).
"""
from __future__ import annotations

import numpy as np

import oracle
from paper_2212_05191_amd import workloads as wl
from paper_2212_05191_amd.runner import GpuLayer, to_host

TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 4e-3}
TOL_LOGITS = 1e-5
NEAR_TIE = 1e-4


def normwise(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    if a.size == 0:
        return 0.0
    return float(np.max(np.abs(a - b)) / max(float(np.max(np.abs(b))), 1e-30))


def host_inputs(cfg):
    x = wl.gen_tokens(cfg)
    wi, wq = wl.gen_router_weights(cfg)
    bi, bq = wl.gen_routing_biases(cfg)
    return x, wi, wq, bi, bq


def fetch(layer: GpuLayer) -> dict:
    import torch
    torch.cuda.synchronize()
    return {k: to_host(v) for k, v in layer.buf.__dict__.items()}


def check_logits_and_routing(cfg, out, x, wi, wq, bi, bq):
    """Stages (i), (ii) and (iv).  Returns the oracle routing computed from the GPU's logits."""
    li, lq = oracle.gate_logits(x, wi, wq)
    assert normwise(out["logits_inter"], li) <= TOL_LOGITS, "inter logits"
    assert normwise(out["logits_intra"], lq) <= TOL_LOGITS, "intra logits"

    r = oracle.route(out["logits_inter"], out["logits_intra"], cfg.capacity, bi, bq, cfg.group_capacity)
    for name in ("group_idx", "local_idx", "pos_in_group", "slot", "group_count", "local_count",
                 "expert_count", "kept_count"):
        np.testing.assert_array_equal(out[name], getattr(r, name), err_msg=name)
    # probabilities: fp32 on the GPU, fp64 in the oracle; 1e-5 relative per element in either dtype
    for name in ("gate", "p_top", "q_top"):
        np.testing.assert_allclose(out[name], getattr(r, name), rtol=1e-5, atol=0, err_msg=name)
    np.testing.assert_allclose(out["p_sum"], r.p_sum, rtol=1e-5, err_msg="p_sum")
    np.testing.assert_allclose(out["q_sum"], r.q_sum, rtol=1e-5, err_msg="q_sum")
    loss = oracle.aux_loss(r.group_count, r.local_count, r.p_sum, r.q_sum, cfg.T, 0.005, 0.005)
    np.testing.assert_allclose(out["loss3"], loss, rtol=1e-5, err_msg="loss")

    # (iv) independent oracle run: differences only at near-ties
    ri = oracle.route(li, lq, cfg.capacity, bi, bq, cfg.group_capacity)
    diff = np.nonzero((ri.group_idx != r.group_idx) | (ri.local_idx != r.local_idx))[0]
    for t in diff:
        a = li[t] + (bi if bi is not None else 0)
        top2 = np.sort(a)[-2:] if a.size > 1 else np.array([0.0, 1.0])
        if ri.group_idx[t] != r.group_idx[t]:
            assert top2[1] - top2[0] < NEAR_TIE, f"token {t}: group differs without a near-tie"
        else:
            c = lq[t] + (bq[r.group_idx[t]] if bq is not None else 0)
            top2 = np.sort(c)[-2:]
            assert top2[1] - top2[0] < NEAR_TIE, f"token {t}: local expert differs without a near-tie"
    return r, len(diff)


def check_dispatch_exact(cfg, out, x, r):
    xe_ref = oracle.dispatch(x, r.group_idx, r.local_idx, r.slot, cfg.n_groups, cfg.m_local, cfg.capacity)
    mask = np.arange(cfg.capacity)[None, :] < r.kept_count[:, None]
    np.testing.assert_array_equal(out["xe"][mask], xe_ref[mask], err_msg="xe (dispatch must be a bit-exact copy)")
    return xe_ref


def check_full(cfg, layer: GpuLayer):
    """Element-by-element parity of every output (sizes the oracle finishes in seconds)."""
    tol = TOL[cfg.dtype]
    out = fetch(layer)
    x, wi, wq, bi, bq = host_inputs(cfg)
    r, nflip = check_logits_and_routing(cfg, out, x, wi, wq, bi, bq)
    xe_ref = check_dispatch_exact(cfg, out, x, r)
    w1 = np.stack([wl.gen_expert_weights(cfg, e)[0] for e in range(cfg.N)])
    w2 = np.stack([wl.gen_expert_weights(cfg, e)[1] for e in range(cfg.N)])
    ye_ref = oracle.expert_ffn(xe_ref, r.kept_count, w1, w2, cfg.act, cfg.dtype)
    mask = np.arange(cfg.capacity)[None, :] < r.kept_count[:, None]
    assert normwise(out["ye"][mask], ye_ref[mask]) <= tol, "ye"
    y_ref = oracle.combine(ye_ref, r.group_idx, r.local_idx, r.slot, r.gate, cfg.m_local, cfg.dtype)
    assert normwise(out["y"], y_ref) <= tol, "y"
    assert np.all(out["y"][r.slot < 0] == 0), "dropped tokens must give zero rows"
    return dict(flips=nflip, kept=int(r.kept_count.sum()), dropped=int((r.slot < 0).sum()),
                err_ye=normwise(out["ye"][mask], ye_ref[mask]), err_y=normwise(out["y"], y_ref))


def check_full_streamed(cfg, layer: GpuLayer, workers=8):
    """check_full for the full-size configurations: every row of ye and y against the oracle, with the expert
    weights regenerated one expert at a time (a thread pool draws them ahead while the oracle, itself running on
    all host threads, works on the expert before), so that host memory stays at a few experts' weights.
    Returns the summary and the oracle's y, for comparing other paths that must produce the same output."""
    from concurrent.futures import ThreadPoolExecutor
    tol = TOL[cfg.dtype]
    out = fetch(layer)
    x, wi, wq, bi, bq = host_inputs(cfg)
    r, nflip = check_logits_and_routing(cfg, out, x, wi, wq, bi, bq)
    xe_ref = check_dispatch_exact(cfg, out, x, r)
    ye_ref = np.zeros_like(xe_ref)
    worst_e, diff_max, ref_max = 0.0, 0.0, 0.0
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for e, (w1, w2) in enumerate(pool.map(lambda e: wl.gen_expert_weights(cfg, e), range(cfg.N))):
            k = int(r.kept_count[e])
            if k == 0:
                continue
            ref = oracle.expert_ffn(xe_ref[e:e + 1, :k], [k], w1[None], w2[None], cfg.act, cfg.dtype)[0]
            ye_ref[e, :k] = ref
            got = out["ye"][e, :k]
            err = normwise(got, ref)
            worst_e = max(worst_e, err)
            assert err <= tol, f"ye of expert {e} ({k} rows): {err}"
            diff_max = max(diff_max, float(np.max(np.abs(got.astype(np.float64) - ref))))
            ref_max = max(ref_max, float(np.max(np.abs(ref))))
    y_ref = oracle.combine(ye_ref, r.group_idx, r.local_idx, r.slot, r.gate, cfg.m_local, cfg.dtype)
    err_y = normwise(out["y"], y_ref)
    assert err_y <= tol, f"y: {err_y}"
    assert np.all(out["y"][r.slot < 0] == 0), "dropped tokens must give zero rows"
    info = dict(flips=nflip, kept=int(r.kept_count.sum()), dropped=int((r.slot < 0).sum()),
                err_ye=diff_max / max(ref_max, 1e-30), err_ye_worst_expert=worst_e, err_y=err_y)
    return info, y_ref, r


def check_sampled(cfg, layer: GpuLayer, experts_to_sample=6, rows_per_expert=24, seed=0):
    """Full-size configurations: routing and dispatch compared completely, the FFN / combine on rows
    the oracle computes one by one (first / last / tile-boundary / random rows of the fullest,
    emptiest, first, last and random experts)."""
    tol = TOL[cfg.dtype]
    out = fetch(layer)
    x, wi, wq, bi, bq = host_inputs(cfg)
    r, nflip = check_logits_and_routing(cfg, out, x, wi, wq, bi, bq)
    check_dispatch_exact(cfg, out, x, r)
    assert np.all(out["y"][r.slot < 0] == 0), "dropped tokens must give zero rows"

    rng = np.random.default_rng(seed)
    nonempty = np.nonzero(r.kept_count > 0)[0]
    picks = {int(nonempty[0]), int(nonempty[-1]), int(nonempty[np.argmax(r.kept_count[nonempty])]),
             int(nonempty[np.argmin(r.kept_count[nonempty])])}
    while len(picks) < min(experts_to_sample, len(nonempty)):
        picks.add(int(rng.choice(nonempty)))
    e_of_t = r.group_idx * cfg.m_local + r.local_idx
    worst_ye = worst_y = 0.0
    for e in sorted(picks):
        k = int(r.kept_count[e])
        cand = {0, k - 1, k // 2, 31, 32, 63, 64, 127, 128, 255, 256, k - 2}
        rows = sorted(c for c in cand if 0 <= c < k)
        extra = rng.choice(k, size=min(k, rows_per_expert), replace=False)
        rows = sorted(set(rows) | set(int(v) for v in extra))[:max(rows_per_expert, 12)]
        w1, w2 = wl.gen_expert_weights(cfg, e)
        xs = out["xe"][e, rows][None]                       # already verified bit-exact against x
        ye_ref = oracle.expert_ffn(xs, [len(rows)], w1[None], w2[None], cfg.act, cfg.dtype)[0]
        err = normwise(out["ye"][e, rows], ye_ref)
        worst_ye = max(worst_ye, err)
        assert err <= tol, f"ye of expert {e}: {err}"
        # the tokens sitting in those rows
        toks = np.nonzero((e_of_t == e) & np.isin(r.slot, rows))[0]
        order = np.argsort(r.slot[toks])
        toks = toks[order]
        assert len(toks) == len(rows)
        y_ref = oracle.combine(ye_ref[None], np.zeros(len(rows), np.int32), np.zeros(len(rows), np.int32),
                               np.arange(len(rows), dtype=np.int32), r.gate[toks], 1, cfg.dtype)
        err = normwise(out["y"][toks], y_ref)
        worst_y = max(worst_y, err)
        assert err <= tol, f"y of expert {e}: {err}"
    return dict(flips=nflip, kept=int(r.kept_count.sum()), dropped=int((r.slot < 0).sum()),
                err_ye=worst_ye, err_y=worst_y, experts=sorted(picks))
