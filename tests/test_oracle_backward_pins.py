"""Pins of the oracle's backward pass against things other than itself: automatic differentiation of
an independently written fp64 model of the layer (torch CPU ops), central finite differences of the
oracle's own forward pass, and closed forms of single steps.  No GPU."""
import numpy as np
import pytest
import torch

import oracle


def _case(seed, T=40, d=8, F=12, n=3, m=2, C=9, scale=1.0):
    rng = np.random.default_rng(seed)
    f = lambda *s: (scale * rng.standard_normal(s)).astype(np.float32)
    return dict(x=f(T, d), wi=f(n, d), wq=f(m, d), w1=0.5 * f(n * m, F, d), w2=0.5 * f(n * m, d, F),
                dy=f(T, d), bi=0.3 * f(n), bq=0.3 * f(n, m), C=C)


def _torch_model(c, act, alpha, beta, dloss, with_bias):
    """The layer written again with torch fp64 ops; returns autograd's gradients of
    L = <dy, y> + dloss * (alpha * inter + beta * intra)."""
    t64 = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    x, wi, wq, w1, w2 = (t64(c[k]) for k in ("x", "wi", "wq", "w1", "w2"))
    dy = torch.tensor(c["dy"].astype(np.float64))
    T, n, m, C = x.shape[0], wi.shape[0], wq.shape[0], c["C"]
    a = x @ wi.T
    if with_bias:
        a = a + torch.tensor(c["bi"].astype(np.float64))
    p = torch.softmax(a, dim=1)
    g = torch.argmax(a, dim=1)
    cl = x @ wq.T
    if with_bias:
        cl = cl + torch.tensor(c["bq"].astype(np.float64))[g]
    q = torch.softmax(cl, dim=1)
    l = torch.argmax(cl, dim=1)
    e = g * m + l
    onehot = torch.nn.functional.one_hot(e, n * m)
    rank = (torch.cumsum(onehot, 0) - onehot)[torch.arange(T), e]
    kept = rank < C
    gate = p[torch.arange(T), g] * q[torch.arange(T), l]
    pre = torch.einsum("tk,tfk->tf", x, w1[e])
    h = torch.relu(pre) if act == "relu" else torch.nn.functional.gelu(pre)
    out = torch.einsum("tf,tcf->tc", h, w2[e])
    y = torch.where(kept[:, None], gate[:, None] * out, torch.zeros_like(out))
    f_i = torch.bincount(g, minlength=n).double() / T
    f_j = torch.bincount(l, minlength=m).double() / T
    inter = n * (f_i * p.mean(0)).sum()
    intra = m * (f_j * q.mean(0)).sum()
    L = (dy * y).sum() + dloss * (alpha * inter + beta * intra)
    L.backward()
    return dict(dx=x.grad.numpy(), dw_inter=wi.grad.numpy(), dw_intra=wq.grad.numpy(), dw1=w1.grad.numpy(),
                dw2=w2.grad.numpy(), drops=int((~kept).sum()))


def _oracle_backward(c, act, alpha, beta, dloss, with_bias, dtype="f32", Cg=0):
    bi, bq = (c["bi"], c["bq"]) if with_bias else (None, None)
    fwd = oracle.layer_forward(c["x"], c["wi"], c["wq"], c["w1"], c["w2"], c["C"], act, dtype, alpha, beta,
                               bias_inter=bi, bias_intra=bq, group_capacity=Cg)
    bwd = oracle.layer_backward(fwd, c["x"], c["wi"], c["wq"], c["w1"], c["w2"], c["dy"], act, dtype, alpha, beta,
                                dloss, bi, bq)
    return fwd, bwd


def _close(a, b, tol, name):
    err = np.abs(np.asarray(a, np.float64) - b).max() / max(np.abs(b).max(), 1e-30)
    assert err <= tol, f"{name}: normwise error {err:.3e}"


@pytest.mark.parametrize("seed,act,with_bias", [(0, "relu", False), (1, "gelu", False), (2, "gelu", True),
                                                (3, "relu", True), (4, "gelu", False)])
def test_backward_against_autograd_of_a_separate_model(seed, act, with_bias):
    # large auxiliary coefficients so that a slip in the Eq. 4 terms cannot hide below the tolerance
    alpha, beta, dloss = 0.7, 0.4, 1.3
    c = _case(seed)
    ref = _torch_model(c, act, alpha, beta, dloss, with_bias)
    assert ref["drops"] > 0, "the case must contain dropped tokens"
    _, bwd = _oracle_backward(c, act, alpha, beta, dloss, with_bias)
    for k in ("dx", "dw_inter", "dw_intra", "dw1", "dw2"):
        _close(bwd[k], ref[k], 2e-6, k)      # fp32 storage of intermediate tensors in the oracle


def test_aux_loss_gradient_alone():
    # dy = 0: only Eq. 4 contributes, the expert weights get no gradient
    c = _case(7)
    c["dy"][:] = 0
    ref = _torch_model(c, "gelu", 0.5, 0.25, 2.0, False)
    _, bwd = _oracle_backward(c, "gelu", 0.5, 0.25, 2.0, False)
    assert np.all(bwd["dw1"] == 0) and np.all(bwd["dw2"] == 0) and np.all(bwd["dgate"] == 0)
    for k in ("dx", "dw_inter", "dw_intra"):
        _close(bwd[k], ref[k], 2e-6, k)
    assert np.abs(ref["dx"]).max() > 0
    # softmax Jacobian: the logit gradients of every token sum to zero
    np.testing.assert_allclose(bwd["dlp"].sum(1), 0, atol=1e-15)
    np.testing.assert_allclose(bwd["dlq"].sum(1), 0, atol=1e-15)


def test_finite_differences_of_the_oracle_forward():
    """Directional derivative of L along a random direction of (x, W_p, W_q, W1, W2) by central differences of the
    oracle's own forward pass, against the inner product with the oracle's gradient."""
    alpha, beta, dloss = 0.3, 0.2, 1.0
    c = _case(11, T=24, d=8, F=8, n=2, m=2, C=5, scale=0.7)
    fwd, bwd = _oracle_backward(c, "gelu", alpha, beta, dloss, True)
    rng = np.random.default_rng(3)
    keys = [("x", "dx"), ("wi", "dw_inter"), ("wq", "dw_intra"), ("w1", "dw1"), ("w2", "dw2")]
    direction = {k: rng.standard_normal(c[k].shape) for k, _ in keys}
    analytic = sum(float((direction[k] * np.asarray(bwd[gk], np.float64)).sum()) for k, gk in keys)

    def loss_at(eps):
        cc = dict(c)
        for k, _ in keys:
            cc[k] = (c[k].astype(np.float64) + eps * direction[k]).astype(np.float32)
        f = oracle.layer_forward(cc["x"], cc["wi"], cc["wq"], cc["w1"], cc["w2"], c["C"], "gelu", "f32", alpha, beta,
                                 bias_inter=c["bi"], bias_intra=c["bq"])
        # same decisions on both sides of the difference, or the function is not differentiable there
        np.testing.assert_array_equal(f["route"].slot, fwd["route"].slot)
        np.testing.assert_array_equal(f["route"].group_idx, fwd["route"].group_idx)
        # Eq. 4 with the counts held fixed is linear in the probability sums
        return float((c["dy"].astype(np.float64) * f["y"]).sum()) + dloss * float(f["loss"][2])

    eps = 2e-3
    numeric = (loss_at(eps) - loss_at(-eps)) / (2 * eps)
    assert abs(numeric - analytic) <= 2e-3 * max(abs(analytic), 1.0), (numeric, analytic)


def test_combine_backward_closed_form():
    rng = np.random.default_rng(5)
    T, n, m, C, d = 30, 2, 2, 6, 4
    li = rng.standard_normal((T, n)).astype(np.float32)
    lq = rng.standard_normal((T, m)).astype(np.float32)
    r = oracle.route(li, lq, C)
    ye = rng.standard_normal((n * m, C, d)).astype(np.float32)
    dy = rng.standard_normal((T, d)).astype(np.float32)
    dye, dgate = oracle.combine_backward(dy, ye, r.group_idx, r.local_idx, r.slot, r.gate, m, "f32", fill=-3.0)
    e = r.group_idx * m + r.local_idx
    k = r.slot >= 0
    assert (~k).any()
    want = np.full_like(ye, -3.0)
    want[e[k], r.slot[k]] = (r.gate[k, None] * dy[k]).astype(np.float32)
    np.testing.assert_array_equal(dye, want)
    np.testing.assert_allclose(dgate[k], (dy[k].astype(np.float64) * ye[e[k], r.slot[k]]).sum(1), rtol=1e-12)
    assert np.all(dgate[~k] == 0)
    # bf16 storage: dye is the rounded product
    dye16, _ = oracle.combine_backward(dy, ye, r.group_idx, r.local_idx, r.slot, r.gate, m, "bf16")
    prod = torch.tensor(r.gate[k, None] * dy[k].astype(np.float64)).to(torch.bfloat16).float().numpy()
    np.testing.assert_array_equal(dye16[e[k], r.slot[k]], prod)


def test_ffn_backward_one_expert_against_torch():
    rng = np.random.default_rng(9)
    Cap, d, F = 17, 8, 12
    xe = rng.standard_normal((1, Cap, d)).astype(np.float32)
    w1 = rng.standard_normal((1, F, d)).astype(np.float32)
    w2 = rng.standard_normal((1, d, F)).astype(np.float32)
    dye = rng.standard_normal((1, Cap, d)).astype(np.float32)
    rows = 11
    for act in ("relu", "gelu"):
        X = torch.tensor(xe[0, :rows].astype(np.float64), requires_grad=True)
        A = torch.tensor(w1[0].astype(np.float64), requires_grad=True)
        Bm = torch.tensor(w2[0].astype(np.float64), requires_grad=True)
        pre = X @ A.T
        h = torch.relu(pre) if act == "relu" else torch.nn.functional.gelu(pre)
        ((h @ Bm.T) * torch.tensor(dye[0, :rows].astype(np.float64))).sum().backward()
        dxe, dw1, dw2 = oracle.expert_ffn_backward(xe, [rows], w1, w2, dye, act, "f32", fill=-1.0)
        _close(dxe[0, :rows], X.grad.numpy(), 1e-6, "dxe")
        assert np.all(dxe[0, rows:] == -1.0)          # rows beyond kept are not written
        _close(dw1[0], A.grad.numpy(), 1e-6, "dw1")
        _close(dw2[0], Bm.grad.numpy(), 1e-6, "dw2")
    # an expert without tokens gets zero weight gradients
    _, dw1, dw2 = oracle.expert_ffn_backward(xe, [0], w1, w2, dye, "gelu", "f32")
    assert np.all(dw1 == 0) and np.all(dw2 == 0)


def test_bf16_backward_stays_close_to_fp32_backward():
    c = _case(21, T=200, d=16, F=32, n=2, m=3, C=40, scale=1.0)
    for k in ("x", "wi", "wq", "w1", "w2", "dy"):
        c[k] = torch.tensor(c[k]).to(torch.bfloat16).float().numpy()
    _, b32 = _oracle_backward(c, "gelu", 0.01, 0.01, 1.0, False, "f32")
    _, b16 = _oracle_backward(c, "gelu", 0.01, 0.01, 1.0, False, "bf16")
    for k in ("dx", "dw1", "dw2", "dw_inter", "dw_intra"):
        _close(b16[k], np.asarray(b32[k], np.float64), 2e-2, k)
    # and its stored tensors are bf16 values
    for k in ("dx", "dw1", "dw2", "dxe", "dye"):
        v = b16[k]
        np.testing.assert_array_equal(v, torch.tensor(v).to(torch.bfloat16).float().numpy())


def test_group_capacity_drops_send_nothing_back():
    c = _case(31, T=60, d=8, F=8, n=2, m=2, C=60)
    fwd, bwd = _oracle_backward(c, "relu", 0.0, 0.0, 0.0, False, Cg=12)
    late = fwd["route"].pos_in_group >= 12
    assert late.any()
    assert np.all(bwd["dgate"][late] == 0) and np.all(bwd["dx"][late] == 0)
    assert np.abs(bwd["dx"][~late]).max() > 0
