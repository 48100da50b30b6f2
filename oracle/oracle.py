"""ctypes front end of the C oracle (oracle/smile_oracle.c).

TEST INFRASTRUCTURE ONLY: marshals numpy arrays into the C functions and
allocates their outputs.  No arithmetic of the method lives here; the one
exception is layer_forward(), which only chains the C steps in the order the
layer runs them (Section 3.2.1: route, dispatch, expert, combine; Eq. 4 loss).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "smile_oracle.c")
_LIB = os.path.join(_HERE, "libsmile_oracle.so")
_lib = None

_ACT = {"relu": 0, "gelu": 1}
_DTYPE = {"f32": 0, "bf16": 1, "f16": 2}


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_LIB)
        _lib.smile_oracle_capacity.restype = C.c_int32
        _lib.smile_oracle_capacity.argtypes = [C.c_int32, C.c_int32, C.c_double]
        _lib.smile_oracle_threads.restype = C.c_int
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def threads() -> int:
    return int(_load().smile_oracle_threads())


def capacity(T: int, N: int, cf: float) -> int:
    return int(_load().smile_oracle_capacity(int(T), int(N), float(cf)))


def gate_logits(x, w_inter, w_intra):
    x, w_inter, w_intra = _f32(x), _f32(w_inter), _f32(w_intra)
    T, d = x.shape
    n, m = w_inter.shape[0], w_intra.shape[0]
    assert w_inter.shape == (n, d) and w_intra.shape == (m, d)
    li = np.empty((T, n), np.float32)
    lq = np.empty((T, m), np.float32)
    _load().smile_oracle_gate_logits(_p(x), _p(w_inter), _p(w_intra), C.c_int32(T), C.c_int32(d),
                                     C.c_int32(n), C.c_int32(m), _p(li), _p(lq))
    return li, lq


@dataclass
class RouteResult:
    group_idx: np.ndarray
    local_idx: np.ndarray
    pos_in_group: np.ndarray
    slot: np.ndarray
    gate: np.ndarray        # float64
    p_top: np.ndarray
    q_top: np.ndarray
    group_count: np.ndarray
    local_count: np.ndarray
    expert_count: np.ndarray
    kept_count: np.ndarray
    p_sum: np.ndarray       # float64
    q_sum: np.ndarray


def route(logits_inter, logits_intra, capacity_rows: int, bias_inter=None, bias_intra=None,
          group_capacity: int = 0) -> RouteResult:
    li, lq = _f32(logits_inter), _f32(logits_intra)
    T, n = li.shape
    m = lq.shape[1]
    assert lq.shape[0] == T
    bi = None if bias_inter is None else _f32(bias_inter).reshape(n)
    bq = None if bias_intra is None else _f32(bias_intra).reshape(n, m)
    N = n * m
    r = RouteResult(
        np.empty(T, np.int32), np.empty(T, np.int32), np.empty(T, np.int32), np.empty(T, np.int32),
        np.empty(T, np.float64), np.empty(T, np.float64), np.empty(T, np.float64),
        np.empty(n, np.int32), np.empty(m, np.int32), np.empty(N, np.int32), np.empty(N, np.int32),
        np.empty(n, np.float64), np.empty(m, np.float64))
    _load().smile_oracle_route(_p(li), _p(lq), _p(bi), _p(bq), C.c_int32(T), C.c_int32(n), C.c_int32(m),
                               C.c_int32(int(capacity_rows)), C.c_int32(int(group_capacity)),
                               _p(r.group_idx), _p(r.local_idx), _p(r.pos_in_group), _p(r.slot),
                               _p(r.gate), _p(r.p_top), _p(r.q_top),
                               _p(r.group_count), _p(r.local_count), _p(r.expert_count), _p(r.kept_count),
                               _p(r.p_sum), _p(r.q_sum))
    return r


def slots_two_stage(group_idx, local_idx, n: int, m: int, capacity_rows: int, group_capacity: int = 0):
    g, l = _i32(group_idx), _i32(local_idx)
    T = g.shape[0]
    pos = np.full(T, -7, np.int32)
    slot = np.full(T, -7, np.int32)
    _load().smile_oracle_slots_two_stage(_p(g), _p(l), C.c_int32(T), C.c_int32(n), C.c_int32(m),
                                         C.c_int32(int(capacity_rows)), C.c_int32(int(group_capacity)), _p(pos),
                                         _p(slot))
    return pos, slot


def dispatch_stage1(x, group_idx, pos_in_group, n: int, group_rows: int, fill: float = 0.0):
    x = _f32(x)
    T, d = x.shape
    xg = np.full((n, int(group_rows), d), fill, np.float32)
    _load().smile_oracle_dispatch_stage1(_p(x), _p(_i32(group_idx)), _p(_i32(pos_in_group)), C.c_int32(T),
                                         C.c_int32(d), C.c_int32(int(group_rows)), _p(xg))
    return xg


def dispatch_stage2(xg, group_idx, local_idx, pos_in_group, slot, m: int, capacity_rows: int, fill: float = 0.0):
    xg = _f32(xg)
    n, Cg, d = xg.shape
    g = _i32(group_idx)
    T = g.shape[0]
    xe = np.full((n * m, int(capacity_rows), d), fill, np.float32)
    _load().smile_oracle_dispatch_stage2(_p(xg), _p(g), _p(_i32(local_idx)), _p(_i32(pos_in_group)), _p(_i32(slot)),
                                         C.c_int32(T), C.c_int32(d), C.c_int32(m), C.c_int32(int(capacity_rows)),
                                         C.c_int32(Cg), _p(xe))
    return xe


def dispatch(x, group_idx, local_idx, slot, n: int, m: int, capacity_rows: int, fill: float = 0.0):
    x = _f32(x)
    T, d = x.shape
    xe = np.full((n * m, int(capacity_rows), d), fill, np.float32)
    _load().smile_oracle_dispatch(_p(x), _p(_i32(group_idx)), _p(_i32(local_idx)), _p(_i32(slot)),
                                  C.c_int32(T), C.c_int32(d), C.c_int32(m), C.c_int32(int(capacity_rows)), _p(xe))
    return xe


def expert_ffn(xe, kept_count, w1, w2, act: str, dtype: str, b1=None, b2=None):
    xe, w1, w2 = _f32(xe), _f32(w1), _f32(w2)
    N, Cap, d = xe.shape
    F = w1.shape[1]
    assert w1.shape == (N, F, d) and w2.shape == (N, d, F)
    kept = _i32(kept_count)
    assert kept.shape == (N,) and kept.min(initial=0) >= 0 and kept.max(initial=0) <= Cap
    b1 = None if b1 is None else _f32(b1).reshape(N, F)
    b2 = None if b2 is None else _f32(b2).reshape(N, d)
    ye = np.zeros((N, Cap, d), np.float32)
    _load().smile_oracle_expert_ffn(_p(xe), _p(kept), _p(w1), _p(b1), _p(w2), _p(b2),
                                    C.c_int32(N), C.c_int32(Cap), C.c_int32(d), C.c_int32(F),
                                    C.c_int32(_ACT[act]), C.c_int32(_DTYPE[dtype]), _p(ye))
    return ye


def combine(ye, group_idx, local_idx, slot, gate, m: int, dtype: str):
    ye = _f32(ye)
    N, Cap, d = ye.shape
    g = _i32(group_idx)
    T = g.shape[0]
    y = np.empty((T, d), np.float32)
    _load().smile_oracle_combine(_p(ye), _p(g), _p(_i32(local_idx)), _p(_i32(slot)), _p(_f64(gate)),
                                 C.c_int32(T), C.c_int32(d), C.c_int32(m), C.c_int32(Cap),
                                 C.c_int32(_DTYPE[dtype]), _p(y))
    return y


def aux_loss(group_count, local_count, p_sum, q_sum, T: int, alpha: float, beta: float):
    gc, lc = _i32(group_count), _i32(local_count)
    ps, qs = _f64(p_sum), _f64(q_sum)
    out = np.empty(3, np.float64)
    _load().smile_oracle_aux_loss(_p(gc), _p(lc), _p(ps), _p(qs), C.c_int32(int(T)),
                                  C.c_int32(gc.shape[0]), C.c_int32(lc.shape[0]),
                                  C.c_double(alpha), C.c_double(beta), _p(out))
    return out


def layer_forward(x, w_inter, w_intra, w1, w2, capacity_rows: int, act: str, dtype: str,
                  alpha: float = 0.005, beta: float = 0.005, bias_inter=None, bias_intra=None,
                  logits=None, group_capacity: int = 0):
    """Chain the steps of one layer forward.  `logits` (inter, intra) overrides step 1."""
    n, m = np.shape(w_inter)[0], np.shape(w_intra)[0]
    li, lq = gate_logits(x, w_inter, w_intra) if logits is None else logits
    r = route(li, lq, capacity_rows, bias_inter, bias_intra, group_capacity)
    xe = dispatch(x, r.group_idx, r.local_idx, r.slot, n, m, capacity_rows)
    ye = expert_ffn(xe, r.kept_count, w1, w2, act, dtype)
    y = combine(ye, r.group_idx, r.local_idx, r.slot, r.gate, m, dtype)
    loss = aux_loss(r.group_count, r.local_count, r.p_sum, r.q_sum, np.shape(x)[0], alpha, beta)
    return dict(logits_inter=li, logits_intra=lq, route=r, xe=xe, ye=ye, y=y, loss=loss)


# ---------------------------------------------------------------- backward pass

def combine_backward(dy, ye, group_idx, local_idx, slot, gate, m: int, dtype: str, fill: float = 0.0):
    dy, ye = _f32(dy), _f32(ye)
    N, Cap, d = ye.shape
    T = dy.shape[0]
    dye = np.full((N, Cap, d), fill, np.float32)
    dgate = np.empty(T, np.float64)
    _load().smile_oracle_combine_backward(_p(dy), _p(ye), _p(_i32(group_idx)), _p(_i32(local_idx)), _p(_i32(slot)),
                                          _p(_f64(gate)), C.c_int32(T), C.c_int32(d), C.c_int32(m), C.c_int32(Cap),
                                          C.c_int32(_DTYPE[dtype]), _p(dye), _p(dgate))
    return dye, dgate


def route_backward(logits_inter, logits_intra, group_idx, local_idx, dgate, group_count, local_count,
                   alpha: float, beta: float, dloss: float = 1.0, bias_inter=None, bias_intra=None):
    li, lq = _f32(logits_inter), _f32(logits_intra)
    T, n = li.shape
    m = lq.shape[1]
    bi = None if bias_inter is None else _f32(bias_inter).reshape(n)
    bq = None if bias_intra is None else _f32(bias_intra).reshape(n, m)
    dlp = np.empty((T, n), np.float64)
    dlq = np.empty((T, m), np.float64)
    _load().smile_oracle_route_backward(_p(li), _p(lq), _p(bi), _p(bq), _p(_i32(group_idx)), _p(_i32(local_idx)),
                                        _p(_f64(dgate)), _p(_i32(group_count)), _p(_i32(local_count)),
                                        C.c_int32(T), C.c_int32(n), C.c_int32(m), C.c_double(alpha), C.c_double(beta),
                                        C.c_double(dloss), _p(dlp), _p(dlq))
    return dlp, dlq


def expert_ffn_backward(xe, kept_count, w1, w2, dye, act: str, dtype: str, fill: float = 0.0):
    xe, w1, w2, dye = _f32(xe), _f32(w1), _f32(w2), _f32(dye)
    N, Cap, d = xe.shape
    F = w1.shape[1]
    assert w1.shape == (N, F, d) and w2.shape == (N, d, F) and dye.shape == xe.shape
    kept = _i32(kept_count)
    dxe = np.full((N, Cap, d), fill, np.float32)
    dw1 = np.empty((N, F, d), np.float32)
    dw2 = np.empty((N, d, F), np.float32)
    _load().smile_oracle_expert_ffn_backward(_p(xe), _p(kept), _p(w1), _p(w2), _p(dye), C.c_int32(N), C.c_int32(Cap),
                                             C.c_int32(d), C.c_int32(F), C.c_int32(_ACT[act]),
                                             C.c_int32(_DTYPE[dtype]), _p(dxe), _p(dw1), _p(dw2))
    return dxe, dw1, dw2


def dispatch_backward(dxe, group_idx, local_idx, slot, dlp, dlq, w_inter, w_intra, dtype: str):
    dxe, wi, wq = _f32(dxe), _f32(w_inter), _f32(w_intra)
    N, Cap, d = dxe.shape
    n, m = wi.shape[0], wq.shape[0]
    g = _i32(group_idx)
    T = g.shape[0]
    dx = np.empty((T, d), np.float32)
    _load().smile_oracle_dispatch_backward(_p(dxe), _p(g), _p(_i32(local_idx)), _p(_i32(slot)), _p(_f64(dlp)),
                                           _p(_f64(dlq)), _p(wi), _p(wq), C.c_int32(T), C.c_int32(d), C.c_int32(n),
                                           C.c_int32(m), C.c_int32(Cap), C.c_int32(_DTYPE[dtype]), _p(dx))
    return dx


def gate_weights_backward(x, dlp, dlq):
    x, dlp, dlq = _f32(x), _f64(dlp), _f64(dlq)
    T, d = x.shape
    n, m = dlp.shape[1], dlq.shape[1]
    dwi = np.empty((n, d), np.float64)
    dwq = np.empty((m, d), np.float64)
    _load().smile_oracle_gate_weights_backward(_p(x), _p(dlp), _p(dlq), C.c_int32(T), C.c_int32(d), C.c_int32(n),
                                               C.c_int32(m), _p(dwi), _p(dwq))
    return dwi, dwq


def layer_backward(fwd: dict, x, w_inter, w_intra, w1, w2, dy, act: str, dtype: str,
                   alpha: float = 0.005, beta: float = 0.005, dloss: float = 1.0, bias_inter=None, bias_intra=None):
    """Chain the backward steps in reverse order of layer_forward(); `fwd` is its result."""
    r = fwd["route"]
    m = np.shape(w_intra)[0]
    dye, dgate = combine_backward(dy, fwd["ye"], r.group_idx, r.local_idx, r.slot, r.gate, m, dtype)
    dlp, dlq = route_backward(fwd["logits_inter"], fwd["logits_intra"], r.group_idx, r.local_idx, dgate,
                              r.group_count, r.local_count, alpha, beta, dloss, bias_inter, bias_intra)
    dxe, dw1, dw2 = expert_ffn_backward(fwd["xe"], r.kept_count, w1, w2, dye, act, dtype)
    dx = dispatch_backward(dxe, r.group_idx, r.local_idx, r.slot, dlp, dlq, w_inter, w_intra, dtype)
    dwi, dwq = gate_weights_backward(x, dlp, dlq)
    return dict(dye=dye, dgate=dgate, dlp=dlp, dlq=dlq, dxe=dxe, dw1=dw1, dw2=dw2, dx=dx,
                dw_inter=dwi, dw_intra=dwq)
