"""Host-side checks of the C-ABI library: it loads, exports every function the header declares,
and its argument validation (which runs before anything touches a GPU) behaves as documented.
No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

import oracle
from paper_2212_05191_amd import binding as B
from paper_2212_05191_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "smile.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(smile_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = B.load()
    names = _declared_functions()
    assert len(names) >= 15
    for name in names:
        assert hasattr(lib, name), f"{name} declared in include/smile.h but not exported"
    assert sorted(B.EXPORTS) == names
    assert B.version().count(".") == 2


def test_status_strings():
    seen = {B.status_string(s) for s in range(6)}
    assert len(seen) == 6 and "ok" in seen
    assert B.status_string(99) == "unknown status"


def test_capacity_helper_matches_the_rule_and_the_configs():
    for cfg in wl.CONFIGS.values():
        assert B.smile_capacity(cfg.T, cfg.N, cfg.capacity_factor) == cfg.capacity
    for T, N, cf in [(10, 4, 1.0), (1, 64, 1.0), (16384, 128, 2.0), (1000, 7, 1.3), (5, 5, 0.01)]:
        assert B.smile_capacity(T, N, cf) == oracle.capacity(T, N, cf)
    assert B.smile_capacity(0, 4, 1.0) == -1
    assert B.smile_capacity(4, 0, 1.0) == -1
    assert B.smile_capacity(4, 4, 0.0) == -1
    assert B.smile_capacity(4, 4, float("nan")) == -1


def _desc(**kw):
    base = dict(T=512, d_model=64, d_ff=128, n_groups=2, m_local=2, capacity=160, dtype="f32", act="relu")
    base.update(kw)
    return B.make_desc(**base)


def test_validate_desc_accepts_the_five_configs():
    for cfg in wl.CONFIGS.values():
        d = B.make_desc(cfg.T, cfg.d_model, cfg.d_ff, cfg.n_groups, cfg.m_local, cfg.capacity, cfg.dtype, cfg.act)
        assert B.smile_validate_desc(d) == B.OK
        assert B.smile_workspace_bytes(d) > 0
        d.group_capacity = 7
        assert B.smile_validate_desc(d) == B.OK
        if cfg.dtype == "bf16":
            d.dtype = B.DTYPE["f16"]
            assert B.smile_validate_desc(d) == B.OK


def test_desc_layout_matches_the_header():
    """The ctypes mirror has the fields of the C struct, in the header's order (all 4-byte members)."""
    text = open(os.path.join(ROOT, "include", "smile.h")).read()
    body = re.search(r"typedef struct smile_layer_desc \{(.*?)\} smile_layer_desc;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = re.findall(r"(?:int32_t|float)\s+(\w+)\s*;", body)
    assert names == [k for k, _ in B.LayerDesc._fields_]
    assert C.sizeof(B.LayerDesc) == 4 * len(names)


@pytest.mark.parametrize("kw,status", [
    (dict(T=0), B.BAD_SHAPE), (dict(capacity=0), B.BAD_SHAPE), (dict(n_groups=0), B.BAD_SHAPE),
    (dict(m_local=-1), B.BAD_SHAPE), (dict(d_model=60), B.BAD_SHAPE), (dict(d_ff=100), B.BAD_SHAPE),
    (dict(dtype="bf16", d_model=72), B.BAD_SHAPE), (dict(dtype="bf16", d_ff=96), B.BAD_SHAPE),
    (dict(dtype="f16", d_model=72), B.BAD_SHAPE),
    (dict(n_groups=2048), B.BAD_SHAPE), (dict(n_groups=128, m_local=64), B.BAD_SHAPE),
    (dict(capacity=2 ** 30, n_groups=4), B.BAD_SHAPE),
    (dict(dtype=7), B.UNSUPPORTED), (dict(act=3), B.UNSUPPORTED),
    (dict(alpha=float("inf")), B.BAD_SHAPE), (dict(group_capacity=-1), B.BAD_SHAPE),
])
def test_validate_desc_rejects(kw, status):
    assert B.smile_validate_desc(_desc(**kw)) == status


def test_null_arguments():
    lib = B.load()
    assert lib.smile_validate_desc(None) == B.INVALID_ARG
    assert lib.smile_workspace_bytes(C.byref(_desc()), None) == B.INVALID_ARG
    assert lib.smile_create(C.byref(_desc()), None) == B.INVALID_ARG
    assert lib.smile_destroy(None) == B.OK
    h = C.c_void_p(None)
    assert lib.smile_create(C.byref(_desc(T=0)), C.byref(h)) == B.BAD_SHAPE and not h
    assert lib.smile_create_with_workspace(C.byref(_desc()), None, 0, C.byref(h)) == B.INVALID_ARG


def test_workspace_size_and_alignment_checks():
    """A ctx on a caller 'workspace' needs no GPU: the address is only stored, never touched by the host."""
    lib = B.load()
    d = _desc()
    need = B.smile_workspace_bytes(d)
    h = C.c_void_p(None)
    fake = 0x7F0000000000   # 256-byte aligned, never dereferenced
    assert lib.smile_create_with_workspace(C.byref(d), fake, need - 1, C.byref(h)) == B.WORKSPACE
    assert lib.smile_create_with_workspace(C.byref(d), fake + 16, need, C.byref(h)) == B.WORKSPACE
    assert lib.smile_create_with_workspace(C.byref(d), fake, need, C.byref(h)) == B.OK and h
    assert lib.smile_destroy(h) == B.OK


def test_entry_points_reject_bad_pointers_before_any_launch():
    lib = B.load()
    d = _desc(n_groups=100, m_local=40)
    need = B.smile_workspace_bytes(d)
    h = C.c_void_p(None)
    fake = 0x7F0000000000
    assert lib.smile_create_with_workspace(C.byref(d), fake, need, C.byref(h)) == B.OK
    p = fake + 4096          # aligned dummy pointer; every call below has a bad argument, so the checks
                             # fail before anything could be enqueued with it
    try:
        # NULL ctx
        assert lib.smile_gate_logits(None, p, p, p, p, p, None) == B.INVALID_ARG
        # NULL and misaligned tensors
        assert lib.smile_gate_logits(h, None, p, p, p, p, None) == B.INVALID_ARG
        assert lib.smile_gate_logits(h, p, p, p, p + 4, p, None) == B.INVALID_ARG
        args = [p] * 17
        for i in [0, 1, 4, 7, 16]:
            bad = list(args)
            bad[i] = None
            assert lib.smile_route_bilevel(h, *bad, None) == B.INVALID_ARG
        mis = list(args)
        mis[2] = p + 8      # optional bias given but misaligned
        assert lib.smile_route_bilevel(h, *mis, None) == B.INVALID_ARG
        assert lib.smile_dispatch(h, p, p, p, None, p, None) == B.INVALID_ARG
        assert lib.smile_dispatch_hop1(h, p, p, None, 8, p, None) == B.INVALID_ARG
        assert lib.smile_dispatch_hop1(h, p, p, p, 0, p, None) == B.BAD_SHAPE
        assert lib.smile_dispatch_hop1(h, p, p, p, 2 ** 30, p, None) == B.BAD_SHAPE
        assert lib.smile_dispatch_hop2(h, p, p, p, p, p, 8, p + 4, None) == B.INVALID_ARG
        assert lib.smile_dispatch_hop2(h, p, p, p, p, p, -1, p, None) == B.BAD_SHAPE
        assert lib.smile_expert_ffn(h, p, None, p, None, p, None, p, None) == B.INVALID_ARG
        assert lib.smile_expert_ffn(h, p, p, p, p + 2, p, None, p, None) == B.INVALID_ARG
        assert lib.smile_combine(h, p, p, p, p, None, p, None) == B.INVALID_ARG
        assert lib.smile_aux_loss(h, p, p, p, p, None, None) == B.INVALID_ARG
        assert lib.smile_layer_forward(h, None, None) == B.INVALID_ARG
        io = B.LayerIO()
        for k, _ in B.LayerIO._fields_:
            setattr(io, k, p)
        io.y = None
        assert lib.smile_layer_forward(h, C.byref(io), None) == B.INVALID_ARG
        io.y = p
        io.xe = None                # expert buffers come as a pair or not at all
        assert lib.smile_layer_forward(h, C.byref(io), None) == B.INVALID_ARG
        io.xe = p
        io.prof_up_stop = None      # timing events come as a pair or not at all
        assert lib.smile_layer_forward(h, C.byref(io), None) == B.INVALID_ARG
        io.prof_up_stop = p
        io.pre_save = None          # saved activations come as a pair or not at all
        assert lib.smile_layer_forward(h, C.byref(io), None) == B.INVALID_ARG
        assert lib.smile_expert_ffn_up_timed(h, p, p, p, None, p, None, None) == B.INVALID_ARG
    finally:
        assert lib.smile_destroy(h) == B.OK


def test_backward_entry_points_reject_bad_arguments_before_any_launch():
    lib = B.load()
    d = _desc()
    h = C.c_void_p(None)
    fake = 0x7F0000000000
    assert lib.smile_create_with_workspace(C.byref(d), fake, B.smile_workspace_bytes(d), C.byref(h)) == B.OK
    p = fake + 4096
    need = B.smile_backward_workspace_bytes(d)
    assert need > 0
    ws = fake + (1 << 30)
    f1 = C.c_float(1.0)
    try:
        assert lib.smile_backward_workspace_bytes(C.byref(d), None) == B.INVALID_ARG
        assert lib.smile_combine_backward(h, p, p, p, p, p, p, None, p, None) == B.INVALID_ARG
        assert lib.smile_combine_backward(None, p, p, p, p, p, p, p, p, None) == B.INVALID_ARG
        assert lib.smile_route_backward(h, p, p, None, None, p, p, p, p, p, f1, p, None, None) == B.INVALID_ARG
        assert lib.smile_route_backward(h, p, p, None, None, p, p, p, p, p, C.c_float(float("nan")), p, p, None) \
            == B.BAD_SHAPE
        assert lib.smile_expert_ffn_backward(h, p, p, p, p, p, None, None, p, p, None, ws, need, None) == B.INVALID_ARG
        assert lib.smile_expert_ffn_backward(h, p, p, p, p, p, p, None, p, p, p, ws, need, None) == B.INVALID_ARG
        assert lib.smile_expert_ffn_backward(h, p, p, p, p, p, p, p, p, p, p, None, need, None) == B.INVALID_ARG
        assert lib.smile_expert_ffn_backward(h, p, p, p, p, p, None, None, p, p, p, ws, need - 1, None) == B.WORKSPACE
        assert lib.smile_expert_ffn_backward(h, p, p, p, p, p, p, p, p, p, p, ws + 16, need, None) == B.WORKSPACE
        assert lib.smile_dispatch_backward(h, p, p, p, p, p, p, p, p + 4, p, None) == B.INVALID_ARG
        assert lib.smile_gate_weights_backward(h, p, p, p, p, p, ws, need - 1, None) == B.WORKSPACE
        assert lib.smile_gate_weights_backward(h, p, p, p, None, p, ws, need, None) == B.INVALID_ARG
        io = B.BackwardIO()
        for k, _ in B.BackwardIO._fields_:
            setattr(io, k, p)
        assert lib.smile_layer_backward(h, None, f1, ws, need, None) == B.INVALID_ARG
        assert lib.smile_layer_backward(h, C.byref(io), f1, ws, need - 1, None) == B.WORKSPACE
        io.dw2 = None
        assert lib.smile_layer_backward(h, C.byref(io), f1, ws, need, None) == B.INVALID_ARG
        io.dw2 = p
        io.h = None                 # saved activations come as a pair or not at all
        assert lib.smile_layer_backward(h, C.byref(io), f1, ws, need, None) == B.INVALID_ARG
        io.pre = None
        io.bias_inter = None        # optional
        io.dy = p + 2
        assert lib.smile_layer_backward(h, C.byref(io), f1, ws, need, None) == B.INVALID_ARG
    finally:
        assert lib.smile_destroy(h) == B.OK


def test_binding_raises_with_status():
    with pytest.raises(B.SmileError) as ei:
        B.smile_workspace_bytes(_desc(T=-5))
    assert ei.value.status == B.BAD_SHAPE


def test_static_scratch_routing_rejects_before_any_launch():
    """smile_route_bilevel_static checks the description, the pointers and the size of its fixed scratch
    array on the host before it looks up that array or enqueues anything (so this needs no GPU)."""
    lib = B.load()
    p = 0x7F0000000000 + 4096
    args = [p] * 17
    assert lib.smile_route_bilevel_static(None, *args, None) == B.INVALID_ARG
    assert lib.smile_route_bilevel_static(C.byref(_desc(T=0)), *args, None) == B.BAD_SHAPE
    assert lib.smile_route_bilevel_static(C.byref(_desc(dtype=7)), *args, None) == B.UNSUPPORTED
    for i in [0, 1, 4, 7, 16]:
        bad = list(args)
        bad[i] = None
        assert lib.smile_route_bilevel_static(C.byref(_desc()), *bad, None) == B.INVALID_ARG
    bad = list(args)
    bad[5] = p + 4
    assert lib.smile_route_bilevel_static(C.byref(_desc()), *bad, None) == B.INVALID_ARG
    # routing scratch beyond the fixed array: 16384 blocks x 256 experts x 4 bytes alone is 16 MiB
    huge = _desc(T=1 << 22, n_groups=32, m_local=8, capacity=20000)
    assert lib.smile_validate_desc(C.byref(huge)) == B.OK
    assert lib.smile_route_bilevel_static(C.byref(huge), *args, None) == B.WORKSPACE


def test_kernel_timing_argument_checks():
    """smile_kernel_timing stores caller-owned event handles in the ctx; its checks need no GPU."""
    lib = B.load()
    d = _desc()
    h = C.c_void_p(None)
    fake = 0x7F0000000000
    assert lib.smile_create_with_workspace(C.byref(d), fake, B.smile_workspace_bytes(d), C.byref(h)) == B.OK
    try:
        ev = (C.c_void_p * 8)(*[fake + 64 * (i + 1) for i in range(8)])
        assert lib.smile_kernel_timing(None, ev, 4) == B.INVALID_ARG
        assert lib.smile_kernel_timing(h, None, 4) == B.INVALID_ARG
        assert lib.smile_kernel_timing(h, ev, -1) == B.INVALID_ARG
        holes = (C.c_void_p * 8)(*[fake + 64 * (i + 1) if i != 5 else None for i in range(8)])
        assert lib.smile_kernel_timing(h, holes, 4) == B.INVALID_ARG       # a NULL handle among the 2 * pairs
        assert lib.smile_kernel_timing(h, ev, 4) == B.OK
        assert lib.smile_kernel_timing_count(h) == 0                        # no call has run yet
        assert lib.smile_kernel_timing_name(h, 0) == b"" and lib.smile_kernel_timing_name(h, -1) == b""
        assert lib.smile_kernel_timing(h, None, 0) == B.OK                  # detach
        assert lib.smile_kernel_timing_count(None) == 0
    finally:
        assert lib.smile_destroy(h) == B.OK
