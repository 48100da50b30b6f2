"""Thin ctypes binding of libsmile (include/smile.h): argument marshalling only.

Every step of the layer runs in the HIP kernels of the library; PyTorch is used
for device memory (tensor.data_ptr()) and the current stream.  There is no
fallback: if the built library is missing, load() raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsmile.so")
_lib = None

DTYPE = {"f32": 0, "bf16": 1, "f16": 2}
ACT = {"relu": 0, "gelu": 1}

OK, INVALID_ARG, BAD_SHAPE, UNSUPPORTED, WORKSPACE, HIP_ERROR = range(6)


class SmileError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class LayerDesc(C.Structure):
    _fields_ = [("T", C.c_int32), ("d_model", C.c_int32), ("d_ff", C.c_int32), ("n_groups", C.c_int32),
                ("m_local", C.c_int32), ("capacity", C.c_int32), ("dtype", C.c_int32), ("act", C.c_int32),
                ("alpha", C.c_float), ("beta", C.c_float), ("group_capacity", C.c_int32)]


class LayerIO(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in (
        "x", "w_inter", "w_intra", "w1", "b1", "w2", "b2", "bias_inter", "bias_intra",
        "logits_inter", "logits_intra", "group_idx", "local_idx", "pos_in_group", "slot",
        "gate", "p_top", "q_top", "group_count", "local_count", "expert_count", "kept_count",
        "p_sum", "q_sum", "xe", "ye", "y", "loss3", "prof_up_start", "prof_up_stop", "h_save", "pre_save")]


class BackwardIO(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in (
        "x", "w_inter", "w_intra", "w1", "w2", "bias_inter", "bias_intra",
        "logits_inter", "logits_intra", "group_idx", "local_idx", "slot", "gate",
        "group_count", "local_count", "kept_count", "xe", "ye", "h", "pre", "dy",
        "dye", "dgate", "dlp", "dlq", "dxe", "dx", "dw_inter", "dw_intra", "dw1", "dw2")]


EXPORTS = (
    "smile_status_string", "smile_version", "smile_capacity", "smile_validate_desc", "smile_workspace_bytes",
    "smile_create", "smile_create_with_workspace", "smile_destroy", "smile_gate_logits", "smile_route_bilevel",
    "smile_route_bilevel_static", "smile_kernel_timing", "smile_kernel_timing_count", "smile_kernel_timing_name",
    "smile_dispatch", "smile_dispatch_hop1", "smile_dispatch_hop2", "smile_expert_ffn", "smile_expert_ffn_up", "smile_expert_ffn_down", "smile_expert_ffn_up_timed", "smile_combine", "smile_aux_loss", "smile_layer_forward",
    "smile_backward_workspace_bytes", "smile_combine_backward", "smile_route_backward", "smile_expert_ffn_backward",
    "smile_dispatch_backward", "smile_gate_weights_backward", "smile_layer_backward",
)


def load() -> C.CDLL:
    """Load libsmile.so built in-tree by paper_2212_05191_amd.build; raise if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2212_05191_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int32
    lib.smile_status_string.restype = C.c_char_p
    lib.smile_status_string.argtypes = [i32]
    lib.smile_version.restype = C.c_char_p
    lib.smile_capacity.restype = i32
    lib.smile_capacity.argtypes = [i32, i32, C.c_double]
    lib.smile_validate_desc.argtypes = [C.POINTER(LayerDesc)]
    lib.smile_workspace_bytes.argtypes = [C.POINTER(LayerDesc), C.POINTER(C.c_size_t)]
    lib.smile_create.argtypes = [C.POINTER(LayerDesc), C.POINTER(vp)]
    lib.smile_create_with_workspace.argtypes = [C.POINTER(LayerDesc), vp, C.c_size_t, C.POINTER(vp)]
    lib.smile_destroy.argtypes = [vp]
    lib.smile_gate_logits.argtypes = [vp] * 7
    lib.smile_kernel_timing.argtypes = [vp, C.POINTER(vp), i32]
    lib.smile_kernel_timing_count.argtypes = [vp]
    lib.smile_kernel_timing_count.restype = i32
    lib.smile_kernel_timing_name.argtypes = [vp, i32]
    lib.smile_route_bilevel.argtypes = [vp] * 19
    lib.smile_route_bilevel_static.argtypes = [C.POINTER(LayerDesc)] + [vp] * 18
    lib.smile_dispatch.argtypes = [vp] * 7
    lib.smile_dispatch_hop1.argtypes = [vp, vp, vp, vp, i32, vp, vp]
    lib.smile_dispatch_hop2.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.smile_expert_ffn.argtypes = [vp] * 9
    lib.smile_expert_ffn_up.argtypes = [vp] * 6
    lib.smile_expert_ffn_down.argtypes = [vp] * 6
    lib.smile_expert_ffn_up_timed.argtypes = [vp] * 8
    lib.smile_combine.argtypes = [vp] * 8
    lib.smile_aux_loss.argtypes = [vp] * 7
    lib.smile_layer_forward.argtypes = [vp, C.POINTER(LayerIO), vp]
    lib.smile_backward_workspace_bytes.argtypes = [C.POINTER(LayerDesc), C.POINTER(C.c_size_t)]
    lib.smile_combine_backward.argtypes = [vp] * 10
    lib.smile_route_backward.argtypes = [vp] * 10 + [C.c_float, vp, vp, vp]
    lib.smile_expert_ffn_backward.argtypes = [vp] * 12 + [C.c_size_t, vp]
    lib.smile_dispatch_backward.argtypes = [vp] * 11
    lib.smile_gate_weights_backward.argtypes = [vp] * 7 + [C.c_size_t, vp]
    lib.smile_layer_backward.argtypes = [vp, C.POINTER(BackwardIO), C.c_float, vp, C.c_size_t, vp]
    for name in EXPORTS[3:]:
        getattr(lib, name).restype = i32
    lib.smile_kernel_timing_name.restype = C.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().smile_status_string(int(status)).decode()


def version() -> str:
    return load().smile_version().decode()


def smile_capacity(T: int, N: int, capacity_factor: float) -> int:
    return int(load().smile_capacity(int(T), int(N), float(capacity_factor)))


def make_desc(T, d_model, d_ff, n_groups, m_local, capacity, dtype="bf16", act="gelu",
              alpha=0.005, beta=0.005, group_capacity=0) -> LayerDesc:
    return LayerDesc(int(T), int(d_model), int(d_ff), int(n_groups), int(m_local), int(capacity),
                     DTYPE[dtype] if isinstance(dtype, str) else int(dtype),
                     ACT[act] if isinstance(act, str) else int(act), float(alpha), float(beta), int(group_capacity))


def smile_validate_desc(desc: LayerDesc) -> int:
    return int(load().smile_validate_desc(C.byref(desc)))


def smile_workspace_bytes(desc: LayerDesc) -> int:
    out = C.c_size_t(0)
    st = load().smile_workspace_bytes(C.byref(desc), C.byref(out))
    if st != OK:
        raise SmileError(st, "smile_workspace_bytes")
    return int(out.value)


def _ptr(t):
    """Device pointer of a torch tensor (None -> NULL); ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "tensors must be dense row-major"
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _check(st: int, where: str):
    if st != OK:
        raise SmileError(int(st), where)


class Ctx:
    """Owner of a smile_ctx.  workspace=None: the library allocates; else a uint8 torch tensor."""

    def __init__(self, desc: LayerDesc, workspace=None):
        self.desc = desc
        self._h = C.c_void_p(None)
        self._ws = workspace
        lib = load()
        if workspace is None:
            _check(lib.smile_create(C.byref(desc), C.byref(self._h)), "smile_create")
        else:
            nbytes = workspace.numel() * workspace.element_size()
            _check(lib.smile_create_with_workspace(C.byref(desc), workspace.data_ptr(), nbytes, C.byref(self._h)),
                   "smile_create_with_workspace")

    @property
    def handle(self):
        return self._h

    def close(self):
        if self._h:
            load().smile_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def smile_gate_logits(ctx: Ctx, x, w_inter, w_intra, logits_inter, logits_intra, stream=None):
    _check(load().smile_gate_logits(ctx.handle, _ptr(x), _ptr(w_inter), _ptr(w_intra), _ptr(logits_inter),
                                    _ptr(logits_intra), _stream(stream)), "smile_gate_logits")


def smile_route_bilevel(ctx: Ctx, logits_inter, logits_intra, bias_inter, bias_intra, group_idx, local_idx,
                        pos_in_group, slot, gate, p_top, q_top, group_count, local_count, expert_count,
                        kept_count, p_sum, q_sum, stream=None):
    _check(load().smile_route_bilevel(ctx.handle, _ptr(logits_inter), _ptr(logits_intra), _ptr(bias_inter),
                                      _ptr(bias_intra), _ptr(group_idx), _ptr(local_idx), _ptr(pos_in_group),
                                      _ptr(slot), _ptr(gate), _ptr(p_top), _ptr(q_top), _ptr(group_count),
                                      _ptr(local_count), _ptr(expert_count), _ptr(kept_count), _ptr(p_sum),
                                      _ptr(q_sum), _stream(stream)), "smile_route_bilevel")


def smile_route_bilevel_static(desc: LayerDesc, logits_inter, logits_intra, bias_inter, bias_intra, group_idx,
                               local_idx, pos_in_group, slot, gate, p_top, q_top, group_count, local_count,
                               expert_count, kept_count, p_sum, q_sum, stream=None):
    """smile_route_bilevel without a ctx: the scratch memory is a fixed array inside the library."""
    _check(load().smile_route_bilevel_static(C.byref(desc), _ptr(logits_inter), _ptr(logits_intra),
                                             _ptr(bias_inter), _ptr(bias_intra), _ptr(group_idx), _ptr(local_idx),
                                             _ptr(pos_in_group), _ptr(slot), _ptr(gate), _ptr(p_top), _ptr(q_top),
                                             _ptr(group_count), _ptr(local_count), _ptr(expert_count),
                                             _ptr(kept_count), _ptr(p_sum), _ptr(q_sum), _stream(stream)),
           "smile_route_bilevel_static")


def smile_dispatch(ctx: Ctx, x, group_idx, local_idx, slot, xe, stream=None):
    _check(load().smile_dispatch(ctx.handle, _ptr(x), _ptr(group_idx), _ptr(local_idx), _ptr(slot), _ptr(xe),
                                 _stream(stream)), "smile_dispatch")


def smile_dispatch_hop1(ctx: Ctx, x, group_idx, pos_in_group, group_rows, xg, stream=None):
    _check(load().smile_dispatch_hop1(ctx.handle, _ptr(x), _ptr(group_idx), _ptr(pos_in_group), int(group_rows),
                                      _ptr(xg), _stream(stream)), "smile_dispatch_hop1")


def smile_dispatch_hop2(ctx: Ctx, xg, group_idx, local_idx, pos_in_group, slot, group_rows, xe, stream=None):
    _check(load().smile_dispatch_hop2(ctx.handle, _ptr(xg), _ptr(group_idx), _ptr(local_idx), _ptr(pos_in_group),
                                      _ptr(slot), int(group_rows), _ptr(xe), _stream(stream)), "smile_dispatch_hop2")


def smile_expert_ffn(ctx: Ctx, xe, kept_count, w1, b1, w2, b2, ye, stream=None):
    _check(load().smile_expert_ffn(ctx.handle, _ptr(xe), _ptr(kept_count), _ptr(w1), _ptr(b1), _ptr(w2), _ptr(b2),
                                   _ptr(ye), _stream(stream)), "smile_expert_ffn")


def smile_expert_ffn_up(ctx: Ctx, xe, kept_count, w1, b1, stream=None):
    _check(load().smile_expert_ffn_up(ctx.handle, _ptr(xe), _ptr(kept_count), _ptr(w1), _ptr(b1),
                                      _stream(stream)), "smile_expert_ffn_up")


def smile_expert_ffn_down(ctx: Ctx, kept_count, w2, b2, ye, stream=None):
    _check(load().smile_expert_ffn_down(ctx.handle, _ptr(kept_count), _ptr(w2), _ptr(b2), _ptr(ye),
                                        _stream(stream)), "smile_expert_ffn_down")


def smile_combine(ctx: Ctx, ye, group_idx, local_idx, slot, gate, y, stream=None):
    _check(load().smile_combine(ctx.handle, _ptr(ye), _ptr(group_idx), _ptr(local_idx), _ptr(slot), _ptr(gate),
                                _ptr(y), _stream(stream)), "smile_combine")


def smile_aux_loss(ctx: Ctx, group_count, local_count, p_sum, q_sum, out3, stream=None):
    _check(load().smile_aux_loss(ctx.handle, _ptr(group_count), _ptr(local_count), _ptr(p_sum), _ptr(q_sum),
                                 _ptr(out3), _stream(stream)), "smile_aux_loss")


def smile_layer_forward(ctx: Ctx, io: LayerIO, stream=None):
    _check(load().smile_layer_forward(ctx.handle, C.byref(io), _stream(stream)), "smile_layer_forward")


def torch_dtype(dtype):
    """torch storage type of a desc.dtype code or name."""
    import torch
    code = DTYPE[dtype] if isinstance(dtype, str) else int(dtype)
    return {0: torch.float32, 1: torch.bfloat16, 2: torch.float16}[code]


# ------------------------------------------------------------------ backward pass

def smile_backward_workspace_bytes(desc: LayerDesc) -> int:
    out = C.c_size_t(0)
    _check(load().smile_backward_workspace_bytes(C.byref(desc), C.byref(out)), "smile_backward_workspace_bytes")
    return int(out.value)


def smile_combine_backward(ctx: Ctx, dy, ye, group_idx, local_idx, slot, gate, dye, dgate, stream=None):
    _check(load().smile_combine_backward(ctx.handle, _ptr(dy), _ptr(ye), _ptr(group_idx), _ptr(local_idx), _ptr(slot),
                                         _ptr(gate), _ptr(dye), _ptr(dgate), _stream(stream)), "smile_combine_backward")


def smile_route_backward(ctx: Ctx, logits_inter, logits_intra, bias_inter, bias_intra, group_idx, local_idx, dgate,
                         group_count, local_count, dloss, dlp, dlq, stream=None):
    _check(load().smile_route_backward(ctx.handle, _ptr(logits_inter), _ptr(logits_intra), _ptr(bias_inter),
                                       _ptr(bias_intra), _ptr(group_idx), _ptr(local_idx), _ptr(dgate),
                                       _ptr(group_count), _ptr(local_count), float(dloss), _ptr(dlp), _ptr(dlq),
                                       _stream(stream)), "smile_route_backward")


def smile_expert_ffn_backward(ctx: Ctx, xe, kept_count, w1, w2, dye, dxe, dw1, dw2, workspace, h=None, pre=None,
                              stream=None):
    _check(load().smile_expert_ffn_backward(ctx.handle, _ptr(xe), _ptr(kept_count), _ptr(w1), _ptr(w2), _ptr(dye),
                                            _ptr(h), _ptr(pre), _ptr(dxe), _ptr(dw1), _ptr(dw2), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream)),
           "smile_expert_ffn_backward")


def smile_dispatch_backward(ctx: Ctx, dxe, group_idx, local_idx, slot, dlp, dlq, w_inter, w_intra, dx, stream=None):
    _check(load().smile_dispatch_backward(ctx.handle, _ptr(dxe), _ptr(group_idx), _ptr(local_idx), _ptr(slot),
                                          _ptr(dlp), _ptr(dlq), _ptr(w_inter), _ptr(w_intra), _ptr(dx),
                                          _stream(stream)), "smile_dispatch_backward")


def smile_gate_weights_backward(ctx: Ctx, x, dlp, dlq, dw_inter, dw_intra, workspace, stream=None):
    _check(load().smile_gate_weights_backward(ctx.handle, _ptr(x), _ptr(dlp), _ptr(dlq), _ptr(dw_inter),
                                              _ptr(dw_intra), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream(stream)),
           "smile_gate_weights_backward")


def smile_layer_backward(ctx: Ctx, io: BackwardIO, dloss, workspace, stream=None):
    _check(load().smile_layer_backward(ctx.handle, C.byref(io), float(dloss), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream(stream)),
           "smile_layer_backward")


@dataclass
class BackwardBuffers:
    """Intermediates and results of one backward pass as torch tensors on the GPU."""
    dye: object
    dgate: object
    dlp: object
    dlq: object
    dxe: object
    dx: object
    dw_inter: object
    dw_intra: object
    dw1: object
    dw2: object


def alloc_backward_buffers(desc: LayerDesc, device="cuda:0") -> BackwardBuffers:
    import torch
    T, d, F, n, m, Cap = desc.T, desc.d_model, desc.d_ff, desc.n_groups, desc.m_local, desc.capacity
    N = n * m
    st = torch_dtype(desc.dtype)
    f32 = torch.float32

    def e(shape, dt):
        return torch.empty(shape, dtype=dt, device=device)

    return BackwardBuffers(e((N, Cap, d), st), e((T,), f32), e((T, n), f32), e((T, m), f32), e((N, Cap, d), st),
                           e((T, d), st), e((n, d), f32), e((m, d), f32), e((N, F, d), st), e((N, d, F), st))


def make_backward_io(x, w_inter, w_intra, w1, w2, fwd: "LayerBuffers", dy, bwd: BackwardBuffers, bias_inter=None,
                     bias_intra=None, h=None, pre=None) -> BackwardIO:
    io = BackwardIO()
    for k, v in dict(x=x, w_inter=w_inter, w_intra=w_intra, w1=w1, w2=w2, bias_inter=bias_inter,
                     bias_intra=bias_intra, dy=dy, h=h, pre=pre).items():
        setattr(io, k, _ptr(v))
    for k in ("logits_inter", "logits_intra", "group_idx", "local_idx", "slot", "gate", "group_count", "local_count",
              "kept_count", "xe", "ye"):
        setattr(io, k, _ptr(getattr(fwd, k)))
    for k, v in bwd.__dict__.items():
        setattr(io, k, _ptr(v))
    return io


# ------------------------------------------------------------------ device buffers for one layer

@dataclass
class LayerBuffers:
    """All intermediates/outputs of one forward pass as torch tensors on the GPU."""
    logits_inter: object
    logits_intra: object
    group_idx: object
    local_idx: object
    pos_in_group: object
    slot: object
    gate: object
    p_top: object
    q_top: object
    group_count: object
    local_count: object
    expert_count: object
    kept_count: object
    p_sum: object
    q_sum: object
    xe: object
    ye: object
    y: object
    loss3: object


def alloc_buffers(desc: LayerDesc, device="cuda:0") -> LayerBuffers:
    import torch
    T, d, n, m, Cap = desc.T, desc.d_model, desc.n_groups, desc.m_local, desc.capacity
    N = n * m
    st = torch_dtype(desc.dtype)
    f32, i32 = torch.float32, torch.int32

    def e(shape, dt):
        return torch.empty(shape, dtype=dt, device=device)

    return LayerBuffers(
        e((T, n), f32), e((T, m), f32), e((T,), i32), e((T,), i32), e((T,), i32), e((T,), i32),
        e((T,), f32), e((T,), f32), e((T,), f32), e((n,), i32), e((max(m, 4),), i32)[:m], e((N,), i32),
        e((N,), i32), e((n,), f32), e((m,), f32), e((N, Cap, d), st), e((N, Cap, d), st), e((T, d), st),
        e((4,), f32)[:3])


def make_io(x, w_inter, w_intra, w1, w2, buf: LayerBuffers, b1=None, b2=None, bias_inter=None,
            bias_intra=None) -> LayerIO:
    io = LayerIO()
    for k, v in dict(x=x, w_inter=w_inter, w_intra=w_intra, w1=w1, b1=b1, w2=w2, b2=b2,
                     bias_inter=bias_inter, bias_intra=bias_intra).items():
        setattr(io, k, _ptr(v))
    for k, v in buf.__dict__.items():
        setattr(io, k, _ptr(v))
    io.h_save = None
    io.pre_save = None
    return io
