"""Device-side set-up of one layer from a workloads.LayerConfig: uploads the seeded inputs,
allocates the buffers and calls the six library entry points in order.  Marshalling only."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from . import binding as B
from . import workloads as wl


def to_device(a: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """Host float32 array (values representable in `dtype`) -> device tensor of the storage type."""
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).to(device).view(torch.bfloat16).reshape(a.shape)
    if dtype == "f16":
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).astype(np.float16)).to(device)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host numpy (bf16 widened to float32, exactly)."""
    if t.dtype == torch.bfloat16:
        return wl.bf16_bits_to_f32(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)).reshape(t.shape)
    if t.dtype == torch.float16:
        return t.cpu().numpy().astype(np.float32)
    return t.cpu().numpy()


class GpuLayer:
    """One layer resident on the GPU: inputs, weights, buffers and the library ctx."""

    def __init__(self, cfg: wl.LayerConfig, device="cuda:0", alpha=0.005, beta=0.005, workers=8,
                 own_workspace=False):
        self.cfg = cfg
        self.device = device
        self.desc = B.make_desc(cfg.T, cfg.d_model, cfg.d_ff, cfg.n_groups, cfg.m_local, cfg.capacity,
                                cfg.dtype, cfg.act, alpha, beta, cfg.group_capacity)
        self.x = to_device(wl.gen_tokens(cfg), cfg.dtype, device)
        wi, wq = wl.gen_router_weights(cfg)
        self.w_inter, self.w_intra = to_device(wi, cfg.dtype, device), to_device(wq, cfg.dtype, device)
        st = B.torch_dtype(cfg.dtype)
        self.w1 = torch.empty((cfg.N, cfg.d_ff, cfg.d_model), dtype=st, device=device)
        self.w2 = torch.empty((cfg.N, cfg.d_model, cfg.d_ff), dtype=st, device=device)
        with ThreadPoolExecutor(max_workers=workers) as pool:
            for e, (a, b) in enumerate(pool.map(lambda e: wl.gen_expert_weights(cfg, e), range(cfg.N))):
                self.w1[e].copy_(to_device(a, cfg.dtype, device))
                self.w2[e].copy_(to_device(b, cfg.dtype, device))
        bi, bq = wl.gen_routing_biases(cfg)
        self.bias_inter = None if bi is None else torch.from_numpy(bi).to(device)
        self.bias_intra = None if bq is None else torch.from_numpy(bq).to(device)
        self.b1 = self.b2 = None
        if own_workspace:
            nbytes = B.smile_workspace_bytes(self.desc)
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
            self.ctx = B.Ctx(self.desc, self.workspace)
        else:
            self.ctx = B.Ctx(self.desc)
        self.buf = B.alloc_buffers(self.desc, device)
        self.io = B.make_io(self.x, self.w_inter, self.w_intra, self.w1, self.w2, self.buf, self.b1, self.b2,
                            self.bias_inter, self.bias_intra)
        self.io_fused = B.make_io(self.x, self.w_inter, self.w_intra, self.w1, self.w2, self.buf, self.b1, self.b2,
                                  self.bias_inter, self.bias_intra)
        self.io_fused.xe = None
        self.io_fused.ye = None

    # the six steps, one call each
    def gate_logits(self):
        b = self.buf
        B.smile_gate_logits(self.ctx, self.x, self.w_inter, self.w_intra, b.logits_inter, b.logits_intra)

    def route(self):
        b = self.buf
        B.smile_route_bilevel(self.ctx, b.logits_inter, b.logits_intra, self.bias_inter, self.bias_intra,
                              b.group_idx, b.local_idx, b.pos_in_group, b.slot, b.gate, b.p_top, b.q_top,
                              b.group_count, b.local_count, b.expert_count, b.kept_count, b.p_sum, b.q_sum)

    def dispatch(self):
        b = self.buf
        B.smile_dispatch(self.ctx, self.x, b.group_idx, b.local_idx, b.slot, b.xe)

    def expert_ffn(self):
        b = self.buf
        B.smile_expert_ffn(self.ctx, b.xe, b.kept_count, self.w1, self.b1, self.w2, self.b2, b.ye)

    def combine(self):
        b = self.buf
        B.smile_combine(self.ctx, b.ye, b.group_idx, b.local_idx, b.slot, b.gate, b.y)

    def aux_loss(self):
        b = self.buf
        B.smile_aux_loss(self.ctx, b.group_count, b.local_count, b.p_sum, b.q_sum, b.loss3)

    def forward_steps(self):
        self.gate_logits(); self.route(); self.dispatch(); self.expert_ffn(); self.combine(); self.aux_loss()

    def forward(self):
        """All six steps through the single chained entry point (expert buffers materialised)."""
        B.smile_layer_forward(self.ctx, self.io)

    def enable_saved_activations(self):
        """Training mode of the chained entry points: the forward pass also stores h and the pre-activation
        ([N,C,F] each) and the backward pass reads them instead of recomputing."""
        st = B.torch_dtype(self.cfg.dtype)
        shape = (self.cfg.N, self.cfg.capacity, self.cfg.d_ff)
        self.h_save = torch.empty(shape, dtype=st, device=self.device)
        self.pre_save = torch.empty(shape, dtype=st, device=self.device)
        for io in (self.io, self.io_fused):
            io.h_save = self.h_save.data_ptr()
            io.pre_save = self.pre_save.data_ptr()

    def forward_fused(self):
        """The chained entry point without expert buffers: permutations fused into the expert GEMMs."""
        B.smile_layer_forward(self.ctx, self.io_fused)

    # ---- backward pass (buffers and scratch memory are allocated on first use)
    def prepare_backward(self, dy):
        """dy: the upstream gradient of y as a host float32 array [T, d] (values representable in the dtype)."""
        self.dy = to_device(dy, self.cfg.dtype, self.device)
        if getattr(self, "bwd", None) is None:
            self.bwd = B.alloc_backward_buffers(self.desc, self.device)
            nbytes = B.smile_backward_workspace_bytes(self.desc)
            self.bwd_workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.bwd_io = B.make_backward_io(self.x, self.w_inter, self.w_intra, self.w1, self.w2, self.buf, self.dy,
                                         self.bwd, self.bias_inter, self.bias_intra,
                                         getattr(self, "h_save", None), getattr(self, "pre_save", None))

    def backward_steps(self, dloss=1.0):
        b, g = self.buf, self.bwd
        B.smile_combine_backward(self.ctx, self.dy, b.ye, b.group_idx, b.local_idx, b.slot, b.gate, g.dye, g.dgate)
        B.smile_route_backward(self.ctx, b.logits_inter, b.logits_intra, self.bias_inter, self.bias_intra,
                               b.group_idx, b.local_idx, g.dgate, b.group_count, b.local_count, dloss, g.dlp, g.dlq)
        B.smile_expert_ffn_backward(self.ctx, b.xe, b.kept_count, self.w1, self.w2, g.dye, g.dxe, g.dw1, g.dw2,
                                    self.bwd_workspace, getattr(self, "h_save", None), getattr(self, "pre_save", None))
        B.smile_dispatch_backward(self.ctx, g.dxe, b.group_idx, b.local_idx, b.slot, g.dlp, g.dlq, self.w_inter,
                                  self.w_intra, g.dx)
        B.smile_gate_weights_backward(self.ctx, self.x, g.dlp, g.dlq, g.dw_inter, g.dw_intra, self.bwd_workspace)

    def backward(self, dloss=1.0):
        """The five backward steps through the single chained entry point."""
        B.smile_layer_backward(self.ctx, self.bwd_io, dloss, self.bwd_workspace)

    def close(self):
        torch.cuda.synchronize()
        self.ctx.close()
