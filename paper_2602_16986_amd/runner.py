"""Places a synthetic workload on the GPU and drives the library's entry points over it.

Marshalling only: tensors are uploaded once, every computation is a call into the C ABI.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as hb
from .workloads import Workload


def _dev(x: np.ndarray, dtype: str, device) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x))
    return t.to(device=device, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)


class DeviceWorkload:
    """Device-resident copy of a Workload plus output and scratch buffers."""

    def __init__(self, w: Workload, device="cuda:0", fused_qkvu: bool = False, bias_grad: bool = False):
        self.w = w
        self.device = torch.device(device)
        dt = w.dtype
        if fused_qkvu:
            # one [T, 4*H*d] buffer holding U|V|Q|K, the layout the layer's first projection produces
            fused = np.concatenate([w.u.reshape(w.T, -1), w.v.reshape(w.T, -1), w.q.reshape(w.T, -1),
                                    w.k.reshape(w.T, -1)], axis=1)
            self.fused = _dev(fused, dt, self.device)
            D = w.H * w.d
            self.u, self.v, self.q, self.k = (self.fused[:, i * D:(i + 1) * D].view(w.T, w.H, w.d) for i in range(4))
        else:
            self.q, self.k, self.v, self.u = (_dev(x, dt, self.device) for x in (w.q, w.k, w.v, w.u))
        # the gated norm takes contiguous [T, H*d] rows
        self.u_rows = self.u if self.u.is_contiguous() else self.u.contiguous()
        self.dout = _dev(w.dout, dt, self.device)
        self.dy = _dev(w.dy, dt, self.device)
        self.offsets = torch.from_numpy(w.offsets).to(self.device)
        self.num_targets = None if w.num_targets is None else torch.from_numpy(w.num_targets).to(self.device)
        self.table = None if w.table is None else torch.from_numpy(w.table).to(self.device)
        self.bounds = None if w.bounds is None else torch.from_numpy(w.bounds).to(self.device)
        self.gamma = torch.from_numpy(w.gamma).to(self.device)
        self.out = torch.empty_like(self.dout)
        self.y = torch.empty_like(self.dout)
        if fused_qkvu:
            # gradients land in one [T, 4*H*d] buffer too (dU|dV|dQ|dK), no concatenation afterwards
            self.dfused = torch.empty_like(self.fused)
            D = w.H * w.d
            _, self.dv, self.dq, self.dk = (self.dfused[:, i * D:(i + 1) * D].view(w.T, w.H, w.d) for i in range(4))
        else:
            self.dq, self.dk, self.dv = (torch.empty_like(self.dout) for _ in range(3))
        self.dattn, self.du = torch.empty_like(self.dout), torch.empty_like(self.dout)
        self.dgamma = torch.empty(w.H * w.d, dtype=torch.float32, device=self.device)
        self.mean = torch.empty(w.T, dtype=torch.float32, device=self.device)
        self.rstd = torch.empty(w.T, dtype=torch.float32, device=self.device)
        # optional gradient of the bias table, written by the attention backward
        self.dtable = torch.empty_like(self.table) if (bias_grad and self.table is not None) else None
        self.problem = hb.AttnProblem(self.q, self.k, self.v, self.out, self.offsets, max_seqlen=w.max_seqlen,
                                      seq_offsets_host=w.offsets, num_targets=self.num_targets,
                                      local_window=w.K1, global_prefix=w.K2, alpha=w.alpha, inv_n=1.0 / w.N,
                                      rab_table=self.table, rab_bounds=self.bounds, d_rab_table=self.dtable)
        self.ws_fwd = hb.new_workspace(hb.hstu_attn_workspace_bytes(self.problem, False), self.device)
        self.ws_bwd = hb.new_workspace(hb.hstu_attn_workspace_bytes(self.problem, True), self.device)
        self.ws_norm = hb.new_workspace(hb.hstu_gated_norm_bwd_workspace_bytes(w.T, w.H * w.d), self.device)

    # each method is one C-ABI call
    def attn_fwd(self, stream=None):
        hb.hstu_attn_fwd(self.problem, self.q, self.k, self.v, self.out, self.ws_fwd, stream)
        return self.out

    def attn_bwd(self, dout=None, stream=None):
        hb.hstu_attn_bwd(self.problem, self.q, self.k, self.v, self.dout if dout is None else dout,
                         self.dq, self.dk, self.dv, self.ws_bwd, stream)
        return self.dq, self.dk, self.dv

    def norm_fwd(self, attn=None, stream=None):
        hb.hstu_gated_norm_fwd(self.out if attn is None else attn, self.u_rows, self.gamma, None, self.w.eps, self.y,
                               self.mean, self.rstd, stream)
        return self.y

    def norm_bwd(self, attn=None, stream=None):
        hb.hstu_gated_norm_bwd(self.dy, self.out if attn is None else attn, self.u_rows, self.gamma, None, self.w.eps,
                               self.dattn, self.du, self.dgamma, None, self.ws_norm, stream)
        return self.dattn, self.du, self.dgamma

    def layer_step(self, stream=None):
        """The whole hot path once: attention forward, gated norm forward, gated norm backward,
        attention backward (fed by the gated norm's dA)."""
        self.attn_fwd(stream)
        self.norm_fwd(stream=stream)
        self.norm_bwd(stream=stream)
        self.attn_bwd(dout=self.dattn, stream=stream)


class DeviceLayer:
    """Device-resident copy of a LayerCase (token rows, weights) plus the buffers of hstu_layer_fwd / hstu_layer_bwd."""

    def __init__(self, c, device="cuda:0", bias_grad: bool = False, fp8: bool = False):
        assert c.dtype == "bf16"
        self.c = c
        self.device = dev = torch.device(device)
        HD = c.H * c.d
        self.z, self.w1, self.w2, self.dout = (_dev(x, "bf16", dev) for x in (c.z, c.w1, c.w2, c.dout))
        self.norm_w = torch.from_numpy(c.norm_w).to(dev)
        self.gated_norm_w = torch.from_numpy(c.gated_norm_w).to(dev)
        self.offsets = torch.from_numpy(c.offsets).to(dev)
        self.num_targets = None if c.num_targets is None else torch.from_numpy(c.num_targets).to(dev)
        self.table = None if c.table is None else torch.from_numpy(c.table).to(dev)
        self.bounds = None if c.bounds is None else torch.from_numpy(c.bounds).to(dev)
        self.dtable = torch.empty_like(self.table) if (bias_grad and self.table is not None) else None
        # forward outputs: the layer output and the tensors saved for the backward
        self.out = torch.empty_like(self.z)
        self.u_saved = torch.empty(c.T, HD, dtype=torch.bfloat16, device=dev)
        self.attn_saved = torch.empty(c.T, HD, dtype=torch.bfloat16, device=dev)
        self.mean = torch.empty(c.T, dtype=torch.float32, device=dev)
        self.rstd = torch.empty(c.T, dtype=torch.float32, device=dev)
        # backward outputs
        self.dz = torch.empty_like(self.z)
        self.d_norm_w = torch.empty(c.E, dtype=torch.float32, device=dev)
        self.d_w1 = torch.empty(4 * HD, c.E, dtype=torch.float32, device=dev)
        self.d_gated_norm_w = torch.empty(HD, dtype=torch.float32, device=dev)
        self.d_w2 = torch.empty(c.E, HD, dtype=torch.float32, device=dev)
        fp8_args = {}
        if fp8:   # weights quantised once, row-wise (one scale per output feature), by the library's own quantiser
            self.w1_q = torch.empty(self.w1.shape, dtype=torch.uint8, device=dev)
            self.w1_scale = torch.empty(self.w1.shape[0], dtype=torch.float32, device=dev)
            self.w2_q = torch.empty(self.w2.shape, dtype=torch.uint8, device=dev)
            self.w2_scale = torch.empty(self.w2.shape[0], dtype=torch.float32, device=dev)
            hb.hstu_norm_quant_fp8(self.w1, None, None, None, 0.0, self.w1_q, self.w1_scale)
            hb.hstu_norm_quant_fp8(self.w2, None, None, None, 0.0, self.w2_q, self.w2_scale)
            fp8_args = dict(w1_q=self.w1_q, w1_scale=self.w1_scale, w2_q=self.w2_q, w2_scale=self.w2_scale)
        self.problem = hb.LayerProblem(num_heads=c.H, head_dim=c.d, embed_dim=c.E, total_tokens=c.T, seq_offsets=self.offsets,
                                       max_seqlen=c.max_seqlen, norm_w=self.norm_w, w1=self.w1, gated_norm_w=self.gated_norm_w,
                                       w2=self.w2, num_targets=self.num_targets, local_window=c.K1, global_prefix=c.K2,
                                       alpha=c.alpha, inv_n=1.0 / c.N, rab_table=self.table, rab_bounds=self.bounds,
                                       d_rab_table=self.dtable, norm_eps=c.eps, gated_norm_eps=c.eps, **fp8_args)
        self.ws_fwd = hb.new_workspace(hb.hstu_layer_workspace_bytes(self.problem, False), dev)
        self.ws_bwd = hb.new_workspace(hb.hstu_layer_workspace_bytes(self.problem, True), dev)

    def fwd(self, stream=None):
        hb.hstu_layer_fwd(self.problem, self.z, self.out, self.u_saved, self.attn_saved, self.mean, self.rstd, self.ws_fwd, stream)
        return self.out

    def bwd(self, stream=None):
        hb.hstu_layer_bwd(self.problem, self.z, self.u_saved, self.attn_saved, self.mean, self.rstd, self.dout, self.dz,
                          self.d_norm_w, self.d_w1, self.d_gated_norm_w, self.d_w2, self.ws_bwd, stream)
        return self.dz, self.d_norm_w, self.d_w1, self.d_gated_norm_w, self.d_w2

    def step(self, stream=None):
        self.fwd(stream)
        self.bwd(stream)
