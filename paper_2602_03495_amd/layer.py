"""Device-side plumbing around the C ABI: uploads bf16 bit patterns, owns the output and workspace buffers
of one (layer shape, batch size) and issues the calls of one pass in order.  No arithmetic happens here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from . import binding as B
from .workloads import LayerConfig


def to_device_bf16(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 device tensor of the same shape (no value conversion)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def from_device_bf16(t: torch.Tensor) -> np.ndarray:
    """torch.bfloat16 tensor -> uint16 bit patterns on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


@dataclass
class LayerWeights:
    gate_w: torch.Tensor                 # [N,d] bf16
    gate_bias: Optional[torch.Tensor]    # [N] fp32
    w1: torch.Tensor                     # [N,I,d] bf16, packed by moe_pack_weights
    w3: torch.Tensor                     # [N,I,d] bf16, packed
    w2: torch.Tensor                     # [N,d,I] bf16, packed
    sw1: Optional[torch.Tensor] = None   # [S,Is,d] packed
    sw3: Optional[torch.Tensor] = None
    sw2: Optional[torch.Tensor] = None   # [S,d,Is] packed
    w_sg: Optional[torch.Tensor] = None  # [d] bf16 (sigmoid-gated shared expert)

    @staticmethod
    def upload(gate_w, gate_bias, w1, w3, w2, shared=None, device="cuda") -> "LayerWeights":
        """Upload row-major bf16 bit patterns and pack the expert matrices on the device (one time)."""
        def packed(bits):
            return B.moe_pack_weights(to_device_bf16(bits, device))

        lw = LayerWeights(to_device_bf16(gate_w, device),
                          None if gate_bias is None else torch.from_numpy(np.asarray(gate_bias, np.float32)).to(device),
                          packed(w1), packed(w3), packed(w2))
        if shared is not None:
            sw1, sw3, sw2, w_sg = shared
            lw.sw1, lw.sw3, lw.sw2 = (packed(a) for a in (sw1, sw3, sw2))
            lw.w_sg = None if w_sg is None else to_device_bf16(w_sg, device)
        torch.cuda.synchronize()
        return lw


class MoeLayer:
    """Buffers and call sequence of one MoE layer pass for a fixed batch size T."""

    def __init__(self, cfg: LayerConfig, T: int, ffn_path: int = B.FFN_AUTO, device="cuda"):
        self.cfg, self.T, self.device = cfg, T, device
        self.shape = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I, ffn_path)
        self.ws = B.alloc_workspace(self.shape, device)
        self.routing = B.alloc_routing(self.shape, device)
        self.y = torch.empty((T * cfg.k, cfg.d), dtype=torch.bfloat16, device=device)
        self.out = torch.empty((T, cfg.d), dtype=torch.bfloat16, device=device)
        self.pred_counts = torch.empty(cfg.N, dtype=torch.int32, device=device)
        self.n_shared = cfg.n_shared
        if cfg.n_shared:
            S = cfg.n_shared
            self.sshape = B.shape(T, cfg.d, S, S, cfg.I_shared, ffn_path)
            self.sws = B.alloc_workspace(self.sshape, device)
            i32 = dict(dtype=torch.int32, device=device)
            self.s_counts, self.s_offsets = torch.empty(S, **i32), torch.empty(S + 1, **i32)
            self.s_perm = torch.empty(T * S, **i32)
            self.shared_y = torch.empty((S * T, cfg.d), dtype=torch.bfloat16, device=device)
            self.shared_scale = (torch.empty(T, dtype=torch.float32, device=device)
                                 if cfg.shared_gate == "sigmoid" else None)
            B.moe_dense_route(self.sshape, self.s_counts, self.s_offsets, self.s_perm)

    def route(self, h, w: LayerWeights, bias=None):
        b = w.gate_bias if bias is None else bias
        return B.moe_route(self.shape, h, w.gate_w, b, self.cfg.norm_mode, self.routing, self.ws)

    def route_predict(self, h, w: LayerWeights, res_vec, next_w: LayerWeights, p: int, top_experts, bias=None, next_bias=None):
        """Routing of this layer and workload prediction of the next in one call."""
        b = w.gate_bias if bias is None else bias
        nb = next_w.gate_bias if next_bias is None else next_bias
        return B.moe_route_predict(self.shape, h, w.gate_w, b, self.cfg.norm_mode, self.routing, res_vec, next_w.gate_w, nb, p,
                                   self.pred_counts, top_experts, self.ws)

    def expert_ffn(self, h, w: LayerWeights, mask):
        r = self.routing
        return B.moe_expert_ffn(self.shape, h, r.perm, r.offsets, r.counts, w.w1, w.w3, w.w2, mask, self.y, self.ws)

    def shared_ffn(self, h, w: LayerWeights):
        if self.shared_scale is not None:
            B.moe_shared_gate(self.sshape, h, w.w_sg, self.shared_scale)
        return B.moe_expert_ffn(self.sshape, h, self.s_perm, self.s_offsets, self.s_counts, w.sw1, w.sw3, w.sw2, None,
                                self.shared_y, self.sws)

    def combine(self, mask, with_shared=True):
        r = self.routing
        sy = self.shared_y if (self.n_shared and with_shared) else None
        sc = self.shared_scale if (self.n_shared and with_shared) else None
        return B.moe_combine(self.shape, self.y, r.topk_idx, r.topk_w, r.inv_perm, mask, sy, self.n_shared if sy is not None else 0,
                             sc, self.out)

    def forward(self, h, w: LayerWeights, mask, bias=None, with_shared=True):
        """route -> expert FFN (masked) -> [shared experts] -> combine; returns out [T,d] bf16."""
        self.route(h, w, bias)
        self.expert_ffn(h, w, mask)
        if self.n_shared and with_shared:
            self.shared_ffn(h, w)
        return self.combine(mask, with_shared)

    def predict(self, h, res_vec, next_w: LayerWeights, p: int, top_experts, next_bias=None, ws=None):
        """ws: a workspace of its own when the prediction runs concurrently with this layer's other calls."""
        b = next_w.gate_bias if next_bias is None else next_bias
        return B.moe_predict_workload(self.shape, h, res_vec, next_w.gate_w, b, p, self.pred_counts, top_experts,
                                      self.ws if ws is None else ws)
