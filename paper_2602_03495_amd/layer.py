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
    xw1: Optional[torch.Tensor] = None   # [N+S',I,d] packed: routed experts, then the shared ones cut into inner blocks of I
    xw3: Optional[torch.Tensor] = None
    xw2: Optional[torch.Tensor] = None   # [N+S',d,I] packed

    @staticmethod
    def upload(gate_w, gate_bias, w1, w3, w2, shared=None, device="cuda", merge_shared=False) -> "LayerWeights":
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
            S, Is, d = sw1.shape
            I = w1.shape[1]
            if merge_shared and Is % I == 0:
                # a shared expert of inner size m*I as m experts of inner size I, stored after the routed ones
                m = Is // I
                c1, c3 = sw1.reshape(S * m, I, d), sw3.reshape(S * m, I, d)
                c2 = np.ascontiguousarray(sw2.reshape(S, d, m, I).transpose(0, 2, 1, 3)).reshape(S * m, d, I)
                lw.xw1, lw.xw3, lw.xw2 = (packed(np.concatenate(p)) for p in ((w1, c1), (w3, c3), (w2, c2)))
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
        self.n_merged = 0
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
            if cfg.I_shared % cfg.I == 0:
                # the same layer as N + n_merged experts with k + n_merged slots per token (one grouped launch for all)
                Sm = S * (cfg.I_shared // cfg.I)
                if cfg.N + Sm <= B.MAX_EXPERTS and cfg.k + Sm <= B.MAX_TOPK:
                    self.n_merged = Sm
                    self.xshape = B.shape(T, cfg.d, cfg.N + Sm, cfg.k + Sm, cfg.I, ffn_path)
                    self.xws = B.alloc_workspace(self.xshape, device)
                    self.xrouting = B.alloc_routing(self.xshape, device)
                    self.xy = torch.empty((T * (cfg.k + Sm), cfg.d), dtype=torch.bfloat16, device=device)

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

    def merged_mask(self, mask) -> torch.Tensor:
        """mask [N] over the routed experts (None = all on) -> mask [N + n_merged] with the shared experts on."""
        on = torch.ones(self.cfg.N + self.n_merged, dtype=torch.uint8, device=self.device)
        if mask is not None:
            on[: self.cfg.N].copy_(mask)
        return on

    def forward_merged(self, h, w: LayerWeights, xmask, bias=None):
        """The same layer with the shared experts inside the grouped launches: route -> append the shared slots ->
        one expert FFN over routed and shared experts -> combine.  xmask: merged_mask(mask), or None for all on."""
        if not self.n_merged or w.xw1 is None:
            raise B.MoeError("this layer has no shared experts that split into experts of the routed inner size")
        b = w.gate_bias if bias is None else bias
        x = B.moe_route_shared(self.shape, self.n_merged, h, w.gate_w, b, self.cfg.norm_mode,
                               w.w_sg if self.shared_scale is not None else None, self.routing, self.xrouting, self.ws)
        B.moe_expert_ffn(self.xshape, h, x.perm, x.offsets, x.counts, w.xw1, w.xw3, w.xw2, xmask, self.xy, self.xws)
        return B.moe_combine(self.xshape, self.xy, x.topk_idx, x.topk_w, x.inv_perm, xmask, None, 0, None, self.out)

    def predict(self, h, res_vec, next_w: LayerWeights, p: int, top_experts, next_bias=None, ws=None):
        """ws: a workspace of its own when the prediction runs concurrently with this layer's other calls."""
        b = next_w.gate_bias if next_bias is None else next_bias
        return B.moe_predict_workload(self.shape, h, res_vec, next_w.gate_w, b, p, self.pred_counts, top_experts,
                                      self.ws if ws is None else ws)
