"""Shared pieces of the GPU parity tests: build one synthetic layer on the host, run the oracle, upload the
same bits, and compare under the rules below.

Comparison rules
  * routing: a token is "exempt" when the oracle's k-th and (k+1)-th logits differ by less than 1e-4; every
    other token must have the oracle's expert set, and the oracle's slot order wherever adjacent selected
    logits differ by at least 1e-4.  Weights are compared per expert (rtol 2e-5).
  * counts must equal the bincount of the GPU's own indices exactly, and differ from the oracle's by at most
    2 per exempt token in L1; with no exempt token they are identical.
  * perm must be the stable grouping of the GPU's indices, inv_perm its inverse.
  * floating-point outputs: max |gpu - ref| <= 1e-2 * max |ref|  (bf16 inputs, fp32 accumulation, one bf16
    rounding of the inner activation and one of the output).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

import oracle
from paper_2602_03495_amd import workloads as wl

GAP = 1e-4
OUT_TOL = 1e-2


@dataclass
class HostLayer:
    cfg: wl.LayerConfig
    gate_w: np.ndarray
    bias: Optional[np.ndarray]
    w1: np.ndarray
    w3: np.ndarray
    w2: np.ndarray
    shared: Optional[tuple] = None

    @property
    def shared_mode(self) -> int:
        return {"none": 0, "one": 1, "sigmoid": 2}[self.cfg.shared_gate] if self.cfg.n_shared else 0


def make_host_layer(cfg: wl.LayerConfig, layer: int = 0, with_bias: bool = True) -> HostLayer:
    w1, w3, w2 = wl.expert_weights(cfg, layer)
    return HostLayer(cfg, wl.gate_weights(cfg, layer), wl.gate_bias(cfg, layer) if with_bias else None, w1, w3, w2,
                     wl.shared_expert_weights(cfg, layer))


def exempt_tokens(logits: np.ndarray, k: int) -> np.ndarray:
    """Boolean [T]: oracle's k-th and (k+1)-th logits closer than GAP."""
    T, N = logits.shape
    if k >= N:
        return np.zeros(T, dtype=bool)
    srt = -np.sort(-logits.astype(np.float64), axis=1)
    return (srt[:, k - 1] - srt[:, k]) < GAP


def check_routing(lg, o_idx, o_w, o_counts, g_idx, g_w, g_counts, g_offsets, g_perm, g_inv, N, k):
    """Assert routing parity; returns the boolean exempt mask."""
    T = lg.shape[0]
    ex = exempt_tokens(lg, k)
    nex = int(ex.sum())
    assert g_idx.min() >= 0 and g_idx.max() < N
    assert all(len(set(r)) == k for r in g_idx[: min(T, 4096)])
    ok = ~ex
    # expert sets and per-expert weights
    o_sorted = np.sort(o_idx, axis=1)
    g_sorted = np.sort(g_idx, axis=1)
    assert np.array_equal(o_sorted[ok], g_sorted[ok]), "expert sets differ on non-exempt tokens"
    o_ord = np.argsort(o_idx, axis=1, kind="stable")
    g_ord = np.argsort(g_idx, axis=1, kind="stable")
    ow = np.take_along_axis(o_w, o_ord, 1)[ok]
    gw = np.take_along_axis(g_w, g_ord, 1)[ok]
    assert np.allclose(gw, ow, rtol=2e-5, atol=1e-7), float(np.abs(gw - ow).max())
    # slot order where the oracle's selected logits are well separated
    sel = np.take_along_axis(lg.astype(np.float64), o_idx.astype(np.int64), 1)
    sep = np.all((sel[:, :-1] - sel[:, 1:]) >= GAP, axis=1) if k > 1 else np.ones(T, bool)
    strict = ok & sep
    assert np.array_equal(o_idx[strict], g_idx[strict]), "slot order differs"
    # exempt tokens: the GPU may only swap experts whose logit is within GAP of the k-th
    for t in np.nonzero(ex)[0]:
        kth = np.sort(lg[t].astype(np.float64))[::-1][k - 1]
        diff = set(g_idx[t]) ^ set(o_idx[t])
        assert all(abs(float(lg[t, e]) - kth) < GAP for e in diff)
    # workload histogram
    assert np.array_equal(g_counts, np.bincount(g_idx.ravel(), minlength=N))
    assert int(np.abs(g_counts.astype(np.int64) - o_counts.astype(np.int64)).sum()) <= 2 * nex
    assert g_counts.sum() == T * k
    # offsets / permutation
    assert np.array_equal(g_offsets, np.concatenate([[0], np.cumsum(g_counts)]).astype(np.int32))
    want_perm = np.argsort(g_idx.ravel(), kind="stable").astype(np.int32)
    assert np.array_equal(g_perm, want_perm), "perm is not the stable grouping"
    inv = np.empty_like(want_perm)
    inv[want_perm] = np.arange(want_perm.size, dtype=np.int32)
    assert np.array_equal(g_inv, inv)
    return ex


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    scale = float(np.abs(ref).max())
    if scale == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got.astype(np.float64) - ref).max()) / scale


def sample_tokens(T: int, n: int, seed: int, extra=()) -> np.ndarray:
    rng = np.random.default_rng(seed)
    s = set(rng.choice(T, size=min(n, T), replace=False).tolist()) | set(int(x) for x in extra)
    return np.array(sorted(s), dtype=np.int32)


SENTINEL = 0x5A5A      # bf16 bits of a large finite value (1.5e16): a row that was not written still holds it


def run_layer(B, Lm, cfg, T, masks, ffn_path, draw=0):
    """One layer pass per mask through the library, compared with the oracle on the same bits: routing tables, every
    expert row of the masked-on experts, the layer output; rows of masked-off experts must be left untouched."""
    import torch
    _np = lambda t: t.cpu().numpy()
    hl = make_host_layer(cfg)
    h = wl.hidden_states(cfg, T, draw=draw)
    lg, o_idx, o_w, o_counts = oracle.route(h, hl.gate_w, hl.bias, cfg.k, cfg.norm_mode)
    dw = Lm.LayerWeights.upload(hl.gate_w, hl.bias, hl.w1, hl.w3, hl.w2, hl.shared)
    L = Lm.MoeLayer(cfg, T, ffn_path)
    hd = Lm.to_device_bf16(h)
    for mask in masks:
        md = None if mask is None else torch.from_numpy(mask).cuda()
        L.y.view(torch.int16).fill_(SENTINEL)
        out = L.forward(hd, dw, md)
        torch.cuda.synchronize()
        r = L.routing
        ex = check_routing(lg, o_idx, o_w, o_counts, _np(r.topk_idx), _np(r.topk_w), _np(r.counts), _np(r.offsets),
                           _np(r.perm), _np(r.inv_perm), cfg.N, cfg.k)
        keep = np.nonzero(~ex)[0].astype(np.int32)
        # expert rows, in the oracle's (token, slot) order
        y_ref = oracle.expert_rows(h, o_idx, hl.w1, hl.w3, hl.w2, mask, tokens=keep)
        y_bits = Lm.from_device_bf16(L.y)
        y_gpu = wl.bf16_bits_to_f32(y_bits)
        g_idx, inv = _np(r.topk_idx), _np(r.inv_perm).reshape(T, cfg.k)
        on = np.ones(cfg.N, bool) if mask is None else mask.astype(bool)
        for n, t in enumerate(keep):
            for s_o in range(cfg.k):
                e = o_idx[t, s_o]
                if not on[e]:
                    continue
                s_g = int(np.nonzero(g_idx[t] == e)[0][0])
                err = rel_err(y_gpu[inv[t, s_g]], y_ref[n, s_o])
                assert err <= OUT_TOL, (t, e, err)
        # rows of masked-off experts are not written (they keep the sentinel); rows of masked-on experts all are
        off_rows = ~on[np.sort(g_idx.ravel(), kind="stable")]          # permuted row p belongs to the p-th smallest expert id
        assert np.all(y_bits[off_rows] == SENTINEL), "a row of a masked-off expert was written"
        assert not np.any(np.all(y_bits[~off_rows] == SENTINEL, axis=1)), "a row of a masked-on expert was not written"
        # layer output
        ref = oracle.layer(h, o_idx, o_w, hl.w1, hl.w3, hl.w2, mask, hl.shared, hl.shared_mode, tokens=keep)
        got = wl.bf16_bits_to_f32(Lm.from_device_bf16(out))[keep]
        if np.abs(ref).max() == 0:
            assert np.all(got == 0)
        else:
            assert rel_err(got, ref) <= OUT_TOL, rel_err(got, ref)
    return L
