"""Seeded synthetic inputs for the MoE expert-layer path.

This module only *draws numbers*: hidden states, gate and expert weights,
gate biases, expert masks and residual drifts with the shapes of the models in
the paper's Table "config_of_moe" (DeepSeek-V2-Lite, Qwen3-30B-A3B,
Mixtral-8x7B) and of the Qwen1.5-MoE layer used in its motivation section.
It holds none of the layer's arithmetic (no gate, no softmax, no FFN), so the
CPU oracle and the HIP library can both be fed from it without sharing code.

Every tensor is produced by a counter-based generator (Philox) keyed by
``(seed, stream)``; the same key always yields the same bits.  Floating-point
tensors are rounded once to bfloat16 (round to nearest even) and handed out as
``uint16`` bit patterns, which is what both consumers read.

The paper's own inputs (C4 prompts, Wikitext calibration sequences, trained
checkpoints; Section "Experimental Setup") are not available; these draws stand
in for their shapes and routing skew only.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

NORM_NONE = 0    # G(x)_i = softmax over all N experts, taken at the selected ones (Eq. 1 literally)
NORM_RENORM = 1  # the k selected scores divided by their sum

# stream ids inside one config's seed space
S_HIDDEN, S_GATE, S_BIAS, S_EXPERTS, S_MASK, S_RES, S_SHARED = range(7)


@dataclass(frozen=True)
class LayerConfig:
    """Shape and input laws of one synthetic MoE layer."""
    cfg_id: int
    name: str
    d: int              # hidden size
    N: int              # routed experts
    k: int              # experts per token
    I: int              # expert SwiGLU inner size
    norm_mode: int
    bias_law: str       # "normal" | "zipf"
    zipf_s: float = 0.0
    n_shared: int = 0   # always-on shared experts
    I_shared: int = 0   # their inner size
    shared_gate: str = "none"   # "none" | "one" (weight 1) | "sigmoid" (sigmoid(x . w_sg))
    n_layers: int = 1

    @property
    def seed(self) -> int:
        return 1000 * self.cfg_id


CONFIGS: Dict[str, LayerConfig] = {
    "tiny": LayerConfig(1, "tiny", d=256, N=8, k=2, I=512, norm_mode=NORM_RENORM, bias_law="normal"),
    "mixtral": LayerConfig(2, "mixtral", d=4096, N=8, k=2, I=14336, norm_mode=NORM_RENORM,
                           bias_law="zipf", zipf_s=1.1),
    "deepseek": LayerConfig(3, "deepseek", d=2048, N=64, k=6, I=1408, norm_mode=NORM_NONE,
                            bias_law="zipf", zipf_s=1.2, n_shared=2, I_shared=1408, shared_gate="one"),
    "qwen15": LayerConfig(4, "qwen15", d=2048, N=60, k=4, I=1408, norm_mode=NORM_RENORM,
                          bias_law="zipf", zipf_s=1.1, n_shared=1, I_shared=5632, shared_gate="sigmoid"),
    "qwen3": LayerConfig(5, "qwen3", d=2048, N=128, k=8, I=768, norm_mode=NORM_RENORM,
                         bias_law="zipf", zipf_s=1.1, n_layers=48),
}


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of ``cfg`` with some sizes replaced (down-scaled test shapes)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# raw draws and bf16 packing
# --------------------------------------------------------------------------

def _rng(seed: int, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 8) + stream, sub]))


def normal_f32(seed: int, stream: int, shape, var: float = 1.0, sub: int = 0) -> np.ndarray:
    """N(0, var) draws, float32."""
    x = _rng(seed, stream, sub).standard_normal(shape, dtype=np.float32)
    if var != 1.0:
        x *= np.float32(np.sqrt(var))
    return x


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed: int, stream: int, shape, var: float = 1.0, sub: int = 0) -> np.ndarray:
    return to_bf16_bits(normal_f32(seed, stream, shape, var, sub))


def _stacked_bf16(seed: int, stream: int, n: int, shape, var: float, sub0: int = 0) -> np.ndarray:
    """``n`` independent N(0,var) bf16 tensors of ``shape`` stacked on axis 0 (one Philox sub-stream each)."""
    out = np.empty((n,) + tuple(shape), dtype=np.uint16)

    def fill(i):
        out[i] = normal_bf16(seed, stream, shape, var, sub0 + i)

    if n * int(np.prod(shape)) < (1 << 22):
        for i in range(n):
            fill(i)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(n)))
    return out


# --------------------------------------------------------------------------
# tensors of one layer
# --------------------------------------------------------------------------

def hidden_states(cfg: LayerConfig, T: int, draw: int = 0) -> np.ndarray:
    """[T, d] bf16 bits, N(0,1).  ``draw`` selects an independent batch."""
    return normal_bf16(cfg.seed, S_HIDDEN, (T, cfg.d), 1.0, sub=draw)


def gate_weights(cfg: LayerConfig, layer: int = 0) -> np.ndarray:
    """[N, d] bf16 bits, N(0, 1/d): row e is column e of the paper's W_g (d x N)."""
    return normal_bf16(cfg.seed, S_GATE, (cfg.N, cfg.d), 1.0 / cfg.d, sub=layer)


def zipf_bias(N: int, s: float, rng: np.random.Generator) -> np.ndarray:
    """b_e = -s ln(rank_e) with ranks a random permutation of 1..N, shifted to zero mean, so that
    the prior share of expert e is proportional to rank_e^-s."""
    ranks = rng.permutation(N) + 1
    b = -s * np.log(ranks.astype(np.float64))
    return (b - b.mean()).astype(np.float32)


def gate_bias(cfg: LayerConfig, layer: int = 0) -> np.ndarray:
    """[N] float32 per-expert logit bias that skews the workloads."""
    rng = _rng(cfg.seed, S_BIAS, layer)
    if cfg.bias_law == "normal":
        return rng.standard_normal(cfg.N, dtype=np.float32)
    if cfg.bias_law == "zipf":
        return zipf_bias(cfg.N, cfg.zipf_s, rng)
    raise ValueError(cfg.bias_law)


def ar1_bias_path(cfg: LayerConfig, layer: int, steps: int, rho: float = 0.9, sigma: float = 1.0) -> np.ndarray:
    """[steps, N] float32: b_t = mu + rho (b_{t-1} - mu) + sqrt(1-rho^2) sigma xi_t around the Zipf mean mu
    (temporally correlated routing of a decode run), started from its stationary law."""
    mu = gate_bias(cfg, layer).astype(np.float64)
    rng = _rng(cfg.seed, S_BIAS, 100000 + layer)
    out = np.empty((steps, cfg.N), dtype=np.float64)
    dev = sigma * rng.standard_normal(cfg.N)
    for t in range(steps):
        if t > 0:
            dev = rho * dev + np.sqrt(1.0 - rho * rho) * sigma * rng.standard_normal(cfg.N)
        out[t] = mu + dev
    return out.astype(np.float32)


def expert_weights(cfg: LayerConfig, layer: int = 0):
    """(w1 [N,I,d], w3 [N,I,d], w2 [N,d,I]) bf16 bits; N(0,1/d) for w1, w3 and N(0,1/I) for w2."""
    base = 3 * cfg.N * layer
    w1 = _stacked_bf16(cfg.seed, S_EXPERTS, cfg.N, (cfg.I, cfg.d), 1.0 / cfg.d, base)
    w3 = _stacked_bf16(cfg.seed, S_EXPERTS, cfg.N, (cfg.I, cfg.d), 1.0 / cfg.d, base + cfg.N)
    w2 = _stacked_bf16(cfg.seed, S_EXPERTS, cfg.N, (cfg.d, cfg.I), 1.0 / cfg.I, base + 2 * cfg.N)
    return w1, w3, w2


def shared_expert_weights(cfg: LayerConfig, layer: int = 0):
    """(w1 [S,Is,d], w3 [S,Is,d], w2 [S,d,Is], w_sg [d] or None) for the always-on shared experts."""
    if cfg.n_shared == 0:
        return None
    S, Is = cfg.n_shared, cfg.I_shared
    base = (3 * S + 1) * layer
    w1 = _stacked_bf16(cfg.seed, S_SHARED, S, (Is, cfg.d), 1.0 / cfg.d, base)
    w3 = _stacked_bf16(cfg.seed, S_SHARED, S, (Is, cfg.d), 1.0 / cfg.d, base + S)
    w2 = _stacked_bf16(cfg.seed, S_SHARED, S, (cfg.d, Is), 1.0 / Is, base + 2 * S)
    w_sg = None
    if cfg.shared_gate == "sigmoid":
        w_sg = normal_bf16(cfg.seed, S_SHARED, (cfg.d,), 1.0 / cfg.d, base + 3 * S)
    return w1, w3, w2, w_sg


# --------------------------------------------------------------------------
# expert masks (the paper's G vector: which routed experts this GPU computes)
# --------------------------------------------------------------------------

def mask_lower(N: int, n_on: int) -> np.ndarray:
    m = np.zeros(N, dtype=np.uint8)
    m[:n_on] = 1
    return m


def mask_random(cfg: LayerConfig, n_on: int) -> np.ndarray:
    rng = _rng(cfg.seed, S_MASK)
    m = np.zeros(cfg.N, dtype=np.uint8)
    m[rng.permutation(cfg.N)[:n_on]] = 1
    return m


def mask_top_by_counts(prev_counts: np.ndarray, n_on: int) -> np.ndarray:
    """The n_on experts with the largest previous-step workloads (ties to the lower index)."""
    c = np.asarray(prev_counts, dtype=np.int64)
    order = np.lexsort((np.arange(c.size), -c))
    m = np.zeros(c.size, dtype=np.uint8)
    m[order[:n_on]] = 1
    return m


# --------------------------------------------------------------------------
# residual drift between adjacent layers (input of the residual-based prediction)
# --------------------------------------------------------------------------

def layer_drift(cfg: LayerConfig, layer: int = 0, var: float = 0.1) -> np.ndarray:
    """[d] float32: the per-dimension drift r shared by all tokens, r ~ N(0, var)."""
    return normal_f32(cfg.seed, S_RES, (cfg.d,), var, sub=2 * layer)


def next_hidden_states(cfg: LayerConfig, h_bits: np.ndarray, layer: int = 0, var: float = 0.1,
                       noise_var: float = 0.01, draw: int = 0) -> np.ndarray:
    """[T, d] bf16 bits: h^(l+1) = h^(l) + r + eps with eps ~ N(0, noise_var) per token and dimension."""
    h = bf16_bits_to_f32(h_bits)
    r = layer_drift(cfg, layer, var)
    eps = normal_f32(cfg.seed, S_RES, h.shape, noise_var, sub=2 * layer + 1 + 1000 * draw)
    return to_bf16_bits(h + r[None, :] + eps)
