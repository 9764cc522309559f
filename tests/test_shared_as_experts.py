"""Shared experts written as further routed experts (oracle only, no GPU).

Eq. 2 sums expert outputs, and a SwiGLU expert is itself a sum over its inner units, so a layer with N routed experts,
k per token, and shared experts whose inner size is a multiple m of the routed one equals a layer of N + S*m experts in
which every token carries S*m extra slots of weight c(t).  The HIP path relies on that identity to run shared experts
inside its grouped launches; here the oracle's own two evaluations must agree."""
import numpy as np
import pytest

import oracle
from paper_2602_03495_amd import workloads as wl


def _split_shared(cfg, w1, w3, w2, shared):
    sw1, sw3, sw2, _ = shared
    S, Is, d = sw1.shape
    m = Is // cfg.I
    c1, c3 = sw1.reshape(S * m, cfg.I, d), sw3.reshape(S * m, cfg.I, d)
    c2 = np.ascontiguousarray(sw2.reshape(S, d, m, cfg.I).transpose(0, 2, 1, 3)).reshape(S * m, d, cfg.I)
    return np.concatenate((w1, c1)), np.concatenate((w3, c3)), np.concatenate((w2, c2)), S * m


@pytest.mark.parametrize("name,kw,mode", [("deepseek", dict(d=128, I=64, I_shared=64), 1),
                                          ("qwen15", dict(d=128, I=64, I_shared=256), 2)])
def test_layer_with_shared_experts_equals_the_wider_layer(name, kw, mode):
    cfg = wl.scaled(wl.CONFIGS[name], **kw)
    T = 9
    h = wl.hidden_states(cfg, T)
    w1, w3, w2 = wl.expert_weights(cfg)
    shared = wl.shared_expert_weights(cfg)
    _, idx, w, _ = oracle.route(h, wl.gate_weights(cfg), wl.gate_bias(cfg), cfg.k, cfg.norm_mode)
    mask = (np.arange(cfg.N) % 3 != 0).astype(np.uint8)
    ref = oracle.layer(h, idx, w, w1, w3, w2, mask, shared, mode)
    xw1, xw3, xw2, Sm = _split_shared(cfg, w1, w3, w2, shared)
    c = oracle.shared_scale(h, shared[3]) if mode == 2 else np.ones(T)
    x_idx = np.concatenate((idx, np.tile(cfg.N + np.arange(Sm, dtype=np.int32), (T, 1))), 1)
    x_w = np.concatenate((w, np.repeat(c[:, None], Sm, 1).astype(np.float32)), 1)
    x_mask = np.concatenate((mask, np.ones(Sm, np.uint8)))
    wide = oracle.layer(h, x_idx, x_w, xw1, xw3, xw2, x_mask)
    # c(t) passes through float32 in the wider layer's weight table
    assert np.abs(wide - ref).max() <= 1e-6 * np.abs(ref).max()
    # and the shared term is not negligible in this comparison
    routed_only = oracle.layer(h, idx, w, w1, w3, w2, mask)
    assert np.abs(routed_only - ref).max() > 0.1 * np.abs(ref).max()


def test_shared_scale_closed_forms_and_the_layer_oracle():
    cfg = wl.scaled(wl.CONFIGS["qwen15"], d=128, I=64, I_shared=128)
    T = 7
    h = wl.hidden_states(cfg, T)
    shared = wl.shared_expert_weights(cfg)
    w_sg = shared[3]
    c = oracle.shared_scale(h, w_sg)
    assert c.shape == (T,) and np.all((c > 0) & (c < 1))
    zero = np.zeros_like(w_sg)
    assert np.array_equal(oracle.shared_scale(h, zero), np.full(T, 0.5))
    neg = w_sg ^ np.uint16(0x8000)                         # -w_sg, exactly
    assert np.allclose(oracle.shared_scale(h, neg), 1.0 - c, rtol=0, atol=1e-15)
    one_hot = np.zeros_like(w_sg)
    one_hot[5] = wl.to_bf16_bits(np.array([1.0], np.float32))[0]
    x5 = wl.bf16_bits_to_f32(h[:, 5]).astype(np.float64)
    assert np.allclose(oracle.shared_scale(h, one_hot), 1.0 / (1.0 + np.exp(-x5)), rtol=1e-15)
    # the C oracle's layer applies the same factor: with the routed weights zeroed, (sigmoid-gated output) = c * (ungated output)
    w1, w3, w2 = wl.expert_weights(cfg)
    idx = np.zeros((T, cfg.k), np.int32) + np.arange(cfg.k, dtype=np.int32)
    w0 = np.zeros((T, cfg.k), np.float32)
    gated = oracle.layer(h, idx, w0, w1, w3, w2, None, shared, 2)
    plain = oracle.layer(h, idx, w0, w1, w3, w2, None, shared, 1)
    assert np.allclose(gated, c[:, None] * plain, rtol=1e-12, atol=1e-300)
