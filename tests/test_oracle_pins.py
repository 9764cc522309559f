"""Pins of the CPU oracle against things other than itself: brute force, hand values, closed forms,
library routines in float64 and the invariants the paper's definitions imply (Eq. 1, Eq. 2, the workload
definition, the mutual-exclusion constraint on C and G, the residual-prefetching equations)."""
import itertools
import os

import numpy as np
import pytest
from scipy.special import expit, softmax

import oracle
from paper_2602_03495_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf(x):
    return wl.to_bf16_bits(np.asarray(x, dtype=np.float32))


def f64(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def rnd(seed, shape, var=1.0):
    return wl.normal_bf16(seed, 0, shape, var)


# ----------------------------------------------------------------------------- bf16 packing

def test_bf16_roundtrip_and_rounding():
    # exactly representable values survive; ties go to even; the decoder is exact
    vals = np.array([0.0, 1.0, -2.5, 0.15625, 3.0e38], dtype=np.float32)
    assert np.array_equal(wl.bf16_bits_to_f32(wl.to_bf16_bits(vals))[:4], vals[:4])
    one_plus = np.array([1.0 + 2.0 ** -8], dtype=np.float32)          # halfway between 1 and 1+2^-7 -> even (1.0)
    assert wl.bf16_bits_to_f32(wl.to_bf16_bits(one_plus))[0] == 1.0
    three_half = np.array([1.0 + 3 * 2.0 ** -8], dtype=np.float32)    # halfway, odd below -> rounds up to 1+2^-6
    assert wl.bf16_bits_to_f32(wl.to_bf16_bits(three_half))[0] == 1.0 + 2.0 ** -6


# ----------------------------------------------------------------------------- logits (gate product)

def test_logits_match_float64_matmul_with_bias_and_non_square_shapes():
    T, d, N = 7, 48, 5                       # N != d: a transposed gate matrix cannot pass
    h, W = rnd(1, (T, d)), rnd(2, (N, d), 1.0 / d)
    b = np.linspace(-1, 1, N).astype(np.float32)
    ref = (f64(h) @ f64(W).T).astype(np.float32) + b
    got = oracle.logits(h, W, b)
    assert np.array_equal(got, ref)
    assert np.array_equal(oracle.logits(h, W), (f64(h) @ f64(W).T).astype(np.float32))


def test_logits_one_hot_gate_closed_form():
    T, d, N = 5, 16, 4
    h = rnd(3, (T, d))
    W = np.zeros((N, d), dtype=np.float32)
    for e in range(N):
        W[e, 3 * e + 1] = 0.5
    got = oracle.logits(h, bf(W))
    want = 0.5 * wl.bf16_bits_to_f32(h)[:, [1, 4, 7, 10]]
    assert np.array_equal(got, want)


def test_logits_with_residual_vector_uses_float32_sum():
    T, d, N = 6, 40, 7
    h, W = rnd(4, (T, d)), rnd(5, (N, d), 1.0 / d)
    r = wl.normal_f32(6, 0, (d,), 0.1)
    ht = (wl.bf16_bits_to_f32(h) + r[None, :]).astype(np.float32)     # formed in float32
    ref = (ht.astype(np.float64) @ f64(W).T).astype(np.float32)
    assert np.array_equal(oracle.logits(h, W, None, r), ref)
    # zero residual vector == plain gate
    assert np.array_equal(oracle.logits(h, W, None, np.zeros(d, np.float32)), oracle.logits(h, W))


# ----------------------------------------------------------------------------- selection and weights (Eq. 1)

@pytest.mark.parametrize("N,k", [(4, 1), (6, 2), (8, 3), (8, 2)])
def test_selection_equals_brute_force_over_all_subsets(N, k):
    rng = np.random.default_rng(10 * N + k)
    lg = rng.standard_normal((32, N)).astype(np.float32)
    idx, w = oracle.select(lg, k, wl.NORM_NONE)
    p = softmax(lg.astype(np.float64), axis=1)
    for t in range(lg.shape[0]):
        best = max(itertools.combinations(range(N), k), key=lambda s: sum(p[t, e] for e in s))
        assert set(idx[t]) == set(best)
        assert list(idx[t]) == sorted(idx[t], key=lambda e: -lg[t, e])   # descending score
        assert np.allclose(w[t], p[t, idx[t]], rtol=1e-6, atol=0)


def test_selection_matches_float64_argsort_and_softmax():
    rng = np.random.default_rng(7)
    lg = rng.standard_normal((200, 60)).astype(np.float32) * 3
    k = 4
    idx, w = oracle.select(lg, k, wl.NORM_NONE)
    order = np.argsort(-lg.astype(np.float64), axis=1, kind="stable")[:, :k]
    assert np.array_equal(idx, order)
    p = softmax(lg.astype(np.float64), axis=1)
    assert np.allclose(w, np.take_along_axis(p, order, 1), rtol=1e-6, atol=0)
    idx2, w2 = oracle.select(lg, k, wl.NORM_RENORM)
    assert np.array_equal(idx2, idx)
    sel = np.take_along_axis(p, order, 1)
    assert np.allclose(w2, sel / sel.sum(1, keepdims=True), rtol=1e-6, atol=0)
    # renormalised weights == softmax over the k selected logits
    assert np.allclose(w2, softmax(np.take_along_axis(lg.astype(np.float64), order, 1), axis=1), rtol=1e-6)
    assert np.allclose(w2.sum(1), 1.0, atol=1e-6)
    assert np.all(w.sum(1) <= 1.0 + 1e-6) and np.all(w > 0)


def test_selection_special_cases():
    N = 8
    lg = np.random.default_rng(3).standard_normal((9, N)).astype(np.float32)
    # k = N: every expert, weights are the full softmax
    idx, w = oracle.select(lg, N, wl.NORM_NONE)
    assert all(sorted(r) == list(range(N)) for r in idx)
    assert np.allclose(np.sort(w, 1), np.sort(softmax(lg.astype(np.float64), 1), 1), rtol=1e-6)
    # k = 1 renormalised: weight exactly 1, expert = argmax
    idx, w = oracle.select(lg, 1, wl.NORM_RENORM)
    assert np.array_equal(idx[:, 0], np.argmax(lg, 1)) and np.all(w == 1.0)
    # all logits equal: lowest indices win, uniform weights
    eq = np.full((3, N), 0.25, dtype=np.float32)
    idx, w = oracle.select(eq, 3, wl.NORM_NONE)
    assert np.array_equal(idx, np.tile(np.arange(3), (3, 1))) and np.allclose(w, 1.0 / N)
    idx, w = oracle.select(eq, 3, wl.NORM_RENORM)
    assert np.allclose(w, 1.0 / 3)
    # a partial tie: equal scores ordered by ascending index
    tie = np.array([[0.0, 2.0, 1.0, 2.0, -1.0]], dtype=np.float32)
    idx, _ = oracle.select(tie, 3, wl.NORM_NONE)
    assert list(idx[0]) == [1, 3, 2]
    # softmax is shift invariant and must not overflow
    big = lg + np.float32(80000.0)
    i1, w1 = oracle.select(big[:, :4].copy(), 2, wl.NORM_NONE)
    assert np.all(np.isfinite(w1))


# ----------------------------------------------------------------------------- workload histogram

def test_histogram_invariants_and_bincount():
    cfg = wl.CONFIGS["tiny"]
    T = 64
    h, W, b = wl.hidden_states(cfg, T), wl.gate_weights(cfg), wl.gate_bias(cfg)
    lg, idx, w, counts = oracle.route(h, W, b, cfg.k, cfg.norm_mode)
    assert counts.sum() == T * cfg.k
    assert counts.min() >= 0 and counts.max() <= T
    assert np.array_equal(counts, np.bincount(idx.ravel(), minlength=cfg.N))
    assert all(len(set(r)) == cfg.k for r in idx)          # an expert appears at most once per token
    # a huge bias on one expert routes every token to it
    b2 = b.copy()
    b2[5] += 1e4
    _, idx2, _, c2 = oracle.route(h, W, b2, cfg.k, cfg.norm_mode)
    assert c2[5] == T and np.all(idx2[:, 0] == 5)


def test_top_p_ordering():
    counts = np.array([3, 9, 9, 0, 7, 9, 1], dtype=np.int32)
    assert list(oracle.top_p(counts, 4)) == [1, 2, 5, 4]
    rng = np.random.default_rng(0)
    c = rng.integers(0, 50, 128).astype(np.int32)
    want = np.lexsort((np.arange(128), -c.astype(np.int64)))[:8]
    assert np.array_equal(oracle.top_p(c, 8), want)


# ----------------------------------------------------------------------------- expert FFN

def _golden_cases():
    cases = []
    with open(os.path.join(GOLDEN, "ffn_hand_values.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.split() for p in line.split("|")]
            d, I = int(parts[0][0]), int(parts[0][1])
            x, W1, W3, W2, y = (np.array(p, dtype=np.float64) for p in parts[1:])
            cases.append((d, I, x, W1.reshape(I, d), W3.reshape(I, d), W2.reshape(d, I), y))
    return cases


def test_expert_ffn_hand_values():
    cases = _golden_cases()
    assert len(cases) == 3
    for d, I, x, W1, W3, W2, y in cases:
        idx = np.zeros((1, 1), dtype=np.int32)
        got = oracle.expert_rows(bf(x[None, :]), idx, bf(W1[None]), bf(W3[None]), bf(W2[None]))
        assert np.allclose(got[0, 0], y, rtol=0, atol=1e-15), (got, y)


def _ffn_ref(x, W1, W3, W2):
    g, u = W1 @ x, W3 @ x
    return W2 @ (g * expit(g) * u)


def test_expert_ffn_matches_float64_matmuls_and_closed_forms():
    d, I, N, T = 24, 40, 3, 5
    h = rnd(11, (T, d))
    w1, w3, w2 = rnd(12, (N, I, d), 1 / d), rnd(13, (N, I, d), 1 / d), rnd(14, (N, d, I), 1 / I)
    idx = np.array([[0, 1], [2, 0], [1, 2], [2, 1], [0, 2]], dtype=np.int32)
    y = oracle.expert_rows(h, idx, w1, w3, w2)
    for t in range(T):
        for s in range(2):
            e = idx[t, s]
            ref = _ffn_ref(f64(h[t]), f64(w1[e]), f64(w3[e]), f64(w2[e]))
            assert np.allclose(y[t, s], ref, rtol=1e-12, atol=1e-14)
    zero = np.zeros_like(w2)
    assert np.all(oracle.expert_rows(h, idx, w1, w3, zero) == 0)                    # W2 = 0
    assert np.all(oracle.expert_rows(h, idx, w1, np.zeros_like(w3), w2) == 0)       # W3 = 0
    assert np.all(oracle.expert_rows(np.zeros_like(h), idx, w1, w3, w2) == 0)       # x = 0
    w2x4 = bf(4.0 * wl.bf16_bits_to_f32(w2))                                        # exact scaling in bf16
    assert np.allclose(oracle.expert_rows(h, idx, w1, w3, w2x4), 4.0 * y, rtol=1e-15)
    # swapping W1 and W3 changes the result (silu sits on W1 only)
    assert not np.allclose(oracle.expert_rows(h, idx, w3, w1, w2), y)
    # masked-off experts give zero rows, the others are unchanged
    m = np.array([1, 0, 1], dtype=np.uint8)
    ym = oracle.expert_rows(h, idx, w1, w3, w2, mask=m)
    on = m[idx].astype(bool)
    assert np.all(ym[~on] == 0) and np.array_equal(ym[on], y[on])


# ----------------------------------------------------------------------------- combine (Eq. 2) and masks

def _tiny_layer(T=16, seed_shift=0):
    cfg = wl.scaled(wl.CONFIGS["tiny"], d=32, I=48, N=8, k=2)
    h = wl.hidden_states(cfg, T, draw=seed_shift)
    W, b = wl.gate_weights(cfg), wl.gate_bias(cfg)
    w1, w3, w2 = wl.expert_weights(cfg)
    _, idx, w, counts = oracle.route(h, W, b, cfg.k, cfg.norm_mode)
    return cfg, h, W, b, w1, w3, w2, idx, w, counts


def test_layer_is_weighted_sum_of_expert_rows():
    cfg, h, W, b, w1, w3, w2, idx, w, _ = _tiny_layer()
    y = oracle.expert_rows(h, idx, w1, w3, w2)
    out = oracle.layer(h, idx, w, w1, w3, w2)
    ref = (w.astype(np.float64)[:, :, None] * y).sum(1)
    assert np.allclose(out, ref, rtol=1e-13, atol=1e-15)
    # token subset selects the same rows
    sel = [3, 0, 11]
    assert np.array_equal(oracle.layer(h, idx, w, w1, w3, w2, tokens=sel), out[sel])


def test_identical_experts_with_renormalised_weights_give_the_single_expert():
    cfg, h, W, b, w1, w3, w2, idx, w, _ = _tiny_layer()
    w1s, w3s, w2s = (np.repeat(a[:1], cfg.N, 0) for a in (w1, w3, w2))
    out = oracle.layer(h, idx, w, w1s, w3s, w2s)
    for t in range(h.shape[0]):
        ref = _ffn_ref(f64(h[t]), f64(w1[0]), f64(w3[0]), f64(w2[0]))
        assert np.allclose(out[t], ref, rtol=1e-6, atol=1e-8)     # weights sum to 1 within float32


def test_mask_all_on_all_off_and_additivity():
    cfg, h, W, b, w1, w3, w2, idx, w, _ = _tiny_layer()
    full = oracle.layer(h, idx, w, w1, w3, w2)
    ones, zeros = np.ones(cfg.N, np.uint8), np.zeros(cfg.N, np.uint8)
    assert np.array_equal(oracle.layer(h, idx, w, w1, w3, w2, mask=ones), full)
    assert np.all(oracle.layer(h, idx, w, w1, w3, w2, mask=zeros) == 0)
    m = wl.mask_lower(cfg.N, 4)
    a = oracle.layer(h, idx, w, w1, w3, w2, mask=m)
    c = oracle.layer(h, idx, w, w1, w3, w2, mask=1 - m)
    assert np.allclose(a + c, full, rtol=1e-13, atol=1e-15)       # each expert runs on exactly one side
    assert not np.allclose(a, full)


def test_token_permutation_and_expert_relabelling():
    cfg, h, W, b, w1, w3, w2, idx, w, _ = _tiny_layer()
    full = oracle.layer(h, idx, w, w1, w3, w2)
    perm = np.random.default_rng(5).permutation(h.shape[0])
    _, idx_p, w_p, _ = oracle.route(h[perm], W, b, cfg.k, cfg.norm_mode)
    assert np.array_equal(oracle.layer(h[perm], idx_p, w_p, w1, w3, w2), full[perm])
    # relabel experts: gate rows, bias, expert weights and mask move together
    sigma = np.random.default_rng(6).permutation(cfg.N)          # new label j holds old expert sigma[j]
    m = wl.mask_lower(cfg.N, 4)
    _, idx_r, w_r, counts_r = oracle.route(h, W[sigma], b[sigma], cfg.k, cfg.norm_mode)
    out_r = oracle.layer(h, idx_r, w_r, w1[sigma], w3[sigma], w2[sigma], mask=m[sigma])
    assert np.allclose(out_r, oracle.layer(h, idx, w, w1, w3, w2, mask=m), rtol=1e-12, atol=1e-14)
    assert np.array_equal(sigma[idx_r], idx)
    assert np.array_equal(counts_r, np.bincount(idx.ravel(), minlength=cfg.N)[sigma])


def test_shared_experts():
    cfg, h, W, b, w1, w3, w2, idx, w, _ = _tiny_layer()
    d, Is = cfg.d, 24
    sw1, sw3, sw2 = rnd(21, (2, Is, d), 1 / d), rnd(22, (2, Is, d), 1 / d), rnd(23, (2, d, Is), 1 / Is)
    routed = oracle.layer(h, idx, w, w1, w3, w2)
    sh = np.stack([_ffn_ref(f64(h[t]), f64(sw1[0]), f64(sw3[0]), f64(sw2[0]))
                   + _ffn_ref(f64(h[t]), f64(sw1[1]), f64(sw3[1]), f64(sw2[1])) for t in range(h.shape[0])])
    out1 = oracle.layer(h, idx, w, w1, w3, w2, shared=(sw1, sw3, sw2, None), shared_mode=1)
    assert np.allclose(out1, routed + sh, rtol=1e-12, atol=1e-14)
    # sigmoid-gated shared expert; a zero gate vector gives exactly one half
    wsg = rnd(24, (d,), 1 / d)
    c = expit(f64(h) @ f64(wsg))
    sh0 = np.stack([_ffn_ref(f64(h[t]), f64(sw1[0]), f64(sw3[0]), f64(sw2[0])) for t in range(h.shape[0])])
    out2 = oracle.layer(h, idx, w, w1, w3, w2, shared=(sw1[:1], sw3[:1], sw2[:1], wsg), shared_mode=2)
    assert np.allclose(out2, routed + c[:, None] * sh0, rtol=1e-12, atol=1e-14)
    out3 = oracle.layer(h, idx, w, w1, w3, w2, shared=(sw1[:1], sw3[:1], sw2[:1], np.zeros_like(wsg)), shared_mode=2)
    assert np.allclose(out3, routed + 0.5 * sh0, rtol=1e-12, atol=1e-14)
    # shared experts ignore the routed mask
    z = np.zeros(cfg.N, np.uint8)
    out4 = oracle.layer(h, idx, w, w1, w3, w2, mask=z, shared=(sw1, sw3, sw2, None), shared_mode=1)
    assert np.allclose(out4, sh, rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------------------- residual-based prediction

def test_prediction_special_cases():
    cfg = wl.CONFIGS["tiny"]
    T = 64
    h, W, b = wl.hidden_states(cfg, T), wl.gate_weights(cfg), wl.gate_bias(cfg)
    _, idx, _, counts = oracle.route(h, W, b, cfg.k, cfg.norm_mode)
    # zero residual and the same gate: the prediction is the routing itself
    _, pidx, pc, top = oracle.predict_workload(h, np.zeros(cfg.d, np.float32), W, b, cfg.k, 3)
    assert np.array_equal(pidx, idx) and np.array_equal(pc, counts)
    assert np.array_equal(top, np.lexsort((np.arange(cfg.N), -counts.astype(np.int64)))[:3])
    # a residual that is a large multiple of one gate row sends every token to that expert
    r = (30.0 * wl.bf16_bits_to_f32(W[6])).astype(np.float32)   # shifts logit 6 by about 30 |W_6|^2 ~ 30
    _, _, pc2, top2 = oracle.predict_workload(h, r, W, b, cfg.k, 1)
    assert pc2[6] == T and pc2.sum() == T * cfg.k and np.sum(pc2 == T) == 1 and top2[0] == 6


def test_res_vec_is_the_mean_feature_difference():
    cfg = wl.scaled(wl.CONFIGS["qwen15"], d=64)
    n = 2048
    h0 = wl.hidden_states(cfg, n)
    h1 = wl.next_hidden_states(cfg, h0)
    rv = oracle.res_vec(h0, h1)
    ref = (f64(h1) - f64(h0)).mean(0)
    assert np.allclose(rv, ref.astype(np.float32), rtol=1e-6, atol=1e-7)
    drift = wl.layer_drift(cfg)
    # the calibrated vector recovers the generator's drift up to noise/sqrt(n) and bf16 rounding
    assert np.abs(rv - drift).max() < 0.02
    # a constant shift that bf16 represents exactly is recovered exactly
    h2 = bf(wl.bf16_bits_to_f32(bf(np.round(wl.bf16_bits_to_f32(h0) * 4) / 4)) + 0.5)
    h0q = bf(np.round(wl.bf16_bits_to_f32(h0) * 4) / 4)
    assert np.allclose(oracle.res_vec(h0q, h2), 0.5)
