"""Decode stack (several layers, several steps, AR(1) gate bias): workload histograms and predictions."""
import numpy as np
import pytest

import oracle
from paper_2602_03495_amd import workloads as wl
from helpers import OUT_TOL, check_routing, exempt_tokens, make_host_layer, rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def stack():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding
    from bench_stack import DecodeStack
    binding.load_library()
    cfg = wl.scaled(wl.CONFIGS["qwen3"], d=256, I=128)
    return cfg, DecodeStack(cfg, 3, 16)


def test_stack_histograms_and_first_layer_parity(stack):
    cfg, st = stack
    steps = 6
    bias = st.bias_paths(steps)
    res = st.run(steps, bias, use_res_vec=False)
    c = res.counts
    assert c.shape == (steps, 3, cfg.N)
    assert np.all(c.sum(-1) == 16 * cfg.k) and c.min() >= 0 and c.max() <= 16
    # layer 0 sees seeded inputs only, so its histograms must equal the oracle's step by step
    b0 = wl.ar1_bias_path(cfg, 0, steps)
    for t in range(steps):
        h = wl.hidden_states(cfg, 16, draw=t)
        lg, _, _, oc = oracle.route(h, wl.gate_weights(cfg, 0), b0[t], cfg.k, cfg.norm_mode)
        srt = -np.sort(-lg.astype(np.float64), 1)
        if np.all(srt[:, cfg.k - 1] - srt[:, cfg.k] >= 1e-4):
            assert np.array_equal(c[t, 0], oc)
        # the prediction made at layer 0 is the next layer's gate on h (no residual vector here)
        _, _, pc, _ = oracle.predict_workload(h, np.zeros(cfg.d, np.float32), wl.gate_weights(cfg, 1),
                                              wl.ar1_bias_path(cfg, 1, steps)[t], cfg.k, 8)
        assert np.abs(res.pred_counts[t, 0].astype(np.int64) - pc).sum() <= 4
    # a second run gives the same histograms
    res2 = st.run(steps, bias, use_res_vec=False)
    assert np.array_equal(res2.counts, c) and np.array_equal(res2.pred_counts, res.pred_counts)
    assert res.tokens_per_s > 0 and set(res.acc) == {1, 4, 8}


def test_every_layer_of_the_stack_matches_the_oracle_on_the_input_it_saw(stack):
    # Layers after the first see inputs that the GPU produced, so each (step, layer) pass is checked on its own: the
    # oracle gets the very hidden states, gate bias and mask that the pass was run with (copied to the host) and must
    # reproduce its routing tables, its workload prediction for the next layer and its output.
    cfg, st = stack
    steps = 4
    bias = st.bias_paths(steps)
    st.calibrate(bias, steps=2)
    res = st.run(steps, bias, use_res_vec=True, predict="fused", keep_io=True)
    assert len(res.io) == steps * 3
    hosts = [make_host_layer(cfg, l) for l in range(3)]
    seen_layers, worst = set(), 0.0
    for rec in res.io:
        l, h, hl = rec["layer"], rec["h"], hosts[rec["layer"]]
        lg, o_idx, o_w, o_counts = oracle.route(h, hl.gate_w, rec["bias"], cfg.k, cfg.norm_mode)
        ex = check_routing(lg, o_idx, o_w, o_counts, rec["topk_idx"], rec["topk_w"], rec["counts"], rec["offsets"], rec["perm"],
                           rec["inv_perm"], cfg.N, cfg.k)
        assert np.array_equal(rec["counts"], res.counts[rec["step"], l])
        keep = np.nonzero(~ex)[0].astype(np.int32)
        ref = oracle.layer(h, o_idx, o_w, hl.w1, hl.w3, hl.w2, rec["mask"], None, 0, tokens=keep)
        got = wl.bf16_bits_to_f32(rec["out"])[keep]
        err = rel_err(got, ref) if np.abs(ref).max() > 0 else float(np.abs(got).max())
        worst = max(worst, err)
        assert err <= OUT_TOL, (rec["step"], l, err)
        if rec["pred_counts"] is not None:
            plg, _, pc, _ = oracle.predict_workload(h, rec["res_vec"], hosts[l + 1].gate_w, rec["next_bias"], cfg.k, 8)
            nex = int(exempt_tokens(plg, cfg.k).sum())
            assert rec["pred_counts"].sum() == 16 * cfg.k
            assert int(np.abs(rec["pred_counts"].astype(np.int64) - pc).sum()) <= 2 * nex
        seen_layers.add(l)
    print(f"  {len(res.io)} layer passes, worst output error {worst:.2e}", flush=True)
    assert seen_layers == {0, 1, 2}
    # the harness's glue between layers is what it says: the next layer's input is rmsnorm(h + out) rounded to bf16
    a, b = res.io[0], res.io[1]
    x = wl.bf16_bits_to_f32(a["h"]).astype(np.float64) + wl.bf16_bits_to_f32(a["out"]).astype(np.float64)
    x = x / np.sqrt((x * x).mean(-1, keepdims=True) + 1e-6)
    assert np.abs(wl.bf16_bits_to_f32(b["h"]) - x).max() <= 2.0 ** -7 * np.abs(x).max()


def test_stack_calibrated_residual_does_not_hurt(stack):
    cfg, st = stack
    steps = 8
    bias = st.bias_paths(steps)
    st.calibrate(bias, steps=4)
    assert all(float(r.abs().max()) < 10 for r in st.res_vec)
    with_rv = st.run(steps, bias, use_res_vec=True)
    without = st.run(steps, bias, use_res_vec=False)
    l1 = lambda r: np.abs(r.pred_counts[:, :2].astype(np.int64) - r.counts[:, 1:]).sum()
    assert l1(with_rv) <= 1.1 * l1(without) + 8


def test_prediction_on_a_side_stream_gives_the_same_results(stack):
    # the prediction issued on a second stream, concurrent with routing / FFN / combine and with a workspace of its
    # own, must change neither the layer results nor the predictions
    cfg, st = stack
    steps = 5
    bias = st.bias_paths(steps)
    inline = st.run(steps, bias, use_res_vec=True, predict="inline")
    side = st.run(steps, bias, use_res_vec=True, predict="side")
    off = st.run(steps, bias, use_res_vec=True, predict="off")
    assert np.array_equal(inline.counts, side.counts) and np.array_equal(inline.counts, off.counts)
    assert np.array_equal(inline.pred_counts, side.pred_counts)
    assert not off.acc and set(side.acc) == {1, 4, 8}
