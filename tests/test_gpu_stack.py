"""Decode stack (several layers, several steps, AR(1) gate bias): workload histograms and predictions."""
import numpy as np
import pytest

import oracle
from paper_2602_03495_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def stack():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding
    from paper_2602_03495_amd.stack import DecodeStack
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
