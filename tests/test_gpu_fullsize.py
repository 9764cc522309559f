"""GPU parity at the full sizes of the five configurations, in the launch configuration bench.py times
(automatic FFN path, same buffers and call order).

Routing, histogram, permutation and prediction are checked on ALL tokens (the oracle's gate is cheap).
Expert rows and layer outputs are checked on a seeded token sample plus every token of the least-loaded
masked-on expert, which the oracle computes one by one; properties that hold at any size (histogram sums,
mask additivity, determinism) cover the rest.
"""
import numpy as np
import pytest

import oracle
from paper_2602_03495_amd import workloads as wl
from helpers import OUT_TOL, check_routing, exempt_tokens, make_host_layer, rel_err, sample_tokens

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding, layer
    binding.load_library()
    return binding, layer


_cache = {}


def host_and_device(Lm, name):
    """Weights of one full-size config, generated once per test module."""
    if name not in _cache:
        _cache.clear()                    # keep one config resident at a time
        torch.cuda.empty_cache()
        hl = make_host_layer(wl.CONFIGS[name])
        dw = Lm.LayerWeights.upload(hl.gate_w, hl.bias, hl.w1, hl.w3, hl.w2, hl.shared, merge_shared=True)
        _cache[name] = (hl, dw)
    return _cache[name]


def _np(t):
    return t.cpu().numpy()


def config_mask(cfg, hl):
    """The expert mask each configuration prescribes."""
    if cfg.name == "mixtral":
        return wl.mask_random(cfg, 6)
    if cfg.name == "deepseek":                      # top-32 experts by the previous step's workloads
        prev = wl.hidden_states(cfg, 2048, draw=99)
        _, _, _, c = oracle.route(prev, hl.gate_w, hl.bias, cfg.k, cfg.norm_mode)
        return wl.mask_top_by_counts(c, 32)
    if cfg.name == "qwen3":                         # top-64 of 128 by the previous step's workloads
        prev = wl.hidden_states(cfg, 16, draw=99)
        _, _, _, c = oracle.route(prev, hl.gate_w, hl.bias, cfg.k, cfg.norm_mode)
        return wl.mask_top_by_counts(c, 64)
    return np.ones(cfg.N, np.uint8)                 # qwen15: all experts on


CASES = [("mixtral", 2048), ("mixtral", 1), ("mixtral", 16), ("mixtral", 64), ("mixtral", 256),   # 64, 256: mid-sized batches
         ("mixtral", 8192), ("mixtral", 16384),                                                                    # 16384 and 32768 routed rows: the tile tables of the larger survey batches
         ("deepseek", 2048), ("deepseek", 16), ("qwen15", 4096), ("qwen15", 1), ("qwen3", 16), ("qwen3", 128), ("qwen3", 2048)]


@pytest.mark.parametrize("name,T", CASES)
def test_full_size_layer(gpu, name, T):
    B, Lm = gpu
    cfg = wl.CONFIGS[name]
    print(f"full size {name} T={T}", flush=True)
    hl, dw = host_and_device(Lm, name)
    mask = config_mask(cfg, hl)
    h = wl.hidden_states(cfg, T, draw=T)
    lg, o_idx, o_w, o_counts = oracle.route(h, hl.gate_w, hl.bias, cfg.k, cfg.norm_mode)

    L = Lm.MoeLayer(cfg, T)
    hd, md = Lm.to_device_bf16(h), torch.from_numpy(mask).cuda()
    out = L.forward(hd, dw, md)
    torch.cuda.synchronize()
    r = L.routing
    g_idx, g_counts = _np(r.topk_idx), _np(r.counts)
    ex = check_routing(lg, o_idx, o_w, o_counts, g_idx, _np(r.topk_w), g_counts, _np(r.offsets), _np(r.perm),
                       _np(r.inv_perm), cfg.N, cfg.k)
    print(f"  exempt tokens: {int(ex.sum())} of {T}; counts min/max {g_counts.min()}/{g_counts.max()}", flush=True)

    # sample: random tokens + every token of the least-loaded masked-on expert with any rows
    on = mask.astype(bool)
    cand = [e for e in range(cfg.N) if on[e] and o_counts[e] > 0]
    extra = []
    if cand:
        e_min = min(cand, key=lambda e: (o_counts[e], e))
        extra = np.nonzero((o_idx == e_min).any(1))[0][:64]
    toks = sample_tokens(T, 24, seed=cfg.seed + T, extra=extra)
    toks = toks[~ex[toks]]
    y_ref = oracle.expert_rows(h, o_idx, hl.w1, hl.w3, hl.w2, mask, tokens=toks)
    inv = _np(r.inv_perm).reshape(T, cfg.k)
    rows = np.array([[inv[t, int(np.nonzero(g_idx[t] == o_idx[t, s])[0][0])] for s in range(cfg.k)] for t in toks])
    y_gpu = wl.bf16_bits_to_f32(Lm.from_device_bf16(L.y[torch.from_numpy(rows.ravel()).cuda().long()]))
    y_gpu = y_gpu.reshape(len(toks), cfg.k, cfg.d)
    worst = 0.0
    for n, t in enumerate(toks):
        for s in range(cfg.k):
            if on[o_idx[t, s]]:
                worst = max(worst, rel_err(y_gpu[n, s], y_ref[n, s]))
    assert worst <= OUT_TOL, worst
    ref = oracle.layer(h, o_idx, o_w, hl.w1, hl.w3, hl.w2, mask, hl.shared, hl.shared_mode, tokens=toks)
    got = wl.bf16_bits_to_f32(Lm.from_device_bf16(out))[toks]
    err = rel_err(got, ref)
    print(f"  sampled {len(toks)} tokens: expert rows {worst:.2e}, layer output {err:.2e}", flush=True)
    assert err <= OUT_TOL, err

    # any-size properties: a second run is bit-identical; the all-off mask gives exactly zero
    first = Lm.from_device_bf16(out).copy()
    out2 = L.forward(hd, dw, md)
    torch.cuda.synchronize()
    assert np.array_equal(first, Lm.from_device_bf16(out2))
    zero = L.forward(hd, dw, torch.zeros(cfg.N, dtype=torch.uint8, device="cuda"), with_shared=False)
    torch.cuda.synchronize()
    assert not bool(zero.view(torch.int16).bitwise_and(0x7FFF).any())


@pytest.mark.parametrize("name,T", [("deepseek", 16), ("deepseek", 2048), ("qwen15", 1), ("qwen15", 4096)])
def test_full_size_layer_with_shared_experts_inside_the_grouped_launches(gpu, name, T):
    B, Lm = gpu
    cfg = wl.CONFIGS[name]
    print(f"full size, shared experts appended: {name} T={T}", flush=True)
    hl, dw = host_and_device(Lm, name)
    mask = config_mask(cfg, hl)
    h = wl.hidden_states(cfg, T, draw=T)
    lg, o_idx, o_w, o_counts = oracle.route(h, hl.gate_w, hl.bias, cfg.k, cfg.norm_mode)
    L = Lm.MoeLayer(cfg, T)
    assert L.n_merged == cfg.n_shared * (cfg.I_shared // cfg.I)
    hd = Lm.to_device_bf16(h)
    out = L.forward_merged(hd, dw, L.merged_mask(torch.from_numpy(mask).cuda()))
    torch.cuda.synchronize()
    r, x = L.routing, L.xrouting
    ex = check_routing(lg, o_idx, o_w, o_counts, _np(r.topk_idx), _np(r.topk_w), _np(r.counts), _np(r.offsets), _np(r.perm),
                       _np(r.inv_perm), cfg.N, cfg.k)
    x_idx, x_counts = _np(x.topk_idx), _np(x.counts)
    assert np.array_equal(x_counts, np.bincount(x_idx.ravel(), minlength=cfg.N + L.n_merged))
    assert np.array_equal(_np(x.perm), np.argsort(x_idx.ravel(), kind="stable"))
    toks = sample_tokens(T, 24, seed=cfg.seed + T)
    toks = toks[~ex[toks]]
    ref = oracle.layer(h, o_idx, o_w, hl.w1, hl.w3, hl.w2, mask, hl.shared, hl.shared_mode, tokens=toks)
    got = wl.bf16_bits_to_f32(Lm.from_device_bf16(out))[toks]
    err = rel_err(got, ref)
    print(f"  sampled {len(toks)} tokens: layer output {err:.2e}", flush=True)
    assert err <= OUT_TOL, err


def test_full_size_mask_additivity_mixtral(gpu):
    B, Lm = gpu
    cfg = wl.CONFIGS["mixtral"]
    hl, dw = host_and_device(Lm, "mixtral")
    T = 2048
    hd = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=T))
    L = Lm.MoeLayer(cfg, T)
    m = wl.mask_random(cfg, 6)

    def run(mask):
        o = L.forward(hd, dw, torch.from_numpy(np.ascontiguousarray(mask)).cuda())
        return o.float().double().cpu().numpy()

    full, a, c = run(np.ones(cfg.N, np.uint8)), run(m), run((1 - m).astype(np.uint8))
    assert rel_err(a + c, full) <= OUT_TOL


def test_full_size_prediction_qwen15(gpu):
    """Residual-based prediction at the Qwen1.5-MoE shape: next layer's gate on h + res_vec, res_vec calibrated
    on 4096 separate tokens of the synthetic stack h' = h + r + eps."""
    B, Lm = gpu
    cfg = wl.CONFIGS["qwen15"]
    T, p = 4096, 4
    h = wl.hidden_states(cfg, T, draw=T)
    cal = wl.hidden_states(cfg, 4096, draw=7)
    rv = oracle.res_vec(cal, wl.next_hidden_states(cfg, cal, draw=7))
    W1, b1 = wl.gate_weights(cfg, 1), wl.gate_bias(cfg, 1)
    lg, o_idx, o_cnt, o_top = oracle.predict_workload(h, rv, W1, b1, cfg.k, p)
    s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
    ws = B.alloc_workspace(s)
    pc = torch.empty(cfg.N, dtype=torch.int32, device="cuda")
    top = torch.empty(p, dtype=torch.int32, device="cuda")
    B.moe_predict_workload(s, Lm.to_device_bf16(h), torch.from_numpy(rv).cuda(), Lm.to_device_bf16(W1),
                           torch.from_numpy(b1).cuda(), p, pc, top, ws)
    torch.cuda.synchronize()
    nex = int(exempt_tokens(lg, cfg.k).sum())
    g = _np(pc)
    assert g.sum() == T * cfg.k and int(np.abs(g.astype(np.int64) - o_cnt).sum()) <= 2 * nex
    assert np.array_equal(_np(top), oracle.top_p(g, p))
    # the prediction is useful: against the true next-layer routing of h' = h + r + eps it beats res_vec = 0
    h_next = wl.next_hidden_states(cfg, h, draw=1)
    _, _, _, true_cnt = oracle.route(h_next, W1, b1, cfg.k, cfg.norm_mode)
    B.moe_predict_workload(s, Lm.to_device_bf16(h), torch.zeros(cfg.d, device="cuda"), Lm.to_device_bf16(W1),
                           torch.from_numpy(b1).cuda(), p, pc, top, ws)
    torch.cuda.synchronize()
    l1_res = np.abs(g.astype(np.int64) - true_cnt).sum()
    l1_raw = np.abs(_np(pc).astype(np.int64) - true_cnt).sum()
    print(f"  histogram L1 error vs true next-layer workloads: with res_vec {l1_res}, without {l1_raw}", flush=True)
    assert l1_res <= l1_raw
