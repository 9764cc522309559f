"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs, at sizes the oracle
finishes in seconds (several tiles plus a ragged tail)."""
import numpy as np
import pytest

import oracle
from paper_2602_03495_amd import workloads as wl
from helpers import OUT_TOL, check_routing, make_host_layer, rel_err, run_layer

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding, layer
    binding.load_library()
    return binding, layer


def _upload(layer_mod, hl):
    return layer_mod.LayerWeights.upload(hl.gate_w, hl.bias, hl.w1, hl.w3, hl.w2, hl.shared)


def _np(t):
    return t.cpu().numpy()


SMALL = {
    "tiny": wl.CONFIGS["tiny"],
    "mixtral_s": wl.scaled(wl.CONFIGS["mixtral"], d=512, I=1792),
    "deepseek_s": wl.scaled(wl.CONFIGS["deepseek"], d=256, I=384, I_shared=128),
    "qwen15_s": wl.scaled(wl.CONFIGS["qwen15"], d=384, I=128, I_shared=640),
    "qwen3_s": wl.scaled(wl.CONFIGS["qwen3"], d=256, I=128),
}


# ------------------------------------------------------------------------------------------- moe_route
@pytest.mark.parametrize("name,T", [("tiny", 64), ("tiny", 1), ("mixtral_s", 300), ("deepseek_s", 1000),
                                    ("qwen15_s", 17), ("qwen15_s", 1100), ("qwen3_s", 16), ("qwen3_s", 777)])
def test_route_matches_oracle(gpu, name, T):
    B, Lm = gpu
    cfg = SMALL[name]
    print(f"route {name} T={T}", flush=True)
    h = wl.hidden_states(cfg, T)
    W, b = wl.gate_weights(cfg), wl.gate_bias(cfg)
    lg, o_idx, o_w, o_counts = oracle.route(h, W, b, cfg.k, cfg.norm_mode)
    s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
    ws = B.alloc_workspace(s)
    r = B.alloc_routing(s)
    B.moe_route(s, Lm.to_device_bf16(h), Lm.to_device_bf16(W), torch.from_numpy(b).cuda(), cfg.norm_mode, r, ws)
    torch.cuda.synchronize()
    check_routing(lg, o_idx, o_w, o_counts, _np(r.topk_idx), _np(r.topk_w), _np(r.counts), _np(r.offsets),
                  _np(r.perm), _np(r.inv_perm), cfg.N, cfg.k)


def test_route_other_norm_mode_and_no_bias(gpu):
    B, Lm = gpu
    cfg = SMALL["deepseek_s"]
    T = 130
    h, W = wl.hidden_states(cfg, T, draw=3), wl.gate_weights(cfg)
    for mode in (wl.NORM_NONE, wl.NORM_RENORM):
        lg, o_idx, o_w, o_counts = oracle.route(h, W, None, cfg.k, mode)
        s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
        r = B.alloc_routing(s)
        B.moe_route(s, Lm.to_device_bf16(h), Lm.to_device_bf16(W), None, mode, r, B.alloc_workspace(s))
        torch.cuda.synchronize()
        check_routing(lg, o_idx, o_w, o_counts, _np(r.topk_idx), _np(r.topk_w), _np(r.counts), _np(r.offsets),
                      _np(r.perm), _np(r.inv_perm), cfg.N, cfg.k)
        if mode == wl.NORM_RENORM:
            assert np.allclose(_np(r.topk_w).sum(1), 1.0, atol=1e-5)


def test_route_extreme_bias_sends_every_token_to_one_expert(gpu):
    B, Lm = gpu
    cfg = SMALL["qwen3_s"]
    T = 200
    h, W, b = wl.hidden_states(cfg, T), wl.gate_weights(cfg), wl.gate_bias(cfg).copy()
    b[77] += 1e4
    s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
    r = B.alloc_routing(s)
    B.moe_route(s, Lm.to_device_bf16(h), Lm.to_device_bf16(W), torch.from_numpy(b).cuda(), cfg.norm_mode, r,
                B.alloc_workspace(s))
    torch.cuda.synchronize()
    assert int(_np(r.counts)[77]) == T and np.all(_np(r.topk_idx)[:, 0] == 77)
    assert np.all(np.isfinite(_np(r.topk_w)))


# ------------------------------------------------------------------------------------------- expert FFN + combine
_run_layer = run_layer


@pytest.mark.parametrize("path", ["tiled", "skinny"])
def test_tiny_layer_with_the_three_masks(gpu, path):
    B, Lm = gpu
    cfg = SMALL["tiny"]
    T = 64 if path == "tiled" else 16
    print(f"tiny layer {path}", flush=True)
    masks = [wl.mask_lower(cfg.N, 4), np.ones(cfg.N, np.uint8), np.zeros(cfg.N, np.uint8), None]
    _run_layer(B, Lm, cfg, T, masks, B.FFN_TILED if path == "tiled" else B.FFN_SKINNY)


@pytest.mark.parametrize("name,T", [("mixtral_s", 300), ("deepseek_s", 333), ("qwen15_s", 257), ("qwen3_s", 190)])
def test_scaled_layers_tiled_path(gpu, name, T):
    B, Lm = gpu
    cfg = SMALL[name]
    print(f"tiled {name} T={T}", flush=True)
    mask = wl.mask_random(cfg, (3 * cfg.N) // 4)
    _run_layer(B, Lm, cfg, T, [mask], B.FFN_TILED)


@pytest.mark.parametrize("name,T", [("mixtral_s", 17), ("mixtral_s", 32), ("deepseek_s", 33), ("qwen15_s", 64),
                                    ("qwen3_s", 48), ("mixtral_s", 65)])
def test_scaled_layers_mid_sized_batches(gpu, name, T):
    # batches between the decode kernels' limit and one full token tile: the tiled kernels run with 2, 4 or 8
    # token subtiles (an expert cannot receive more rows than there are tokens) and narrow down-projection tiles
    B, Lm = gpu
    cfg = SMALL[name]
    print(f"mid {name} T={T}", flush=True)
    _run_layer(B, Lm, cfg, T, [wl.mask_random(cfg, (3 * cfg.N) // 4), None], B.FFN_AUTO)


@pytest.mark.parametrize("name,T", [("mixtral_s", 1), ("mixtral_s", 16), ("deepseek_s", 16), ("qwen15_s", 1),
                                    ("qwen3_s", 16), ("qwen3_s", 5)])
def test_scaled_layers_skinny_path(gpu, name, T):
    B, Lm = gpu
    cfg = SMALL[name]
    print(f"skinny {name} T={T}", flush=True)
    mask = wl.mask_random(cfg, (3 * cfg.N) // 4)
    _run_layer(B, Lm, cfg, T, [mask, None], B.FFN_AUTO)


@pytest.mark.parametrize("T,n_on", [(40, 1), (40, 2), (100, 3), (128, 7), (200, 1), (200, 2), (200, 5), (300, 8)])
def test_few_working_experts_take_split_k_and_half_width_tiles(gpu, T, n_on):
    # with few experts masked on, the tiled kernels decide on the device to split the K range of the down projection
    # (fp32 partial sums + a finishing pass) and to run the up projection on half-width tiles; with all experts on they
    # do neither.  I = 8192 allows up to 8 splits (T = 40: single token tiles; T = 200, 300: scheduled tiles).
    B, Lm = gpu
    cfg = wl.scaled(wl.CONFIGS["mixtral"], d=512, I=8192)
    print(f"few working experts T={T} on={n_on}", flush=True)
    _, _, _, counts = oracle.route(wl.hidden_states(cfg, T), wl.gate_weights(cfg), wl.gate_bias(cfg), cfg.k, cfg.norm_mode)
    mask = np.zeros(cfg.N, np.uint8)
    mask[np.argsort(-counts, kind="stable")[:n_on]] = 1
    _run_layer(B, Lm, cfg, T, [mask], B.FFN_AUTO)


@pytest.mark.parametrize("T", [16, 40, 300])
def test_down_stage_alone_builds_its_own_tile_tables(gpu, T):
    # a down-stage call that no up-stage call preceded must not read tile tables from the workspace: with every workspace
    # byte set to 1 (table entries would be 16843009, activations 2.4e-38) it multiplies those activations and returns
    B, Lm = gpu
    cfg = SMALL["mixtral_s"]
    print(f"down stage alone T={T}", flush=True)
    hl = make_host_layer(cfg)
    dw = _upload(Lm, hl)
    L = Lm.MoeLayer(cfg, T)
    hd = Lm.to_device_bf16(wl.hidden_states(cfg, T))
    L.route(hd, dw)
    L.ws.fill_(1)
    L.y.fill_(1.0)
    r = L.routing
    B.moe_expert_ffn_stage(L.shape, hd, r.perm, r.offsets, r.counts, dw.w1, dw.w3, dw.w2, None, L.y, L.ws, B.STAGE_DOWN)
    torch.cuda.synchronize()
    y = wl.bf16_bits_to_f32(Lm.from_device_bf16(L.y))
    assert np.all(np.abs(y) < 1e-30)


def test_skinny_split_k_down_projection(gpu):
    # inner size above 4096 makes the down projection split K over blocks and finish in a second kernel
    B, Lm = gpu
    cfg = wl.scaled(wl.CONFIGS["mixtral"], d=256, I=4608)
    _run_layer(B, Lm, cfg, 16, [wl.mask_random(cfg, 6)], B.FFN_SKINNY)


def test_skinny_down_projection_without_split(gpu):
    # inner sizes in (2048, 4096] keep the decode-sized down projection on the skinny kernel, one block per row
    # tile over all of K; up to 2048 it runs on the tiled kernel (covered by the scaled shapes above)
    B, Lm = gpu
    cfg = wl.scaled(wl.CONFIGS["mixtral"], d=256, I=2304)
    _run_layer(B, Lm, cfg, 16, [wl.mask_random(cfg, 6), None], B.FFN_SKINNY)
    _run_layer(B, Lm, cfg, 3, [None], B.FFN_SKINNY)


def test_tiled_and_skinny_paths_agree_and_runs_are_deterministic(gpu):
    B, Lm = gpu
    cfg = SMALL["qwen3_s"]
    T = 16
    hl = make_host_layer(cfg)
    dw = _upload(Lm, hl)
    hd = Lm.to_device_bf16(wl.hidden_states(cfg, T))
    outs = []
    for path in (B.FFN_TILED, B.FFN_SKINNY, B.FFN_TILED, B.FFN_SKINNY):
        L = Lm.MoeLayer(cfg, T, path)
        outs.append(Lm.from_device_bf16(L.forward(hd, dw, None)).copy())
    torch.cuda.synchronize()
    assert np.array_equal(outs[0], outs[2]) and np.array_equal(outs[1], outs[3])
    a, b = wl.bf16_bits_to_f32(outs[0]), wl.bf16_bits_to_f32(outs[1])
    assert rel_err(a, b.astype(np.float64)) <= OUT_TOL


def test_mask_additivity_on_gpu(gpu):
    # outputs under a mask and under its complement add up to the all-on output (each expert on one side only)
    B, Lm = gpu
    cfg = SMALL["deepseek_s"]
    T = 200
    hl = make_host_layer(cfg)
    dw = _upload(Lm, hl)
    hd = Lm.to_device_bf16(wl.hidden_states(cfg, T))
    L = Lm.MoeLayer(cfg, T, B.FFN_TILED)
    m = wl.mask_random(cfg, cfg.N // 2)

    def run(mask):
        md = None if mask is None else torch.from_numpy(mask).cuda()
        o = L.forward(hd, dw, md, with_shared=False)
        return wl.bf16_bits_to_f32(Lm.from_device_bf16(o)).astype(np.float64)

    full, a, c = run(None), run(m), run(1 - m)
    assert rel_err(a + c, full) <= OUT_TOL
    assert np.all(run(np.zeros(cfg.N, np.uint8)) == 0)


# ------------------------------------------------------------------------------------------- prediction
@pytest.mark.parametrize("name,T,p", [("tiny", 64, 2), ("qwen15_s", 500, 4), ("qwen3_s", 16, 8), ("deepseek_s", 1, 4)])
def test_predict_workload(gpu, name, T, p):
    B, Lm = gpu
    cfg = SMALL[name]
    h = wl.hidden_states(cfg, T)
    W0, b0 = wl.gate_weights(cfg, 0), wl.gate_bias(cfg, 0)
    W1, b1 = wl.gate_weights(cfg, 1), wl.gate_bias(cfg, 1)
    s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
    ws = B.alloc_workspace(s)
    hd = Lm.to_device_bf16(h)
    pc = torch.empty(cfg.N, dtype=torch.int32, device="cuda")
    top = torch.empty(p, dtype=torch.int32, device="cuda")

    # zero residual and the layer's own gate: prediction == routing, bit for bit
    r = B.alloc_routing(s)
    B.moe_route(s, hd, Lm.to_device_bf16(W0), torch.from_numpy(b0).cuda(), cfg.norm_mode, r, ws)
    B.moe_predict_workload(s, hd, torch.zeros(cfg.d, device="cuda"), Lm.to_device_bf16(W0), torch.from_numpy(b0).cuda(),
                           p, pc, top, ws)
    torch.cuda.synchronize()
    assert np.array_equal(_np(pc), _np(r.counts))
    assert np.array_equal(_np(top), oracle.top_p(_np(r.counts), p))

    # next layer's gate on h + res_vec
    rv = wl.layer_drift(cfg)
    lg, o_idx, o_cnt, o_top = oracle.predict_workload(h, rv, W1, b1, cfg.k, p)
    B.moe_predict_workload(s, hd, torch.from_numpy(rv).cuda(), Lm.to_device_bf16(W1), torch.from_numpy(b1).cuda(), p, pc,
                           top, ws)
    torch.cuda.synchronize()
    from helpers import exempt_tokens
    nex = int(exempt_tokens(lg, cfg.k).sum())
    g_cnt = _np(pc)
    assert g_cnt.sum() == T * cfg.k
    assert int(np.abs(g_cnt.astype(np.int64) - o_cnt).sum()) <= 2 * nex
    assert np.array_equal(_np(top), oracle.top_p(g_cnt, p))
    if nex == 0:
        assert np.array_equal(_np(top), o_top)


@pytest.mark.parametrize("d,batches", [(256, [1000, 37]), (2048, [4097]), (384, [1, 0, 63, 64, 65]), (8, [5000])])
def test_res_vec_calibration_matches_oracle(gpu, d, batches):
    # device reduction of the res_vec equation over a calibration set that arrives in batches, against the
    # oracle on the concatenated set.  Both sum exactly representable bf16 differences in float64 (the orders
    # differ, the sums stay far below 2^53 ulps of the smallest term), so the fp32 results agree to the last bit
    # or, where the float64 sums differ in their last bits at a rounding boundary, to one fp32 ulp.
    B, Lm = gpu
    print(f"res_vec calibration d={d} batches={batches}", flush=True)
    cfg = wl.scaled(wl.CONFIGS["tiny"], d=max(d, 128))
    cal = B.ResVecCalibration(d)
    cur, nxt = [], []
    for i, n in enumerate(batches):
        if n == 0:
            h0 = np.zeros((0, d), np.uint16)
            h1 = np.zeros((0, d), np.uint16)
        else:
            h0 = np.ascontiguousarray(wl.hidden_states(cfg, n, draw=50 + i)[:, :d])
            h1 = np.ascontiguousarray(wl.next_hidden_states(cfg, wl.hidden_states(cfg, n, draw=50 + i), draw=i)[:, :d])
        cur.append(h0)
        nxt.append(h1)
        if n:
            cal.accumulate(Lm.to_device_bf16(h0), Lm.to_device_bf16(h1))
        else:
            cal.accumulate(torch.empty((0, d), dtype=torch.bfloat16, device="cuda"),
                           torch.empty((0, d), dtype=torch.bfloat16, device="cuda"))
    got = cal.finish().cpu().numpy()
    ref = oracle.res_vec(np.concatenate(cur), np.concatenate(nxt))
    assert cal.n_total == sum(batches)
    ulp = np.spacing(np.abs(ref).astype(np.float32))
    assert np.all(np.abs(got - ref) <= ulp), float(np.abs(got - ref).max())
    assert np.mean(got == ref) > 0.99
    assert np.abs(ref).max() > 0     # the drift of the generator is not zero: the comparison is not vacuous


@pytest.mark.parametrize("name,T", [("tiny", 16), ("mixtral_s", 16), ("qwen3_s", 16), ("qwen3_s", 7), ("deepseek_s", 1),
                                    ("qwen15_s", 40), ("qwen3_s", 300)])
def test_route_predict_equals_the_two_calls(gpu, name, T):
    # one call that routes this layer and predicts the next must give exactly what moe_route followed by
    # moe_predict_workload gives (both are checked against the oracle elsewhere), at decode sizes, where the two gates
    # share their launches, and beyond
    B, Lm = gpu
    cfg = SMALL[name]
    print(f"route_predict {name} T={T}", flush=True)
    p = min(8, cfg.N)
    h = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=3))
    W0, b0 = Lm.to_device_bf16(wl.gate_weights(cfg, 0)), torch.from_numpy(wl.gate_bias(cfg, 0)).cuda()
    W1, b1 = Lm.to_device_bf16(wl.gate_weights(cfg, 1)), torch.from_numpy(wl.gate_bias(cfg, 1)).cuda()
    rv = torch.from_numpy(wl.layer_drift(cfg)).cuda()
    s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
    ws = B.alloc_workspace(s)
    ra, rb = B.alloc_routing(s), B.alloc_routing(s)
    pca, pcb = (torch.full((cfg.N,), -1, dtype=torch.int32, device="cuda") for _ in range(2))
    topa, topb = (torch.full((p,), -1, dtype=torch.int32, device="cuda") for _ in range(2))
    B.moe_route(s, h, W0, b0, cfg.norm_mode, ra, ws)
    B.moe_predict_workload(s, h, rv, W1, b1, p, pca, topa, ws)
    torch.cuda.synchronize()
    ws.zero_()
    B.moe_route_predict(s, h, W0, b0, cfg.norm_mode, rb, rv, W1, b1, p, pcb, topb, ws)
    torch.cuda.synchronize()
    for f in ("topk_idx", "topk_w", "counts", "offsets", "perm", "inv_perm"):
        assert torch.equal(getattr(ra, f), getattr(rb, f)), f
    assert torch.equal(pca, pcb) and torch.equal(topa, topb)
    assert int(pcb.sum()) == T * cfg.k and int(rb.counts.sum()) == T * cfg.k


@pytest.mark.parametrize("T", [16, 40])
def test_largest_hidden_size_and_expert_count(gpu, T):
    # the limits of the interface at once: d = 8192, N = 128 experts, k = 8 (the decode kernels stop at d = 4096,
    # so the automatic path choice has to take the tiled kernels for the 16-token batch as well)
    B, Lm = gpu
    cfg = wl.scaled(wl.CONFIGS["qwen3"], d=8192, I=128)
    print(f"limits d=8192 N=128 k=8 T={T}", flush=True)
    _run_layer(B, Lm, cfg, T, [wl.mask_random(cfg, 96)], B.FFN_AUTO)


@pytest.mark.parametrize("name", ["mixtral_s", "qwen3_s"])
def test_graph_replays_equal_eager_runs(gpu, name):
    # the decode numbers are taken from HIP-graph replays: a captured pass (route + prediction, masked FFN, combine),
    # replayed several times with new inputs and with eager work and synchronisations in between, must reproduce the
    # eager results of the same inputs bit for bit
    B, Lm = gpu
    cfg = SMALL[name]
    T, p = 16, min(8, cfg.N)
    print(f"graph replay {name}", flush=True)
    hl = make_host_layer(cfg)
    dw = _upload(Lm, hl)
    W1, b1 = Lm.to_device_bf16(wl.gate_weights(cfg, 1)), torch.from_numpy(wl.gate_bias(cfg, 1)).cuda()
    nxt = Lm.LayerWeights(W1, b1, dw.w1, dw.w3, dw.w2)
    rv = torch.from_numpy(wl.layer_drift(cfg)).cuda()
    mask = torch.from_numpy(wl.mask_random(cfg, (3 * cfg.N) // 4)).cuda()
    L = Lm.MoeLayer(cfg, T)
    top = torch.empty(p, dtype=torch.int32, device="cuda")
    h_static = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=0)).clone()

    def one_pass():
        L.route_predict(h_static, dw, rv, nxt, p, top)
        L.expert_ffn(h_static, dw, mask)
        L.combine(mask, with_shared=False)

    def snapshot():
        torch.cuda.synchronize()
        r = L.routing
        return [x.clone() for x in (r.topk_idx, r.topk_w, r.counts, r.offsets, r.perm, r.inv_perm, L.pred_counts, top, L.out)]

    inputs = [Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=d_)) for d_ in (1, 2, 3, 1)]
    eager = []
    for x in inputs:
        h_static.copy_(x)
        one_pass()
        eager.append(snapshot())
    assert not torch.equal(eager[0][8], eager[1][8])          # the inputs differ, so do the results

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        one_pass()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        one_pass()
    for i, x in enumerate(inputs):
        h_static.copy_(x)
        L.out.zero_()                                         # eager work between the replays
        L.routing.counts.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(got, eager[i]):
            assert torch.equal(a, b), (i, a.dtype, a.shape)


@pytest.mark.parametrize("name,T", [("qwen3_s", 16), ("qwen3_s", 300), ("deepseek_s", 9), ("deepseek_s", 130), ("mixtral_s", 16)])
def test_route_without_a_workspace_gives_the_same_tables(gpu, name, T):
    # moe_route may be called with workspace = NULL: gates with many experts then evaluate all experts of 16 tokens in
    # one block instead of storing logits first; every output must be identical
    B, Lm = gpu
    cfg = SMALL[name]
    print(f"route no-workspace {name} T={T}", flush=True)
    h = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=5))
    W, b = Lm.to_device_bf16(wl.gate_weights(cfg)), torch.from_numpy(wl.gate_bias(cfg)).cuda()
    s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
    ra, rb = B.alloc_routing(s), B.alloc_routing(s)
    B.moe_route(s, h, W, b, cfg.norm_mode, ra, B.alloc_workspace(s))
    B.moe_route(s, h, W, b, cfg.norm_mode, rb, None)
    torch.cuda.synchronize()
    for f in ("topk_idx", "counts", "offsets", "perm", "inv_perm"):
        assert torch.equal(getattr(ra, f), getattr(rb, f)), f
    assert torch.allclose(ra.topk_w, rb.topk_w, rtol=1e-6, atol=0)
    assert int(rb.counts.sum()) == T * cfg.k


# ------------------------------------------------------------------------------------------- shared experts inside the grouped launches
MERGED = {
    "deepseek_m": wl.scaled(wl.CONFIGS["deepseek"], d=256, I=128, I_shared=128),    # 2 shared experts, weight 1
    "qwen15_m": wl.scaled(wl.CONFIGS["qwen15"], d=384, I=128, I_shared=512),        # 1 sigmoid-gated shared expert = 4 x I
}


@pytest.mark.parametrize("name,T", [("deepseek_m", 1), ("deepseek_m", 16), ("deepseek_m", 333), ("qwen15_m", 1),
                                    ("qwen15_m", 40), ("qwen15_m", 700)])
def test_shared_experts_appended_to_the_routing_tables(gpu, name, T):
    B, Lm = gpu
    cfg = MERGED[name]
    print(f"merged shared {name} T={T}", flush=True)
    hl = make_host_layer(cfg)
    h = wl.hidden_states(cfg, T, draw=T)
    lg, o_idx, o_w, o_counts = oracle.route(h, hl.gate_w, hl.bias, cfg.k, cfg.norm_mode)
    dw = Lm.LayerWeights.upload(hl.gate_w, hl.bias, hl.w1, hl.w3, hl.w2, hl.shared, merge_shared=True)
    L = Lm.MoeLayer(cfg, T)
    Sm = L.n_merged
    assert Sm == cfg.n_shared * (cfg.I_shared // cfg.I) and dw.xw1.shape[0] == cfg.N + Sm
    kx, R = cfg.k + Sm, T * cfg.k
    hd = Lm.to_device_bf16(h)
    mask = (np.arange(cfg.N) % 4 != 1).astype(np.uint8)
    for m in (None, mask):
        xm = L.merged_mask(None if m is None else torch.from_numpy(m).cuda())
        out = L.forward_merged(hd, dw, xm)
        torch.cuda.synchronize()
        r, x = L.routing, L.xrouting
        ex = check_routing(lg, o_idx, o_w, o_counts, _np(r.topk_idx), _np(r.topk_w), _np(r.counts), _np(r.offsets),
                           _np(r.perm), _np(r.inv_perm), cfg.N, cfg.k)
        x_idx, x_w, x_counts, x_off = _np(x.topk_idx), _np(x.topk_w), _np(x.counts), _np(x.offsets)
        x_perm, x_inv = _np(x.perm), _np(x.inv_perm)
        # the routed slots are the oracle's (checked above on the routed tables: here they must be those tables, unchanged)
        assert np.array_equal(x_idx[:, :cfg.k], _np(r.topk_idx)) and np.array_equal(x_w[:, :cfg.k], _np(r.topk_w))
        # the shared slots: expert N + j, weight 1 or the oracle's sigmoid gate
        assert np.array_equal(x_idx[:, cfg.k:], np.tile(cfg.N + np.arange(Sm, dtype=np.int32), (T, 1)))
        c = oracle.shared_scale(h, hl.shared[3]) if hl.shared_mode == 2 else np.ones(T)
        assert np.allclose(x_w[:, cfg.k:], np.repeat(c[:, None], Sm, 1), rtol=2e-5, atol=1e-7)
        # histogram, scan and the stable grouping of the wider tables
        assert np.array_equal(x_counts, np.bincount(x_idx.ravel(), minlength=cfg.N + Sm))
        assert np.all(x_counts[cfg.N:] == T) and int(x_counts.sum()) == T * kx
        assert np.array_equal(x_off, np.concatenate(([0], np.cumsum(x_counts))))
        assert np.array_equal(x_perm, np.argsort(x_idx.ravel(), kind="stable"))
        assert np.array_equal(x_inv[x_perm], np.arange(T * kx))
        # layer output against the oracle's layer with shared experts
        keep = np.nonzero(~ex)[0].astype(np.int32)
        ref = oracle.layer(h, o_idx, o_w, hl.w1, hl.w3, hl.w2, m, hl.shared, hl.shared_mode, tokens=keep)
        got = wl.bf16_bits_to_f32(Lm.from_device_bf16(out))[keep]
        assert rel_err(got, ref) <= OUT_TOL, rel_err(got, ref)
        # and against the separate-launch path of the same library (the shared term is rounded to bf16 once per block there)
        sep = L.forward(hd, dw, None if m is None else torch.from_numpy(m).cuda()).float().cpu().numpy()[keep]
        assert rel_err(sep, ref) <= OUT_TOL


@pytest.mark.parametrize("name,T", [("mixtral_s", 300), ("deepseek_s", 700)])
def test_prefill_graph_replays_equal_eager_runs(gpu, name, T):
    # bench.py takes its prefill figure from HIP-graph replays too: a captured pass over a prefill-sized batch (tile
    # schedule kernel, both tiled projections, shared experts, combine), replayed with new inputs and eager work in
    # between, must reproduce the eager results bit for bit
    B, Lm = gpu
    cfg = SMALL[name]
    print(f"prefill graph replay {name} T={T}", flush=True)
    hl = make_host_layer(cfg)
    dw = _upload(Lm, hl)
    mask = torch.from_numpy(wl.mask_random(cfg, (3 * cfg.N) // 4)).cuda()
    L = Lm.MoeLayer(cfg, T)
    h_static = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=0)).clone()

    def snapshot():
        torch.cuda.synchronize()
        r = L.routing
        return [x.clone() for x in (r.topk_idx, r.topk_w, r.counts, r.offsets, r.perm, r.inv_perm, L.out)]

    inputs = [Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=d_)) for d_ in (1, 2, 1)]
    eager = []
    for x in inputs:
        h_static.copy_(x)
        L.forward(h_static, dw, mask)
        eager.append(snapshot())
    assert not torch.equal(eager[0][6], eager[1][6])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        L.forward(h_static, dw, mask)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        L.forward(h_static, dw, mask)
    for i, x in enumerate(inputs):
        h_static.copy_(x)
        L.out.zero_()
        L.y.zero_()
        L.routing.counts.fill_(-7)
        torch.cuda.synchronize()
        g.replay()
        for a, b in zip(snapshot(), eager[i]):
            assert torch.equal(a, b), (i, a.dtype, a.shape)


@pytest.mark.parametrize("name,T", [("deepseek_m", 1), ("deepseek_m", 16), ("deepseek_m", 9), ("qwen15_m", 1), ("qwen15_m", 16),
                                    ("deepseek_m", 333), ("qwen15_m", 40)])
def test_route_shared_equals_the_two_calls(gpu, name, T):
    # one call that routes and appends the shared experts' slots must give exactly what moe_route followed by
    # moe_append_shared gives (both checked against the oracle elsewhere): at decode sizes, where the selecting block
    # writes both sets of tables (8 experts: in the gate kernel itself; more: in the selection kernel), and beyond
    B, Lm = gpu
    cfg = MERGED[name]
    if name == "deepseek_m" and T == 9:
        cfg = wl.scaled(cfg, N=8, k=2)                    # at most 16 experts: gate, selection and tables in one kernel
    print(f"route_shared {cfg.name} N={cfg.N} T={T}", flush=True)
    S = cfg.n_shared * (cfg.I_shared // cfg.I)
    h = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=7))
    W, b = Lm.to_device_bf16(wl.gate_weights(cfg)), torch.from_numpy(wl.gate_bias(cfg)).cuda()
    w_sg = Lm.to_device_bf16(wl.shared_expert_weights(cfg)[3]) if cfg.shared_gate == "sigmoid" else None
    s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
    sx = B.shape(T, cfg.d, cfg.N + S, cfg.k + S, cfg.I)
    for use_ws in (True, False):
        ws = B.alloc_workspace(s) if use_ws else None
        ra, rb, xa, xb = B.alloc_routing(s), B.alloc_routing(s), B.alloc_routing(sx), B.alloc_routing(sx)
        for r in (ra, rb, xa, xb):
            for f in ("topk_idx", "counts", "offsets", "perm", "inv_perm"):
                getattr(r, f).fill_(-5)
            r.topk_w.fill_(-5.0)
        B.moe_route(s, h, W, b, cfg.norm_mode, ra, ws)
        B.moe_append_shared(s, S, h, w_sg, ra, xa)
        B.moe_route_shared(s, S, h, W, b, cfg.norm_mode, w_sg, rb, xb, ws)
        torch.cuda.synchronize()
        for f in ("topk_idx", "topk_w", "counts", "offsets", "perm", "inv_perm"):
            assert torch.equal(getattr(ra, f), getattr(rb, f)), ("routed", f)
            assert torch.equal(getattr(xa, f), getattr(xb, f)), ("wider", f)
        assert int(xb.counts.sum()) == T * (cfg.k + S) and int(xb.counts[cfg.N:].min()) == T
