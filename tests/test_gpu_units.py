"""Entry points of the C ABI one at a time, against what their header comment defines (written out here with numpy
index arithmetic, or the oracle where the operation is part of the layer)."""
import numpy as np
import pytest

import oracle
from helpers import OUT_TOL, make_host_layer, rel_err
from paper_2602_03495_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding, layer
    binding.load_library()
    return binding, layer


@pytest.mark.parametrize("n,rows,K", [(1, 16, 32), (3, 48, 160), (2, 1408, 2048)])
def test_pack_weights_is_the_documented_permutation(gpu, n, rows, K):
    # packed[m][rb][kb][l][j] = src[m][16 rb + l % 16][32 kb + 8 (l / 16) + j]: a pure permutation of bit patterns
    B, Lm = gpu
    print(f"pack {n}x{rows}x{K}", flush=True)
    rng = np.random.Generator(np.random.Philox(key=[7, n * rows + K]))
    src = rng.integers(0, 65536, size=(n, rows, K), dtype=np.uint16)
    got = Lm.from_device_bf16(B.moe_pack_weights(Lm.to_device_bf16(src)))
    m, rb, kb, l, j = np.meshgrid(np.arange(n), np.arange(rows // 16), np.arange(K // 32), np.arange(64), np.arange(8),
                                  indexing="ij")
    want = src[m, 16 * rb + l % 16, 32 * kb + 8 * (l // 16) + j]
    assert np.array_equal(got.reshape(want.shape), want)


def test_dense_route_tables(gpu):
    # every token goes to every one of the S always-on experts: counts = T, rows of expert e are tokens 0..T-1 in order
    B, Lm = gpu
    T, S = 37, 3
    s = B.shape(T, 256, S, S, 128)
    i32 = dict(dtype=torch.int32, device="cuda")
    counts, offsets, perm = torch.empty(S, **i32), torch.empty(S + 1, **i32), torch.empty(T * S, **i32)
    B.moe_dense_route(s, counts, offsets, perm)
    torch.cuda.synchronize()
    assert counts.tolist() == [T] * S and offsets.tolist() == [0, T, 2 * T, 3 * T]
    p = perm.cpu().numpy().reshape(S, T)
    for e in range(S):
        assert np.array_equal(p[e], np.arange(T) * S + e)


def test_shared_gate_is_the_sigmoid_of_the_dot_product(gpu):
    B, Lm = gpu
    cfg = wl.scaled(wl.CONFIGS["qwen15"], d=384, I=128, I_shared=128)
    T = 50
    h = wl.hidden_states(cfg, T)
    w_sg = wl.shared_expert_weights(cfg)[3]
    scale = torch.empty(T, dtype=torch.float32, device="cuda")
    B.moe_shared_gate(B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I), Lm.to_device_bf16(h), Lm.to_device_bf16(w_sg), scale)
    z = wl.bf16_bits_to_f32(h).astype(np.float64) @ wl.bf16_bits_to_f32(w_sg).astype(np.float64)
    assert np.allclose(scale.cpu().numpy(), 1.0 / (1.0 + np.exp(-z)), rtol=2e-5, atol=1e-7)


@pytest.mark.parametrize("T,path", [(16, "skinny"), (100, "tiled")])
def test_staged_ffn_equals_the_single_call(gpu, T, path):
    # up projection, then down projection, through moe_expert_ffn_stage = moe_expert_ffn, bit for bit
    B, Lm = gpu
    cfg = wl.scaled(wl.CONFIGS["mixtral"], d=512, I=1792)
    w1, w3, w2 = wl.expert_weights(cfg)
    dw = Lm.LayerWeights.upload(wl.gate_weights(cfg), wl.gate_bias(cfg), w1, w3, w2)
    L = Lm.MoeLayer(cfg, T, B.FFN_SKINNY if path == "skinny" else B.FFN_TILED)
    h = Lm.to_device_bf16(wl.hidden_states(cfg, T))
    mask = torch.from_numpy(wl.mask_random(cfg, 6)).cuda()
    L.route(h, dw)
    r = L.routing
    L.y.zero_()
    L.expert_ffn(h, dw, mask)
    whole = L.y.clone()
    L.y.zero_()
    L.ws.zero_()
    for stage in (B.STAGE_UP, B.STAGE_DOWN):
        B.moe_expert_ffn_stage(L.shape, h, r.perm, r.offsets, r.counts, dw.w1, dw.w3, dw.w2, mask, L.y, L.ws, stage)
    torch.cuda.synchronize()
    assert torch.equal(whole, L.y)
    assert float(whole.float().abs().max()) > 0


def test_combine_alone_matches_the_weighted_sum(gpu):
    # Eq. 2 on given expert rows: out[t] = sum over masked-on slots of w[t,s] * y[inv_perm[t,s]] (+ scale[t] * shared rows)
    B, Lm = gpu
    T, d, N, k, S = 33, 256, 8, 2, 2
    rng = np.random.Generator(np.random.Philox(key=[11, 5]))
    y = wl.to_bf16_bits(rng.standard_normal((T * k, d)).astype(np.float32))
    sy = wl.to_bf16_bits(rng.standard_normal((S * T, d)).astype(np.float32))
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    w = rng.random((T, k), dtype=np.float32)
    inv = rng.permutation(T * k).astype(np.int32)
    mask = (rng.random(N) < 0.6).astype(np.uint8)
    scale = rng.random(T, dtype=np.float32)
    out = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    s = B.shape(T, d, N, k, 128)
    dev = lambda a: torch.from_numpy(a).cuda()
    B.moe_combine(s, Lm.to_device_bf16(y), dev(idx), dev(w), dev(inv), dev(mask), Lm.to_device_bf16(sy), S, dev(scale), out)
    yf, syf = wl.bf16_bits_to_f32(y).astype(np.float64), wl.bf16_bits_to_f32(sy).astype(np.float64)
    ref = np.zeros((T, d))
    for t in range(T):
        for sl in range(k):
            if mask[idx[t, sl]]:
                ref[t] += float(w[t, sl]) * yf[inv[t * k + sl]]
        for e in range(S):
            ref[t] += float(scale[t]) * syf[e * T + t]
    got = wl.bf16_bits_to_f32(Lm.from_device_bf16(out))
    assert rel_err(got, ref) <= OUT_TOL
    # without shared rows and with everything masked off the output is exactly zero
    B.moe_combine(s, Lm.to_device_bf16(y), dev(idx), dev(w), dev(inv), dev(np.zeros(N, np.uint8)), None, 0, None, out)
    assert float(out.float().abs().max()) == 0.0


def test_block_timeline_records_every_block_of_both_tiled_launches(gpu):
    # diagnostics: with a record buffer set, each block of the tiled up / down launches that had a tile to work on
    # writes one record; the results of the layer are the same with and without it
    B, Lm = gpu
    cfg = wl.scaled(wl.CONFIGS["mixtral"], d=512, I=1792)
    T = 300
    hl = make_host_layer(cfg)
    dw = Lm.LayerWeights.upload(hl.gate_w, hl.bias, hl.w1, hl.w3, hl.w2)
    L = Lm.MoeLayer(cfg, T, B.FFN_TILED)
    hd = Lm.to_device_bf16(wl.hidden_states(cfg, T))
    L.route(hd, dw)
    L.expert_ffn(hd, dw, None)
    want = L.y.clone()
    records = torch.zeros(2 * B.TRACE_MAX_BLOCKS * 8, dtype=torch.int64, device="cuda")
    B.moe_debug_set_trace(records)
    L.expert_ffn(hd, dw, None)
    torch.cuda.synchronize()
    B.moe_debug_set_trace(None)
    assert torch.equal(L.y.view(torch.int16), want.view(torch.int16))
    tr = records.cpu().numpy().reshape(2, B.TRACE_MAX_BLOCKS, 8)
    counts = L.routing.counts.cpu().numpy()
    for mode in (0, 1):
        t = tr[mode][tr[mode][:, 7] == 1]
        assert len(t) > 0
        assert np.all(t[:, 1] >= t[:, 0]) and np.all((t[:, 5] >= 1) & (t[:, 5] <= 128))
        assert set(t[:, 4].tolist()) == set(np.nonzero(counts)[0].tolist())
        # per column tile, the token tiles of an expert cover its rows exactly once (the tile height is the kernel's choice)
        for col_tile in set(t[:, 6].tolist()):
            part = t[t[:, 6] == col_tile]
            for e in np.nonzero(counts)[0]:
                assert int(part[part[:, 4] == e][:, 5].sum()) == int(counts[e]), (mode, col_tile, e)
    # switched off: nothing is written any more
    records.zero_()
    L.expert_ffn(hd, dw, None)
    torch.cuda.synchronize()
    assert not bool(records.any())
