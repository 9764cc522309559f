"""GPU parity on the edges of the routing contract: more than 16384 routed rows (the permutation kernel then walks its
selections in several register loads), exactly equal logits (lower expert index wins, in selection and in slot order),
and k = N."""
import numpy as np
import pytest

import oracle
from paper_2602_03495_amd import workloads as wl
from helpers import GAP, check_routing, run_layer

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding, layer
    binding.load_library()
    return binding, layer


def _np(t):
    return t.cpu().numpy()


QWEN3_S = wl.scaled(wl.CONFIGS["qwen3"], d=256, I=128)
MIXTRAL_S = wl.scaled(wl.CONFIGS["mixtral"], d=512, I=1792)
DEEPSEEK_S = wl.scaled(wl.CONFIGS["deepseek"], d=256, I=384, I_shared=128)


def _route(B, Lm, cfg, h, W, b, mode=None, workspace=True):
    T = h.shape[0]
    s = B.shape(T, cfg.d, cfg.N, cfg.k, cfg.I)
    r = B.alloc_routing(s)
    B.moe_route(s, Lm.to_device_bf16(h), Lm.to_device_bf16(W), None if b is None else torch.from_numpy(b).cuda(),
                cfg.norm_mode if mode is None else mode, r, B.alloc_workspace(s) if workspace else None)
    torch.cuda.synchronize()
    return r


# ------------------------------------------------------------------------------------------- more than 16384 routed rows
@pytest.mark.parametrize("cfg,T", [(QWEN3_S, 2049), (QWEN3_S, 2500), (QWEN3_S, 4200), (wl.CONFIGS["mixtral"], 16384),
                                   (wl.CONFIGS["mixtral"], 8200), (DEEPSEEK_S, 6000)],
                         ids=["qwen3_s-2049", "qwen3_s-2500", "qwen3_s-4200", "mixtral-16384", "mixtral-8200", "deepseek_s-6000"])
def test_route_with_more_than_16384_routed_rows(gpu, cfg, T):
    # T*k = 16392, 20000, 33600, 32768, 16400, 36000: one row past a full load, and two to three loads
    B, Lm = gpu
    print(f"route {cfg.name} d={cfg.d} T={T} rows={T * cfg.k}", flush=True)
    assert T * cfg.k > 16384
    h, W, b = wl.hidden_states(cfg, T, draw=T), wl.gate_weights(cfg), wl.gate_bias(cfg)
    lg, o_idx, o_w, o_counts = oracle.route(h, W, b, cfg.k, cfg.norm_mode)
    r = _route(B, Lm, cfg, h, W, b)
    check_routing(lg, o_idx, o_w, o_counts, _np(r.topk_idx), _np(r.topk_w), _np(r.counts), _np(r.offsets), _np(r.perm),
                  _np(r.inv_perm), cfg.N, cfg.k)


def test_layer_with_more_than_16384_routed_rows(gpu):
    # the whole pass on top of such tables: tile schedule, both projections, combine (20000 rows; every row compared)
    B, Lm = gpu
    print("layer qwen3_s T=2500", flush=True)
    run_layer(B, Lm, QWEN3_S, 2500, [wl.mask_random(QWEN3_S, 96)], B.FFN_AUTO, draw=2500)


# ------------------------------------------------------------------------------------------- exact ties
@pytest.mark.parametrize("cfg,T", [(MIXTRAL_S, 1), (MIXTRAL_S, 16), (MIXTRAL_S, 300), (QWEN3_S, 16), (QWEN3_S, 200),
                                   (DEEPSEEK_S, 16), (DEEPSEEK_S, 1000)],
                         ids=["mixtral_s-1", "mixtral_s-16", "mixtral_s-300", "qwen3_s-16", "qwen3_s-200", "deepseek_s-16", "deepseek_s-1000"])
def test_all_logits_equal_selects_the_first_k_experts(gpu, cfg, T):
    # a zero gate matrix without bias: every logit is exactly 0 on both sides, so every token takes experts 0 .. k-1 in
    # that order, with weight 1/k (renormalised) or 1/N (Eq. 1 as printed)
    B, Lm = gpu
    print(f"all-equal logits {cfg.name} T={T}", flush=True)
    h = wl.hidden_states(cfg, T, draw=1)
    W = np.zeros((cfg.N, cfg.d), np.uint16)
    for mode, want in ((wl.NORM_RENORM, 1.0 / cfg.k), (wl.NORM_NONE, 1.0 / cfg.N)):
        for workspace in (True, False):
            r = _route(B, Lm, cfg, h, W, None, mode, workspace)
            _, o_idx, o_w, o_counts = oracle.route(h, W, None, cfg.k, mode)
            assert np.array_equal(o_idx, np.tile(np.arange(cfg.k, dtype=np.int32), (T, 1)))      # the oracle's own pin, restated
            assert np.array_equal(_np(r.topk_idx), o_idx)
            assert np.allclose(_np(r.topk_w), want, rtol=1e-6, atol=0) and np.allclose(o_w, want, rtol=1e-6, atol=0)
            assert np.array_equal(_np(r.counts), o_counts)
            assert np.array_equal(_np(r.perm), np.argsort(o_idx.ravel(), kind="stable"))
    # the same bias on every expert changes nothing
    r = _route(B, Lm, cfg, h, W, np.full(cfg.N, 0.75, np.float32))
    assert np.array_equal(_np(r.topk_idx), np.tile(np.arange(cfg.k, dtype=np.int32), (T, 1)))


@pytest.mark.parametrize("cfg,T", [(MIXTRAL_S, 16), (MIXTRAL_S, 300), (QWEN3_S, 16), (QWEN3_S, 700), (DEEPSEEK_S, 1),
                                   (DEEPSEEK_S, 130)],
                         ids=["mixtral_s-16", "mixtral_s-300", "qwen3_s-16", "qwen3_s-700", "deepseek_s-1", "deepseek_s-130"])
def test_duplicated_gate_rows_tie_to_the_lower_index(gpu, cfg, T):
    # three experts share one gate row and one (raised) bias: their logits are equal bit for bit on either side, they
    # are nearly always among the best, and whenever not all three fit, the lower indices must be taken; among the
    # selected ones the lower index comes first
    B, Lm = gpu
    print(f"duplicated gate rows {cfg.name} T={T}", flush=True)
    dup = [1, 4, 6] if cfg.N == 8 else [3, 17, cfg.N - 2]
    h, W, b = wl.hidden_states(cfg, T, draw=2), wl.gate_weights(cfg).copy(), wl.gate_bias(cfg).copy()
    W[dup[1]] = W[dup[0]]
    W[dup[2]] = W[dup[0]]
    b[dup] = b.max() + (0.5 if cfg.k > 2 else 1.5)
    lg, o_idx, o_w, o_counts = oracle.route(h, W, b, cfg.k, cfg.norm_mode)
    assert np.array_equal(lg[:, dup[0]], lg[:, dup[1]]) and np.array_equal(lg[:, dup[0]], lg[:, dup[2]])
    r = _route(B, Lm, cfg, h, W, b)
    g_idx, g_w = _np(r.topk_idx), _np(r.topk_w)
    # tokens on which nothing but the exact tie is close: all gaps between different values among the best k+1 logits
    # are at least GAP, so selection and order are decided by exact comparisons alone and must match bit for bit
    srt = -np.sort(-lg.astype(np.float64), axis=1)[:, : cfg.k + 1]
    gaps = srt[:, :-1] - srt[:, 1:]
    strict = np.all((gaps == 0) | (gaps >= GAP), axis=1)
    assert strict.sum() >= max(1, (3 * T) // 4)
    assert np.array_equal(g_idx[strict], o_idx[strict]), "equal logits must be taken by ascending expert index"
    assert np.allclose(g_w[strict], o_w[strict], rtol=2e-5, atol=1e-7)
    # the tie was really exercised: tokens with the duplicated experts selected in index order, and (k < 3 ways or
    # a full field) tokens where one of them had to stay out
    both = [(dup[0] in row) and (dup[1] in row) for row in o_idx[strict]]
    assert any(both)
    for row in g_idx[strict]:
        pos = [int(np.nonzero(row == e)[0][0]) for e in dup if e in row]
        assert pos == sorted(pos)
        if dup[1] in row:
            assert dup[0] in row
        if dup[2] in row:
            assert dup[1] in row
    if cfg.k == 2:
        assert any(dup[0] in row and dup[1] in row and dup[2] not in row for row in g_idx[strict])
    # internal consistency of the tables on all tokens
    assert np.array_equal(_np(r.counts), np.bincount(g_idx.ravel(), minlength=cfg.N))
    assert np.array_equal(_np(r.perm), np.argsort(g_idx.ravel(), kind="stable"))


@pytest.mark.parametrize("T", [1, 16, 300])
def test_every_expert_selected_when_k_equals_N(gpu, T):
    # k = N = 8: every token takes all experts, by descending score; the weights are the whole softmax and sum to 1 in
    # either mode; every workload is T
    B, Lm = gpu
    cfg = wl.scaled(wl.CONFIGS["tiny"], k=8)
    print(f"k = N = 8, T={T}", flush=True)
    h, W, b = wl.hidden_states(cfg, T, draw=4), wl.gate_weights(cfg), wl.gate_bias(cfg)
    for mode in (wl.NORM_NONE, wl.NORM_RENORM):
        lg, o_idx, o_w, o_counts = oracle.route(h, W, b, cfg.k, mode)
        r = _route(B, Lm, cfg, h, W, b, mode)
        check_routing(lg, o_idx, o_w, o_counts, _np(r.topk_idx), _np(r.topk_w), _np(r.counts), _np(r.offsets), _np(r.perm),
                      _np(r.inv_perm), cfg.N, cfg.k)
        assert np.all(_np(r.counts) == T)
        assert np.allclose(_np(r.topk_w).sum(1), 1.0, atol=1e-5)
    # and the whole layer on top of it (16 rows per token)
    if T > 1:
        run_layer(B, Lm, cfg, T, [wl.mask_lower(cfg.N, 5), None], B.FFN_AUTO, draw=4)
