"""The entry point that allocates nothing (moe_expert_ffn_static) against moe_expert_ffn: same tables, same weights,
bit-identical rows, on two calls in a row, the second with a smaller input (all calls share one scratch array)."""
import ctypes as C

import numpy as np
import pytest

from paper_2602_03495_amd import workloads as wl
from helpers import SENTINEL, make_host_layer

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding, layer
    binding.load_library()
    return binding, layer


MIXTRAL_S = wl.scaled(wl.CONFIGS["mixtral"], d=512, I=4608)      # I > 4096: the decode down projection splits K (partial sums in scratch)
QWEN3_S = wl.scaled(wl.CONFIGS["qwen3"], d=256, I=128)


@pytest.mark.parametrize("cfg,sizes", [(MIXTRAL_S, (16, 3)), (MIXTRAL_S, (300, 40)), (QWEN3_S, (700, 16)), (MIXTRAL_S, (200, 1))],
                         ids=["decode-16-then-3", "prefill-300-then-40", "qwen3_s-700-then-16", "prefill-200-then-1"])
def test_static_scratch_entry_point_matches_the_workspace_one(gpu, cfg, sizes):
    B, Lm = gpu
    hl = make_host_layer(cfg)
    dw = Lm.LayerWeights.upload(hl.gate_w, hl.bias, hl.w1, hl.w3, hl.w2)
    mask = torch.from_numpy(wl.mask_random(cfg, (3 * cfg.N) // 4)).cuda()
    assert B.static_scratch_bytes() == 32 << 20
    for T in sizes:
        print(f"no-alloc {cfg.name} I={cfg.I} T={T}", flush=True)
        L = Lm.MoeLayer(cfg, T)
        assert B.workspace_bytes(L.shape) <= B.static_scratch_bytes()
        hd = Lm.to_device_bf16(wl.hidden_states(cfg, T, draw=T))
        L.route(hd, dw)
        r = L.routing
        for m in (mask, None):
            L.y.view(torch.int16).fill_(SENTINEL)
            B.moe_expert_ffn(L.shape, hd, r.perm, r.offsets, r.counts, dw.w1, dw.w3, dw.w2, m, L.y, L.ws)
            want = L.y.clone()
            L.y.view(torch.int16).fill_(SENTINEL)
            before = torch.cuda.memory_allocated()
            B.moe_expert_ffn_static(L.shape, hd, r.perm, r.offsets, r.counts, dw.w1, dw.w3, dw.w2, m, L.y)
            assert torch.cuda.memory_allocated() == before
            torch.cuda.synchronize()
            assert torch.equal(L.y.view(torch.int16), want.view(torch.int16))
            assert bool((want.view(torch.int16) != SENTINEL).any())          # the comparison is not of two untouched buffers


def test_static_scratch_entry_point_rejects_shapes_beyond_its_array(gpu):
    B, Lm = gpu
    big = B.shape(2048, 4096, 8, 2, 14336)                                    # 117 MB of inner activations
    assert B.workspace_bytes(big) > B.static_scratch_bytes()
    z = C.c_void_p(0)
    one = torch.zeros(64, dtype=torch.int32, device="cuda")
    p = C.c_void_p(one.data_ptr())
    lib = B.load_library()
    assert lib.moe_expert_ffn_static(C.byref(big), p, p, p, p, p, p, p, z, p, z) == -5      # MOE_ETOOLARGE, nothing launched
    assert b"static scratch" in lib.moe_strerror(-5)
    small = B.shape(16, 512, 8, 2, 4608)
    assert lib.moe_expert_ffn_static(C.byref(small), z, p, p, p, p, p, p, z, p, z) == -1    # NULL h: MOE_EINVAL
