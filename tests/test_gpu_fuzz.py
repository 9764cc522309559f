"""Seeded random layer shapes against the oracle: sizes, expert counts, batch sizes and masks drawn from the ranges the
library accepts (small enough for the oracle), so that the combinations the hand-picked cases skip get exercised too:
every kernel path (decode kernels, single-tile and scheduled tiled kernels, half-width and split-K items, shared experts)
is chosen by the library from the shape and the mask, not by the test."""
import numpy as np
import pytest

from paper_2602_03495_amd import workloads as wl
from test_gpu_parity import _run_layer

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

BASES = ["tiny", "mixtral", "deepseek", "qwen15", "qwen3"]
D = [128, 256, 384, 512, 1024]
INNER = [128, 256, 384, 640, 1152, 2176, 4096]
TOKENS = [1, 2, 3, 7, 15, 16, 17, 31, 33, 64, 65, 100, 128, 129, 200, 257, 400]


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    base = wl.CONFIGS[BASES[rng.integers(len(BASES))]]
    kw = dict(d=int(rng.choice(D)), I=int(rng.choice(INNER)))
    if base.n_shared:
        kw["I_shared"] = int(rng.choice([128, 256, 384]))
    cfg = wl.scaled(base, **kw)
    T = int(rng.choice(TOKENS))
    n_on = int(rng.integers(0, cfg.N + 1))
    return cfg, T, n_on


@pytest.mark.parametrize("seed", range(16))
def test_random_layer_shape_matches_the_oracle(seed):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding as B, layer as Lm
    B.load_library()
    cfg, T, n_on = _case(seed)
    print(f"fuzz {seed}: {cfg.name} d={cfg.d} I={cfg.I} N={cfg.N} k={cfg.k} shared={cfg.n_shared}x{cfg.I_shared} T={T} on={n_on}", flush=True)
    masks = [wl.mask_random(cfg, n_on) if n_on else np.zeros(cfg.N, np.uint8), None]
    _run_layer(B, Lm, cfg, T, masks, B.FFN_AUTO)


def _big_case(seed):
    # hundreds to thousands of tokens on narrow layers (the oracle stays within seconds): several token tiles per expert,
    # ragged last tiles, tile tables built on the device, the down projection's choice of tile height
    rng = np.random.default_rng(5000 + seed)
    base = wl.CONFIGS[BASES[rng.integers(len(BASES))]]
    kw = dict(d=int(rng.choice([128, 256, 384])), I=int(rng.choice([128, 256, 384, 640, 896])))
    if base.n_shared:
        kw["I_shared"] = int(rng.choice([128, 256]))
    cfg = wl.scaled(base, **kw)
    T = int(rng.integers(300, 4500 if cfg.k <= 2 else 2600))
    n_on = int(rng.integers(1, cfg.N + 1))
    return cfg, T, n_on


@pytest.mark.parametrize("seed", range(12))
def test_random_large_batch_matches_the_oracle(seed):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03495_amd import binding as B, layer as Lm
    B.load_library()
    cfg, T, n_on = _big_case(seed)
    print(f"fuzz large {seed}: {cfg.name} d={cfg.d} I={cfg.I} N={cfg.N} k={cfg.k} shared={cfg.n_shared}x{cfg.I_shared} T={T} on={n_on}", flush=True)
    masks = [wl.mask_random(cfg, n_on)] if seed % 2 else [None]
    _run_layer(B, Lm, cfg, T, masks, B.FFN_AUTO)
