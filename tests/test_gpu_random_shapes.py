"""GPU parity on randomly drawn (seeded) layer shapes: token counts that are not multiples of any
tile, tiny and odd model sizes, up to 24 experts, top-1 to top-4, capacity factors from starving to
generous, MP slices and ESP shards, both storage types.  Every tensor of the forward and backward
pass is compared with the CPU checker as in test_gpu_layer."""
import numpy as np
import pytest

from paper_2407_00599_amd import synth
from test_gpu_layer import run_layer, compare

pytestmark = pytest.mark.gpu


def draw(seed):
    rng = np.random.default_rng(9000 + seed)
    n_mp = int(rng.choice([1, 1, 2, 3]))
    n_esp = int(rng.choice([1, 1, 2, 4]))
    E = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 17, 24]))
    k = int(rng.integers(1, min(E, 4) + 1))
    S = int(rng.integers(1, 260)) * n_mp
    M = 8 * int(rng.integers(1, 34))
    H = 8 * n_esp * int(rng.integers(1, 66 // n_esp + 1))
    f = float(rng.choice([0.25, 0.5, 1.0, 1.25, 2.0, 4.0]))
    dtype = str(rng.choice(["bf16", "f32"]))
    bias = str(rng.choice(["none", "normal"]))
    norm = int(rng.integers(0, 2))
    cfg = synth.MoEConfig(f"random{seed}", S, M, H, E, k, f, dtype=dtype, n_mp=n_mp, mp_idx=int(rng.integers(0, n_mp)),
                          bias=bias, sigma_x=1.0, sigma_w=0.05, cfg_id=100 + seed)
    return cfg, n_esp, norm


@pytest.mark.parametrize("seed", range(32))
def test_random_layer_shapes(seed):
    cfg, n_esp, norm = draw(seed)
    L, r, g, _, _ = run_layer(cfg, n_esp, norm)
    compare(L, r, g, cfg.dtype, cfg.bias != "none")
