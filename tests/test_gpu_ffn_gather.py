"""GPU parity: expert FFN forward and backward with the dispatch fused into the GEMMs (rows read from
the token matrix through the inverse slot map: by the first GEMM, and by the weight gradient of the
first GEMM) against the CPU checker, and value for value against the unfused calls (dispatch, then the
FFN), which compute the same products in the same order from the same bits."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2407_00599_amd import api, synth
from util import DEV, TOL, to_dev, to_host, rel_err, torch_dtype

pytestmark = pytest.mark.gpu


def random_inverse_map(rng, S, k, E, C, fill):
    """A valid inverse slot map: distinct choices t*k+j, the first occ[e] slots of expert e occupied."""
    choices = rng.permutation(S * k)
    inv = np.full((E, C), -1, np.int32)
    occ = np.zeros(E, np.int32)
    pos = 0
    for e in range(E):
        n = int(min(C, rng.integers(0, int(fill * C) + 2), S * k - pos))
        inv[e, :n] = choices[pos:pos + n]
        occ[e] = n
        pos += n
    return inv, occ


CASES = [
    # S, k, E, C, M, H, n_esp, esp_idx, dtype, tile, fill
    (64, 2, 4, 40, 64, 128, 1, 0, "f32", 0, 1.0),
    (100, 1, 3, 50, 72, 256, 2, 1, "f32", 0, 0.5),
    (256, 2, 2, 130, 128, 256, 1, 0, "bf16", api.MOE_TILE_SMALL, 1.0),   # 128x128 register-staged kernel
    (700, 2, 2, 300, 512, 768, 1, 0, "bf16", api.MOE_TILE_256, 1.0),     # 256-row LDS-DMA tiles
    (700, 2, 3, 230, 264, 1040, 2, 0, "bf16", api.MOE_TILE_192, 0.7),    # 192-row tiles, ESP slice, ragged everything
    (512, 4, 4, 600, 256, 512, 1, 0, "bf16", 0, 0.4),                    # mostly empty slots
    (9, 8, 8, 20, 136, 520, 1, 0, "bf16", api.MOE_TILE_256, 1.0),        # k = E = 8, few tokens
]


@pytest.mark.parametrize("S,k,E,C,M,H,n_esp,esp_idx,dtype,tile,fill", CASES)
@pytest.mark.parametrize("with_counts", [False, True])
def test_fused_dispatch_forward(S, k, E, C, M, H, n_esp, esp_idx, dtype, tile, fill, with_counts):
    rng = np.random.default_rng(S * 31 + C)
    tdt = torch_dtype(dtype)
    x = synth.store(rng.standard_normal((S, M)).astype(np.float32), dtype)
    W1 = synth.store((rng.standard_normal((E, M, H)) / np.sqrt(M)).astype(np.float32), dtype)
    W2 = synth.store((rng.standard_normal((E, H, M)) / np.sqrt(H)).astype(np.float32), dtype)
    inv, occ = random_inverse_map(rng, S, k, E, C, fill)
    Hl = H // n_esp
    xd, W1d, W2d, invd = to_dev(x), to_dev(W1), to_dev(W2), to_dev(inv)
    cnt = to_dev(occ.reshape(1, E)) if with_counts else None
    new = lambda *s: torch.full(s, 7.0, dtype=tdt, device=DEV)
    Z, A, Y = new(1, E, C, Hl), new(1, E, C, Hl), new(1, E, C, M)
    Z2, A2, Y2 = new(1, E, C, Hl), new(1, E, C, Hl), new(1, E, C, M)
    buf = new(E, C, M)
    api.moe_expert_ffn_fwd_gather(xd, invd, S, k, W1d, W2d, E, C, M, H, esp_idx, n_esp, Z, A, Y, cnt, tile)
    api.moe_dispatch(xd, S, M, E, k, C, invd, None, buf)
    api.moe_expert_ffn_fwd(buf, W1d, W2d, 1, E, C, M, H, esp_idx, n_esp, Z2, A2, Y2, cnt, tile)
    torch.cuda.synchronize()
    # the definition: slot (e, c) holds token inv // k, or nothing
    X = O.dispatch(x.val, inv, k)[None]
    rZ, rY = O.expert_ffn_fwd(X, W1.val, W2.val, esp_idx, n_esp)
    tol = TOL[dtype]
    assert rel_err(to_host(Z), rZ) <= tol
    assert rel_err(to_host(A), O.gelu(rZ)) <= tol
    assert rel_err(to_host(Y), rY) <= tol
    # the same bits as the unfused calls
    assert torch.equal(Z, Z2) and torch.equal(A, A2) and torch.equal(Y, Y2)
    # empty slots give exactly zero
    empty = torch.from_numpy(inv < 0).to(DEV)
    assert not Z[0][empty].any() and not Y[0][empty].any()

    # backward: dY has zero rows at the empty slots (as the combine backward writes it)
    dYn = rng.standard_normal((1, E, C, M)).astype(np.float32)
    dYn[0][inv < 0] = 0
    dY = synth.store(dYn, dtype); dYd = to_dev(dY)
    dt = api.MOE_BF16 if dtype == "bf16" else api.MOE_F32
    ws = torch.empty(api.moe_ffn_workspace_bytes(dt, 1, E, C, M, H, n_esp), dtype=torch.uint8, device=DEV)
    outs = []
    for fused in (True, False):
        dX = new(1, E, C, M); dW1 = torch.full((E, M, H), 3.0, dtype=tdt, device=DEV)
        dW2 = torch.full((E, H, M), 3.0, dtype=tdt, device=DEV)
        if fused:
            api.moe_expert_ffn_bwd_gather(dYd, xd, invd, S, k, Z, A, W1d, W2d, E, C, M, H, esp_idx, n_esp, dX, dW1,
                                          dW2, ws, cnt, tile)
        else:
            api.moe_expert_ffn_bwd(dYd, buf.view(1, E, C, M), Z2, A2, W1d, W2d, 1, E, C, M, H, esp_idx, n_esp, dX,
                                   dW1, dW2, ws, cnt, tile)
        torch.cuda.synchronize()
        outs.append((dX, dW1, dW2))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    rdX, rdW1, rdW2 = O.expert_ffn_bwd(dY.val, X, W1.val, W2.val, esp_idx, n_esp)
    hs = slice(esp_idx * Hl, (esp_idx + 1) * Hl)
    dX, dW1, dW2 = outs[0]
    assert rel_err(to_host(dX), rdX) <= tol
    assert rel_err(to_host(dW1)[:, :, hs], rdW1) <= tol
    assert rel_err(to_host(dW2)[:, hs, :], rdW2) <= tol


def test_out_of_range_indices_read_as_empty_slots():
    """An index past the token matrix is never dereferenced: the slot is treated as empty."""
    S, k, E, C, M, H = 32, 2, 2, 40, 64, 128
    rng = np.random.default_rng(5)
    for dtype in ("f32", "bf16"):
        tdt = torch_dtype(dtype)
        x = to_dev(synth.store(rng.standard_normal((S, M)).astype(np.float32), dtype))
        W1 = to_dev(synth.store(rng.standard_normal((E, M, H)).astype(np.float32), dtype))
        W2 = to_dev(synth.store(rng.standard_normal((E, H, M)).astype(np.float32), dtype))
        inv = np.full((E, C), -1, np.int32)
        inv[0, 0] = 3; inv[0, 1] = S * k; inv[1, 2] = 2 ** 31 - 1
        Z = torch.empty(1, E, C, H, dtype=tdt, device=DEV); A = torch.empty_like(Z)
        Y = torch.empty(1, E, C, M, dtype=tdt, device=DEV)
        api.moe_expert_ffn_fwd_gather(x, to_dev(inv), S, k, W1, W2, E, C, M, H, 0, 1, Z, A, Y)
        torch.cuda.synchronize()
        assert Y[0, 0, 0].any() and not Y[0, 0, 1:].any() and not Y[0, 1].any()
