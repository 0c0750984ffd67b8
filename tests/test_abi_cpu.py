"""CPU-side tests of the C ABI: the library loads without a GPU, exports every function the
header declares, and rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import moe_oracle as O
from paper_2407_00599_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2407_00599_amd import build
    build.build()            # no-op when the library is newer than its sources
    return api.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "parm_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(L):
    names = declared_functions()
    assert len(names) >= 14
    for n in names:
        assert hasattr(L, n), n
    assert sorted(api.EXPORTED) == names
    for n in names:                       # the Python binding has the same names
        if n not in ("moe_strerror", "moe_abi_version"):
            assert hasattr(api, n), n
    assert L.moe_abi_version() == 6


def test_error_strings(L):
    for code in range(0, -7, -1):
        s = L.moe_strerror(code)
        assert s and b"unknown" not in s
    assert b"unknown" in L.moe_strerror(-99)


def test_capacity_matches_checker_and_rejects_bad_input(L):
    rng = np.random.default_rng(0)
    for _ in range(300):
        E = int(rng.integers(1, 257)); k = int(rng.integers(1, min(E, 8) + 1))
        S = int(rng.integers(1, 70000)); f = float(rng.choice([0.5, 1.0, 1.2, 1.25, 2.0, 2.4, 1.0 + rng.random()]))
        assert L.moe_capacity(S, E, k, f) == O.capacity(S, E, k, f)
    assert L.moe_capacity(0, 8, 2, 1.0) == -1
    assert L.moe_capacity(8, 8, 9, 1.0) == -1          # k > E
    assert L.moe_capacity(8, 8, 2, 0.0) == -1
    assert L.moe_capacity(8, 8, 2, float("nan")) == -1
    with pytest.raises(api.MoEError):
        api.moe_capacity(8, 2, 3, 1.0)


A = ctypes.c_void_p(0x1000)        # aligned dummy pointers: never dereferenced on these paths
U = ctypes.c_void_p(0x1004)        # misaligned


def test_gate_argument_checks(L):
    ws = L.moe_gate_workspace_bytes(256, 8, 2)
    assert ws > 0 and ws % 256 == 0
    ok = dict(x=A, xd=1, Wg=A, b=None, S=256, M=64, E=8, k=2, C=10, mp=0, nmp=1, norm=-1)

    def call(**kw):
        a = dict(ok); a.update(kw)
        return L.moe_gate_topk(a["x"], a["xd"], a["Wg"], a["b"], a["S"], a["M"], a["E"], a["k"], a["C"], a["mp"],
                               a["nmp"], a["norm"], a.get("lg", A), A, A, A, A, A, a.get("ws", A), a.get("wsb", ws), None)
    assert call(k=9, E=8) == -1                    # k > E
    assert call(k=0) == -1
    assert call(S=255, nmp=2) == -1                # S_total % n_mp != 0
    assert call(mp=1, nmp=1) == -1                 # mp_idx out of range
    assert call(C=0) == -1
    assert call(norm=2) == -1
    assert call(xd=7) == -1                        # unknown dtype
    assert call(E=300, k=2) == -2                  # beyond the build's limits
    assert call(k=9, E=16) == -2
    assert call(M=60) == -2                        # M % 8
    assert call(Wg=None) == -6
    assert call(lg=None) == -6
    assert call(x=U) == -3
    assert call(wsb=ws - 1) == -5
    assert call(ws=None) == -5
    # the variant with the library's static scratch array: same checks, and a size limit instead of a workspace
    def call_static(S=256, E=8, k=2, lg=A):
        return L.moe_gate_topk_static(A, 1, A, None, S, 64, E, k, 10, 0, 1, -1, lg, A, A, A, A, A, None)
    assert call_static(k=9) == -1 and call_static(lg=None) == -6 and call_static(lg=U) == -3
    assert L.moe_gate_workspace_bytes(1 << 20, 256, 8) > api.MOE_GATE_STATIC_SCRATCH_BYTES
    assert call_static(S=1 << 20, E=256, k=8) == -7
    assert b"static" in L.moe_strerror(-7)


def test_dispatch_combine_argument_checks(L):
    assert L.moe_dispatch(None, 1, 16, 64, 4, 2, 8, A, None, A, None) == -6
    assert L.moe_dispatch(A, 3, 16, 64, 4, 2, 8, A, None, A, None) == -1
    assert L.moe_dispatch(A, 1, 16, 64, 4, 5, 8, A, None, A, None) == -1       # k > E
    assert L.moe_dispatch(A, 1, 16, 64, 4, 2, 8, U, None, A, None) == -3
    assert L.moe_combine_fwd(A, 1, 0, 16, 64, 4, 2, 8, A, A, None, A, None) == -1   # n_part < 1
    assert L.moe_combine_fwd(A, 1, 1, 16, 64, 4, 2, 8, A, None, None, A, None) == -6
    assert L.moe_combine_bwd(A, A, 1, 1, 16, 64, 4, 2, 8, A, A, A, None, A, A, None) == -6   # w is required
    assert L.moe_combine_bwd(A, A, 0, 1, 0, 64, 4, 2, 8, A, A, A, A, A, A, None) == -1       # S < 1


def test_ffn_argument_checks(L):
    f = L.moe_ffn_workspace_bytes
    assert f(1, 2, 4, 100, 64, 256, 2) == api.moe_ffn_workspace_bytes(1, 2, 4, 100, 64, 256, 2)
    one = f(1, 2, 4, 100, 64, 256, 2)
    assert 2 * 4 * 100 * 128 * 2 <= one < 2 * 4 * 100 * 128 * 2 + 256
    assert f(0, 2, 4, 100, 64, 256, 2) >= 2 * 4 * 100 * 128 * 4
    assert f(1, 2, 4, 100, 64, 250, 4) == 0                 # H % n_esp != 0 -> invalid -> 0

    def fwd(dt=1, n_src=1, G=2, C=10, M=64, H=128, e=0, n=1, X=A, Z=A, Act=A, tile=0):
        return L.moe_expert_ffn_fwd(X, dt, A, A, n_src, G, C, M, H, e, n, None, tile, Z, Act, A, None)
    assert fwd(H=130, n=4) == -1
    assert fwd(e=2, n=2) == -1
    assert fwd(e=-1) == -1
    assert fwd(G=0) == -1
    assert fwd(dt=2) == -1
    assert fwd(M=60) == -2
    assert fwd(H=132, n=1) == -2                   # H_l % 8
    assert fwd(X=None) == -6
    assert fwd(Z=U) == -3
    assert fwd(Act=None) == -6
    assert fwd(tile=4) == -1 and fwd(tile=-1) == -1          # unknown tile hint
    def fwd_g(x=A, S=16, inv=A, k=2, E=2, C=10, M=64, H=128, Z=A):
        return L.moe_expert_ffn_fwd_gather(x, 1, S, inv, k, A, A, E, C, M, H, 0, 1, None, 0, Z, A, A, None)
    assert fwd_g(k=0) == -1 and fwd_g(k=9) == -1 and fwd_g(S=0) == -1
    assert fwd_g(inv=None) == -6 and fwd_g(x=None) == -6
    assert fwd_g(inv=U) == -3
    assert fwd_g(S=1 << 30, k=2) == -2             # S * k must stay below 2^31
    assert fwd_g(M=60) == -2
    assert fwd_g(S=(1 << 28) + 1, k=2) == -2 and fwd_g(S=1 << 28, k=2, x=None) == -6

    def bwd_g(x=A, S=16, inv=A, k=2, dW1=A, ws=A, wsb=1 << 30):
        return L.moe_expert_ffn_bwd_gather(A, x, S, inv, k, A, A, A, A, 1, 2, 10, 64, 128, 0, 1, None, 0, A, dW1, A, ws, wsb, None)
    assert bwd_g(k=0) == -1 and bwd_g(S=0) == -1
    assert bwd_g(inv=None) == -6 and bwd_g(x=U) == -3 and bwd_g(dW1=None) == -6
    assert bwd_g(wsb=64) == -5 and bwd_g(ws=None) == -5
    assert L.moe_expert_ffn_bwd(A, A, A, A, A, A, 1, 1, 2, 10, 64, 128, 0, 1, None, 0, A, A, None, A, 1 << 30, None) == -6
    assert L.moe_expert_ffn_bwd(A, A, A, None, A, A, 1, 1, 2, 10, 64, 128, 0, 1, None, 0, A, A, A, A, 1 << 30, None) == -6
    assert L.moe_expert_ffn_bwd(A, A, A, A, A, A, 1, 1, 2, 10, 64, 128, 0, 1, None, 0, A, A, A, A, 64, None) == -5
    assert L.moe_expert_ffn_bwd(A, A, A, A, A, A, 1, 1, 2, 10, 64, 128, 0, 1, None, 0, A, A, A, None, 1 << 30, None) == -5
    assert L.moe_expert_ffn_bwd(A, A, A, A, A, A, 1, 1, 2, 10, 64, 128, 0, 1, None, 9, A, A, A, A, 1 << 30, None) == -1


def test_executed_flops_accounting(L):
    """Host arithmetic only: executed work of the FFN calls for given row counts."""
    import numpy as np
    f = api.moe_ffn_executed_flops
    n_src, G, C, M, H = 1, 8, 1229, 1024, 4096
    full = 2.0 * G * C * M * H
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1) == 2 * full                 # two GEMMs over every row
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, None, True) == 4 * full
    assert f(api.MOE_F32, n_src, G, C, M, H, 1, np.zeros((1, G), np.int32)) == 2 * full   # fp32 kernels never skip
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, np.full((1, G), C, np.int32)) == 2 * full
    assert f(api.MOE_BF16, n_src, G, C, M, 4100, 3) == 0.0                 # invalid shape
    # empty experts: nothing is multiplied, forward or backward
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, np.zeros((1, G), np.int32)) == 0.0
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, np.zeros((1, G), np.int32), True) == 0.0
    # one token per expert: one row tile per expert in the row-tiled GEMMs, one row in the reductions
    one = np.ones((1, G), np.int32)
    t256 = api.MOE_TILE_256      # 256-row tiles everywhere
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, one, tile=t256) == 2 * (2.0 * G * 256 * M * H)
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, one, True, tile=t256) == 2 * (2.0 * G * 256 * M * H) + 2 * (2.0 * G * 1 * M * H)
    # counts above the capacity are clamped; a count on a tile edge needs no further tile
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, np.full((1, G), C + 7, np.int32), True, tile=t256) == 4 * full
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, np.full((1, G), 512, np.int32), tile=t256) == 2 * (2.0 * G * 512 * M * H)
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, np.full((1, G), 513, np.int32), tile=t256) == 2 * (2.0 * G * 768 * M * H)
    # several source chunks: the reductions run over all rows, the row tiles follow each chunk's count
    got = f(api.MOE_BF16, 2, G, 1024, M, H, 1, np.array([[0] * G, [1] * G], np.int32), True, tile=t256)
    assert got == 2 * (2.0 * G * 256 * M * H) + 2 * (2.0 * G * 2048 * M * H)
    # 192-row tiles in the row-tiled GEMMs only; the small kernel never skips; an unknown hint is an invalid call
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, one, tile=api.MOE_TILE_192) == 2 * (2.0 * G * 192 * M * H)
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, one, tile=api.MOE_TILE_SMALL) == 2 * full
    assert f(api.MOE_BF16, n_src, G, C, M, H, 1, one, tile=7) == 0.0


def test_gate_bwd_argument_checks(L):
    ws = L.moe_gate_bwd_workspace_bytes(512, 64, 8)
    assert ws >= 2 * 65 * 8 * 4

    def call(S=512, M=64, E=8, k=2, norm=1, acc=1, dw=A, dx=A, wsb=ws, xd=1):
        return L.moe_gate_bwd(dw, A, A, A, A, xd, A, S, M, E, k, norm, A, A, None, dx, acc, A, wsb, None)
    assert call(k=9) == -1
    assert call(acc=2) == -1
    assert call(norm=-2) == -1
    assert call(xd=5) == -1
    assert call(dw=None) == -6
    assert call(dx=U) == -3
    assert call(wsb=8) == -5
    assert call(E=257, k=2) == -2
