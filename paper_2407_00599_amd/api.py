"""Thin Python binding of libparm_moe's C ABI (include/parm_moe.h).

Argument marshalling only: each function here has the name and argument order of the C entry
point, takes torch tensors living on the GPU (PyTorch is used for device memory and streams,
nothing else), passes their device pointers and the current HIP stream through ctypes, and
raises MoEError on a negative return code.  There is no CPU fallback: if the shared library
has not been built, importing the symbols fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

MOE_F32, MOE_BF16 = 0, 1
MOE_TILE_AUTO, MOE_TILE_SMALL, MOE_TILE_256, MOE_TILE_192 = 0, 1, 2, 3
MOE_GATE_STATIC_SCRATCH_BYTES = 2 << 20
_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libparm_moe.so")

_lib = None


class MoEError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().moe_strerror(code).decode()} ({code})")


def lib() -> ctypes.CDLL:
    """Loads libparm_moe.so (built by `python -m paper_2407_00599_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2407_00599_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        c_i, c_i64, c_p, c_sz, c_d = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_double
        L.moe_strerror.restype = ctypes.c_char_p
        L.moe_strerror.argtypes = [c_i]
        L.moe_abi_version.restype = c_i
        L.moe_capacity.restype = c_i64
        L.moe_capacity.argtypes = [c_i64, c_i, c_i, c_d]
        L.moe_gate_workspace_bytes.restype = c_sz
        L.moe_gate_workspace_bytes.argtypes = [c_i64, c_i, c_i]
        L.moe_gate_topk.restype = c_i
        L.moe_gate_topk.argtypes = [c_p, c_i, c_p, c_p, c_i64, c_i, c_i, c_i, c_i64, c_i, c_i, c_i,
                                    c_p, c_p, c_p, c_p, c_p, c_p, c_p, c_sz, c_p]
        L.moe_gate_topk_static.restype = c_i
        L.moe_gate_topk_static.argtypes = [c_p, c_i, c_p, c_p, c_i64, c_i, c_i, c_i, c_i64, c_i, c_i, c_i,
                                           c_p, c_p, c_p, c_p, c_p, c_p, c_p]
        L.moe_dispatch.restype = c_i
        L.moe_dispatch.argtypes = [c_p, c_i, c_i64, c_i, c_i, c_i, c_i64, c_p, c_p, c_p, c_p]
        L.moe_ffn_workspace_bytes.restype = c_sz
        L.moe_ffn_workspace_bytes.argtypes = [c_i, c_i, c_i, c_i64, c_i, c_i, c_i]
        L.moe_alpha_beta_fit.restype = c_i
        L.moe_alpha_beta_fit.argtypes = [c_p, c_p, c_i, c_p, c_p]
        L.moe_choose_schedule.restype = c_i
        L.moe_choose_schedule.argtypes = [ctypes.c_double] * 6 + [c_i64, c_i64, c_i, c_i, c_i, ctypes.c_double, c_i, c_i,
                                          c_p, c_p]
        L.moe_dispatch_slots.restype = c_i
        L.moe_dispatch_slots.argtypes = [c_p, c_i, c_i64, c_i, c_i, c_i, c_i64, c_i64, c_i64, c_p, c_p, c_p, c_p]
        L.moe_ffn_executed_flops.restype = ctypes.c_double
        L.moe_ffn_executed_flops.argtypes = [c_i, c_i, c_i, c_i64, c_i, c_i, c_i, c_p, c_i, c_i]
        L.moe_expert_ffn_fwd.restype = c_i
        L.moe_expert_ffn_fwd.argtypes = [c_p, c_i, c_p, c_p, c_i, c_i, c_i64, c_i, c_i, c_i, c_i,
                                         c_p, c_i, c_p, c_p, c_p, c_p]
        L.moe_expert_ffn_fwd_gather.restype = c_i
        L.moe_expert_ffn_fwd_gather.argtypes = [c_p, c_i, c_i64, c_p, c_i, c_p, c_p, c_i, c_i64, c_i, c_i, c_i, c_i,
                                                c_p, c_i, c_p, c_p, c_p, c_p]
        L.moe_expert_ffn_bwd_gather.restype = c_i
        L.moe_expert_ffn_bwd_gather.argtypes = [c_p, c_p, c_i64, c_p, c_i, c_p, c_p, c_p, c_p, c_i, c_i, c_i64, c_i, c_i,
                                                c_i, c_i, c_p, c_i, c_p, c_p, c_p, c_p, c_sz, c_p]
        L.moe_expert_ffn_bwd.restype = c_i
        L.moe_expert_ffn_bwd.argtypes = [c_p, c_p, c_p, c_p, c_p, c_p, c_i, c_i, c_i, c_i64, c_i, c_i, c_i, c_i,
                                         c_p, c_i, c_p, c_p, c_p, c_p, c_sz, c_p]
        L.moe_combine_fwd.restype = c_i
        L.moe_combine_fwd.argtypes = [c_p, c_i, c_i, c_i64, c_i, c_i, c_i, c_i64, c_p, c_p, c_p, c_p, c_p]
        L.moe_combine_bwd.restype = c_i
        L.moe_combine_bwd.argtypes = [c_p, c_p, c_i, c_i, c_i64, c_i, c_i, c_i, c_i64, c_p, c_p, c_p, c_p,
                                      c_p, c_p, c_p]
        L.moe_gate_bwd_workspace_bytes.restype = c_sz
        L.moe_gate_bwd_workspace_bytes.argtypes = [c_i64, c_i, c_i]
        L.moe_gate_bwd.restype = c_i
        L.moe_gate_bwd.argtypes = [c_p, c_p, c_p, c_p, c_p, c_i, c_p, c_i64, c_i, c_i, c_i, c_i,
                                   c_p, c_p, c_p, c_p, c_i, c_p, c_sz, c_p]
        _lib = L
    return _lib


EXPORTED = [
    "moe_strerror", "moe_abi_version", "moe_capacity", "moe_gate_workspace_bytes", "moe_gate_topk",
    "moe_gate_topk_static",
    "moe_dispatch", "moe_dispatch_slots", "moe_ffn_workspace_bytes", "moe_ffn_executed_flops", "moe_expert_ffn_fwd", "moe_expert_ffn_fwd_gather",
    "moe_expert_ffn_bwd", "moe_expert_ffn_bwd_gather",
    "moe_combine_fwd", "moe_combine_bwd", "moe_gate_bwd_workspace_bytes", "moe_gate_bwd", "moe_alpha_beta_fit",
    "moe_choose_schedule",
]


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensors must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensors must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def dtype_code(t) -> int:
    if t.dtype == torch.bfloat16:
        return MOE_BF16
    if t.dtype == torch.float32:
        return MOE_F32
    raise ValueError(f"unsupported dtype {t.dtype}")


def _check(rc: int, where: str):
    if rc != 0:
        raise MoEError(rc, where)


def _ws_args(ws):
    if ws is None:
        return None, 0
    return _ptr(ws), ws.numel() * ws.element_size()


def moe_capacity(S: int, E: int, k: int, f: float) -> int:
    c = lib().moe_capacity(S, E, k, f)
    if c < 0:
        raise MoEError(-1, "moe_capacity")
    return int(c)


def moe_gate_workspace_bytes(S, E, k) -> int:
    return int(lib().moe_gate_workspace_bytes(S, E, k))


def moe_ffn_workspace_bytes(dtype, n_src, G, C, M, H, n_esp) -> int:
    return int(lib().moe_ffn_workspace_bytes(dtype, n_src, G, C, M, H, n_esp))


def moe_gate_bwd_workspace_bytes(S, M, E) -> int:
    return int(lib().moe_gate_bwd_workspace_bytes(S, M, E))


def moe_gate_topk(x, Wg, gate_bias, S_total, M, E, k, C, mp_idx, n_mp, norm_topk,
                  logits, idx, slot, w, inv, counts, ws):
    wp, wb = _ws_args(ws)
    _check(lib().moe_gate_topk(_ptr(x), dtype_code(x) if x is not None else MOE_F32, _ptr(Wg), _ptr(gate_bias),
                               S_total, M, E, k, C, mp_idx, n_mp, norm_topk,
                               _ptr(logits), _ptr(idx), _ptr(slot), _ptr(w), _ptr(inv), _ptr(counts),
                               wp, wb, _stream()), "moe_gate_topk")


def moe_gate_topk_static(x, Wg, gate_bias, S_total, M, E, k, C, mp_idx, n_mp, norm_topk,
                         logits, idx, slot, w, inv, counts):
    _check(lib().moe_gate_topk_static(_ptr(x), dtype_code(x) if x is not None else MOE_F32, _ptr(Wg), _ptr(gate_bias),
                                      S_total, M, E, k, C, mp_idx, n_mp, norm_topk,
                                      _ptr(logits), _ptr(idx), _ptr(slot), _ptr(w), _ptr(inv), _ptr(counts),
                                      _stream()), "moe_gate_topk_static")


def moe_dispatch(x, S, M, E, k, C, inv, w, buf):
    _check(lib().moe_dispatch(_ptr(x), dtype_code(x), S, M, E, k, C, _ptr(inv), _ptr(w), _ptr(buf), _stream()),
           "moe_dispatch")


def moe_alpha_beta_fit(xs, ts):
    """Host arrays in, (alpha, beta) out."""
    n = len(xs)
    ax = (ctypes.c_double * n)(*[float(v) for v in xs])
    at = (ctypes.c_double * len(ts))(*[float(v) for v in ts])
    a, b = ctypes.c_double(), ctypes.c_double()
    _check(lib().moe_alpha_beta_fit(ax, at, min(n, len(ts)) if n == len(ts) else 0, ctypes.byref(a), ctypes.byref(b)),
           "moe_alpha_beta_fit")
    return a.value, b.value


def moe_choose_schedule(a_ag, b_ag, a_a2a, b_a2a, a_o, b_o, B, L, E, M, k, f, n_esp, n_mp):
    """Returns (schedule, t_D1, t_D2) with schedule 1 or 2."""
    t1, t2 = ctypes.c_double(), ctypes.c_double()
    rc = lib().moe_choose_schedule(a_ag, b_ag, a_a2a, b_a2a, a_o, b_o, B, L, E, M, k, f, n_esp, n_mp, ctypes.byref(t1),
                                   ctypes.byref(t2))
    if rc < 0:
        _check(rc, "moe_choose_schedule")
    return rc, t1.value, t2.value


def moe_dispatch_slots(x, S, M, E, k, C, c0, c1, inv, w, buf):
    _check(lib().moe_dispatch_slots(_ptr(x), dtype_code(x), S, M, E, k, C, c0, c1, _ptr(inv), _ptr(w), _ptr(buf),
                                    _stream()), "moe_dispatch_slots")


def moe_ffn_executed_flops(dtype, n_src, G, C, M, H, n_esp, row_counts_host=None, backward=False, tile=0) -> float:
    """row_counts_host: a host int32 array [n_src, G] (numpy or CPU tensor) or None."""
    ptr = None
    if row_counts_host is not None:
        import numpy as np
        arr = np.ascontiguousarray(np.asarray(row_counts_host, dtype=np.int32))
        assert arr.size == n_src * G
        ptr = arr.ctypes.data_as(ctypes.c_void_p)
    return float(lib().moe_ffn_executed_flops(dtype, n_src, G, C, M, H, n_esp, ptr, tile, int(backward)))


def moe_expert_ffn_fwd(X, W1, W2, n_src, G, C, M, H, esp_idx, n_esp, Z, A, Y, row_counts=None, tile=0):
    _check(lib().moe_expert_ffn_fwd(_ptr(X), dtype_code(X), _ptr(W1), _ptr(W2), n_src, G, C, M, H, esp_idx, n_esp,
                                    _ptr(row_counts), tile, _ptr(Z), _ptr(A), _ptr(Y), _stream()), "moe_expert_ffn_fwd")


def moe_expert_ffn_fwd_gather(x, inv, S, k, W1, W2, E, C, M, H, esp_idx, n_esp, Z, A, Y, row_counts=None, tile=0):
    _check(lib().moe_expert_ffn_fwd_gather(_ptr(x), dtype_code(x), S, _ptr(inv), k, _ptr(W1), _ptr(W2), E, C, M, H,
                                           esp_idx, n_esp, _ptr(row_counts), tile, _ptr(Z), _ptr(A), _ptr(Y), _stream()),
           "moe_expert_ffn_fwd_gather")


def moe_expert_ffn_bwd(dY, X, Z, A, W1, W2, n_src, G, C, M, H, esp_idx, n_esp, dX, dW1, dW2, ws, row_counts=None,
                       tile=0):
    wp, wb = _ws_args(ws)
    _check(lib().moe_expert_ffn_bwd(_ptr(dY), _ptr(X), _ptr(Z), _ptr(A), _ptr(W1), _ptr(W2), dtype_code(X),
                                    n_src, G, C, M, H, esp_idx, n_esp, _ptr(row_counts), tile, _ptr(dX), _ptr(dW1),
                                    _ptr(dW2), wp, wb, _stream()), "moe_expert_ffn_bwd")


def moe_expert_ffn_bwd_gather(dY, x, inv, S, k, Z, A, W1, W2, E, C, M, H, esp_idx, n_esp, dX, dW1, dW2, ws,
                              row_counts=None, tile=0):
    wp, wb = _ws_args(ws)
    _check(lib().moe_expert_ffn_bwd_gather(_ptr(dY), _ptr(x), S, _ptr(inv), k, _ptr(Z), _ptr(A), _ptr(W1), _ptr(W2),
                                           dtype_code(x), E, C, M, H, esp_idx, n_esp, _ptr(row_counts), tile, _ptr(dX),
                                           _ptr(dW1), _ptr(dW2), wp, wb, _stream()), "moe_expert_ffn_bwd_gather")


def moe_combine_fwd(Yret, n_part, S, M, E, k, C, idx, slot, w, y):
    _check(lib().moe_combine_fwd(_ptr(Yret), dtype_code(Yret), n_part, S, M, E, k, C, _ptr(idx), _ptr(slot),
                                 _ptr(w), _ptr(y), _stream()), "moe_combine_fwd")


def moe_combine_bwd(dy, Yret, n_part, S, M, E, k, C, idx, slot, inv, w, dYret, dw):
    _check(lib().moe_combine_bwd(_ptr(dy), _ptr(Yret), dtype_code(dy), n_part, S, M, E, k, C, _ptr(idx),
                                 _ptr(slot), _ptr(inv), _ptr(w), _ptr(dYret), _ptr(dw), _stream()),
           "moe_combine_bwd")


def moe_gate_bwd(dw, w, idx, logits, x, Wg, S, M, E, k, norm_topk, dlogits, dWg, dgate_bias, dx,
                 dx_accumulate, ws):
    wp, wb = _ws_args(ws)
    _check(lib().moe_gate_bwd(_ptr(dw), _ptr(w), _ptr(idx), _ptr(logits), _ptr(x), dtype_code(x), _ptr(Wg),
                              S, M, E, k, norm_topk, _ptr(dlogits), _ptr(dWg), _ptr(dgate_bias), _ptr(dx),
                              int(dx_accumulate), wp, wb, _stream()), "moe_gate_bwd")
