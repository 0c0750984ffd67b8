"""Shared helpers of the GPU parity tests (host <-> device marshalling, error measures)."""
import numpy as np
import torch

from paper_2407_00599_amd import synth

DEV = "cuda:0"


def to_dev(st):
    """synth.Stored (or a plain float32 / int32 ndarray) -> device tensor with the same bits."""
    if isinstance(st, synth.Stored):
        if st.bits is None:
            return torch.from_numpy(st.val).to(DEV)
        return torch.from_numpy(st.bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(st)).to(DEV)


def to_host(t):
    """device tensor -> float64 / integer ndarray (bf16 decoded exactly)."""
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    if t.dtype == torch.float32:
        return t.cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


def rel_err(got, ref):
    """tensor-wise max|got-ref| / max|ref| (0 when both are all-zero)."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max() if ref.size else 0.0
    num = np.abs(got - ref).max() if ref.size else 0.0
    if den == 0.0:
        return 0.0 if num == 0.0 else np.inf
    return num / den


TOL = {"f32": 1e-5, "bf16": 2e-2}


FLOOR = 2.0   # per-element bound: |got - ref| <= tol (|ref| + FLOOR rms of the element's group)


def elem_excess(got, ref, tol, group=None):
    """Per-element measure: max over the elements of |got - ref| / (tol (|ref| + FLOOR rms)); at most 1 passes.
    rms is the root mean square of ref over the axes `group` (all axes if None), i.e. over the sums that share the
    element's scale: a row of an activation tensor (group = the last axis: its rows differ in scale, padding rows
    are zero), one expert's matrix of a weight gradient (group = (1, 2)).
    Why a floor at all: an output that is a sum of K rounded products carries an absolute error that scales with
    the size of the terms (eps sqrt(K) times a typical term), however small the sum itself came out, so an element
    far below its group's rms cannot be asked for relative accuracy; it can be asked not to be off by more than
    tol times a small multiple of that rms.  FLOOR = 2: the bf16 path rounds the pre-activation, the activation,
    its gradient and the result (2^-9 relative each); over the 1e6..1e8 elements of a tensor the largest of the
    resulting errors reaches about 6 standard deviations, 0.02..0.03 rms in a CPU emulation of exactly those
    roundings, against the 0.04 rms this allows.  The tensor-wise bound alone would allow tol max|ref|, about
    0.11 rms of the WHOLE tensor, for every element of every group.  A group whose ref is all zero must be
    exactly zero."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    if ref.size == 0:
        return 0.0
    axes = tuple(range(ref.ndim)) if group is None else group
    rms = np.sqrt(np.mean(ref * ref, axis=axes, keepdims=True))
    d = np.abs(got - ref)
    den = tol * (np.abs(ref) + FLOOR * rms)
    live = den > 0
    if (d[~live] != 0).any():
        return np.inf
    return float((d[live] / den[live]).max()) if live.any() else 0.0


ROWS = (-1,)          # group of an activation tensor [..., M]: one row
EXPERT = (1, 2)       # group of a weight gradient [G, ., .]: one expert's matrix


def assert_close(got, ref, tol, name="", group=None):
    """The tensor-wise bound (max|got - ref| <= tol max|ref|) and the per-element one (elem_excess)."""
    e = rel_err(got, ref)
    assert e <= tol, (name, "tensor-wise", e)
    x = elem_excess(got, ref, tol, group)
    assert x <= 1.0, (name, "per element", x)


def torch_dtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16
