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


def torch_dtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16
