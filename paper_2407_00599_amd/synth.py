"""Seeded synthetic inputs for the MoE-layer hot path.

This module holds no arithmetic of the method itself: it only draws random
tensors with the shapes and value distributions of the paper's MoE-layer
workloads (Table 3 shape grid: B, L, M, H, f; E and k supplied by the
benchmark configs), rounds them to the storage dtype on the host, and hands
the identical values to whoever asks (the HIP path and the CPU checker both
take their inputs from here; neither takes inputs from the other).

bf16 tensors are returned as uint16 bit patterns next to the float32 values
those patterns decode to, so both consumers see exactly the same numbers.
"""
from __future__ import annotations

import dataclasses

import numpy as np

BASE_SEED = 240700599


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    """One rank's share of an MP+EP+ESP MoE layer (Table 1 notation).

    S_total tokens enter the layer (B*L); the rank gates the slice mp_idx of
    n_mp (Section III-B, schedule S1).  E experts in total, n_ep expert-parallel
    ranks (G = E/n_ep local experts), hidden size H split n_esp ways.
    """
    name: str
    S_total: int
    M: int
    H: int
    E: int
    k: int
    f: float
    dtype: str = "bf16"        # "bf16" or "f32": storage dtype of activations / expert weights
    n_mp: int = 1
    mp_idx: int = 0
    n_ep: int = 1
    n_esp: int = 1
    esp_idx: int = 0
    sigma_x: float = 1.0
    sigma_w: float = 0.02
    bias: str = "none"         # "none" | "normal" | "zipf"
    cfg_id: int = 0

    @property
    def S(self) -> int:
        return self.S_total // self.n_mp

    @property
    def G(self) -> int:
        return self.E // self.n_ep

    @property
    def n_src(self) -> int:
        return self.n_ep * self.n_esp

    @property
    def H_local(self) -> int:
        return self.H // self.n_esp


# The five benchmark configurations (index 0 is the small fp32 case).
CONFIGS = {
    "tiny_fp32": MoEConfig("tiny_fp32", 256, 64, 128, 4, 1, 1.2, dtype="f32",
                           sigma_x=0.02, sigma_w=0.02, cfg_id=1),
    "layer_bf16": MoEConfig("layer_bf16", 4096, 1024, 4096, 8, 2, 1.2, cfg_id=2),
    "mp4_ep": MoEConfig("mp4_ep", 8192, 768, 3072, 16, 2, 1.0, n_mp=4, mp_idx=1,
                        n_ep=4, bias="normal", cfg_id=3),
    "esp4": MoEConfig("esp4", 16384, 2048, 8192, 64, 2, 1.25, n_ep=8, n_esp=4,
                      esp_idx=1, bias="zipf", cfg_id=4),
    "large": MoEConfig("large", 32768, 4096, 14336, 8, 2, 1.0, n_esp=2, esp_idx=0,
                       sigma_w=0.01, cfg_id=5),
}
CONFIG_ORDER = ["tiny_fp32", "layer_bf16", "mp4_ep", "esp4", "large"]


def rng_for(cfg_id: int, tensor_id: int, extra: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * cfg_id + tensor_id + 100000 * extra))


# ---- storage rounding (host side, so both consumers get identical values) ----

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16).  Inputs are finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclasses.dataclass
class Stored:
    """A tensor as stored on the device: `bits` (uint16 bf16 patterns, or None for fp32)
    and `val`, the float32 values the stored tensor decodes to."""
    val: np.ndarray
    bits: np.ndarray | None

    @property
    def shape(self):
        return self.val.shape


def store(a: np.ndarray, dtype: str) -> Stored:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return Stored(a, None)
    if dtype == "bf16":
        bits = f32_to_bf16_bits(a)
        return Stored(bf16_bits_to_f32(bits), bits)
    raise ValueError(dtype)


def normal(shape, sigma: float, gen: np.random.Generator) -> np.ndarray:
    out = gen.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        out *= np.float32(sigma)
    return out


# ---- per-tensor generators (tensor ids are fixed so a tensor can be drawn alone) ----

T_X, T_WG, T_BIAS, T_W1, T_W2, T_DY, T_LOGITS, T_RECV, T_DYRECV = range(1, 10)


def gate_bias(cfg: MoEConfig) -> np.ndarray | None:
    """Per-expert additive gate bias that skews routing (None for uniform routing)."""
    if cfg.bias == "none":
        return None
    gen = rng_for(cfg.cfg_id, T_BIAS)
    if cfg.bias == "normal":
        return gen.standard_normal(cfg.E).astype(np.float32)
    if cfg.bias == "zipf":
        # popularity rank pi(e) of expert e is a seeded permutation; softmax mass ~ (1+pi)^-1.1
        perm = gen.permutation(cfg.E)
        return (-1.1 * np.log1p(perm.astype(np.float64))).astype(np.float32)
    raise ValueError(cfg.bias)


def tokens(cfg: MoEConfig) -> Stored:
    """Layer input I flattened to [S_total, M] (all MP ranks hold the full tensor)."""
    return store(normal((cfg.S_total, cfg.M), cfg.sigma_x, rng_for(cfg.cfg_id, T_X)), cfg.dtype)


def gate_weight(cfg: MoEConfig) -> np.ndarray:
    return normal((cfg.M, cfg.E), cfg.sigma_w, rng_for(cfg.cfg_id, T_WG))


def expert_weights(cfg: MoEConfig, n_experts: int, first_expert: int = 0):
    """W1 [n,M,H], W2 [n,H,M] for experts first_expert .. first_expert+n-1 (full H)."""
    w1 = np.empty((n_experts, cfg.M, cfg.H), dtype=np.float32)
    w2 = np.empty((n_experts, cfg.H, cfg.M), dtype=np.float32)
    for i in range(n_experts):
        e = first_expert + i
        w1[i] = normal((cfg.M, cfg.H), cfg.sigma_w, rng_for(cfg.cfg_id, T_W1, extra=1 + e))
        w2[i] = normal((cfg.H, cfg.M), cfg.sigma_w, rng_for(cfg.cfg_id, T_W2, extra=1 + e))
    return store(w1, cfg.dtype), store(w2, cfg.dtype)


def upstream_grad(cfg: MoEConfig) -> Stored:
    """dL/dy for the rank's S output rows, N(0,1)."""
    return store(normal((cfg.S, cfg.M), 1.0, rng_for(cfg.cfg_id, T_DY)), cfg.dtype)


def synthetic_logits(S: int, E: int, seed: int, sigma: float = 1.0, ties: bool = False) -> np.ndarray:
    """fp32 gate logits drawn directly (for routing tests that start from logits).
    ties=True quantises them coarsely so that equal logits are common."""
    gen = np.random.Generator(np.random.PCG64(BASE_SEED + 7_000_000 + seed))
    l = gen.standard_normal(size=(S, E), dtype=np.float32) * np.float32(sigma)
    if ties:
        l = np.round(l * 2.0) / np.float32(2.0)
    return l.astype(np.float32)


def recv_buffer(cfg: MoEConfig, C: int, rows_sigma: float = 1.0, fill: float = 0.8,
                tensor_id: int = T_RECV) -> Stored:
    """A rank-shaped expert input [n_src, G, C, M] as it lands after the EP&ESP AlltoAll:
    in every [C, M] chunk a leading run of occupied rows ~N(0, rows_sigma) and a zero tail
    (capacity padding).  C is the per-expert capacity (rows per chunk), given by the caller;
    `fill` is the mean occupied fraction."""
    gen = rng_for(cfg.cfg_id, tensor_id)
    buf = normal((cfg.n_src, cfg.G, C, cfg.M), rows_sigma, gen)
    occ = gen.integers(low=int(C * max(0.0, 2 * fill - 1.0)), high=C + 1, size=(cfg.n_src, cfg.G))
    for s in range(cfg.n_src):
        for g in range(cfg.G):
            buf[s, g, occ[s, g]:, :] = 0.0
    return store(buf, cfg.dtype)
