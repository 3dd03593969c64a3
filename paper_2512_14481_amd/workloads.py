"""Seeded synthetic inputs for the SASQ hot path (LLaMA-2-shaped linear layers).

This module only *draws numbers*: Gaussian / Student-t activations with a few
outlier channels, Gaussian upstream gradients, Gaussian fp32 weights.  It holds
none of the method's arithmetic (no quantizer, no scale rule, no matmul), so it
may serve both the HIP library's callers and the CPU oracle's tests.

The synthetic tensors stand in for the activations of LLaMA-2 linear layers on
WikiText / Pile text at sequence length 2048 (Sec. 5.1 "Models and Datasets",
"Implementation"); the outlier-channel structure follows the paper's remarks on
activation outliers (Sec. 3 "Outlier", Fig. 3).

Every tensor is a pure function of (seed, config name, tensor name): a Philox
counter-based generator keyed by the seed and a CRC of the names.
Storage dtypes are returned as uint16 bit patterns (numpy has no bfloat16).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

F16 = "f16"
BF16 = "bf16"
W_INT8 = "int8"
W_INT4 = "int4"


def _rng(seed: int, *names: str) -> np.random.Generator:
    tid = zlib.crc32("/".join(names).encode())
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tid)]))


def f32_to_storage_bits(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 to the 16-bit storage dtype (nearest-even); uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == F16:
        with np.errstate(over="ignore"):
            h = a.astype(np.float16)
        # saturate to the finite range so that heavy tails never produce inf
        big = np.float16(65504.0)
        h = np.where(np.isinf(h), np.where(a > 0, big, -big), h).astype(np.float16)
        return h.view(np.uint16)
    if dtype == BF16:
        u = a.view(np.uint32)
        u = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
        return u.astype(np.uint16)
    raise ValueError(dtype)


def storage_bits_to_f32(bits: np.ndarray, dtype: str) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float32)
    if dtype == BF16:
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise ValueError(dtype)


@dataclass(frozen=True)
class ActSpec:
    """One activation tensor X[M, K]."""
    name: str
    K: int
    dist: str = "normal"            # "normal" | "student_t3"
    outlier_frac: float = 0.0       # fraction of the K channels that are outliers
    outlier_gain: float = 1.0       # whole column multiplied by this


@dataclass(frozen=True)
class ProjSpec:
    """One linear projection Y[M, N] = X[M, K] . W[N, K]^T with its own scale s."""
    name: str
    x: str                          # name of the ActSpec it consumes
    N: int


@dataclass(frozen=True)
class Config:
    name: str
    dtype: str                      # activation / output storage dtype
    M: int
    acts: Tuple[ActSpec, ...]
    projs: Tuple[ProjSpec, ...]
    w_std: float = 0.02
    w_fmt: str = W_INT8
    seed: int = 0

    def act(self, name: str) -> ActSpec:
        for a in self.acts:
            if a.name == name:
                return a
        raise KeyError(name)

    def K_of(self, proj: ProjSpec) -> int:
        return self.act(proj.x).K


def _llama_layer(hidden: int, kv: int, inter: int, frac: float, gain: float,
                 dist: str = "normal") -> Tuple[Tuple[ActSpec, ...], Tuple[ProjSpec, ...]]:
    acts = (ActSpec("x_qkv", hidden, dist, frac, gain), ActSpec("x_o", hidden, dist, frac, gain),
            ActSpec("x_mlp", hidden, dist, frac, gain), ActSpec("x_down", inter, dist, frac, gain))
    projs = (ProjSpec("q", "x_qkv", hidden), ProjSpec("k", "x_qkv", kv), ProjSpec("v", "x_qkv", kv),
             ProjSpec("o", "x_o", hidden), ProjSpec("gate", "x_mlp", inter),
             ProjSpec("up", "x_mlp", inter), ProjSpec("down", "x_down", hidden))
    return acts, projs


def _make_configs() -> Dict[str, Config]:
    c: Dict[str, Config] = {}
    c["c1_single"] = Config(
        "c1_single", F16, 64,
        (ActSpec("x", 256, "normal", 0.02, 30.0),), (ProjSpec("lin", "x", 256),))
    c["c2_attn7b"] = Config(
        "c2_attn7b", F16, 2048,
        (ActSpec("x_qkv", 4096, "normal", 0.01, 50.0), ActSpec("x_o", 4096, "normal", 0.01, 50.0)),
        (ProjSpec("q", "x_qkv", 4096), ProjSpec("k", "x_qkv", 4096), ProjSpec("v", "x_qkv", 4096),
         ProjSpec("o", "x_o", 4096)))
    c["c3_mlp7b"] = Config(
        "c3_mlp7b", F16, 4096,
        (ActSpec("x_mlp", 4096, "student_t3"), ActSpec("x_down", 11008, "student_t3")),
        (ProjSpec("gate", "x_mlp", 11008), ProjSpec("up", "x_mlp", 11008),
         ProjSpec("down", "x_down", 4096)))
    a, p = _llama_layer(5120, 5120, 13824, 0.01, 50.0)
    c["c4_w4a8_13b"] = Config("c4_w4a8_13b", BF16, 4096, a, p, 0.02, W_INT4)
    a, p = _llama_layer(8192, 1024, 28672, 0.005, 100.0)
    c["c5_layer70b"] = Config("c5_layer70b", BF16, 8192, a, p, 0.015, W_INT8)
    return c


CONFIGS: Dict[str, Config] = _make_configs()


def outlier_columns(cfg: Config, act: ActSpec) -> np.ndarray:
    n = int(round(act.outlier_frac * act.K))
    if n == 0:
        return np.zeros(0, dtype=np.int64)
    cols = _rng(cfg.seed, cfg.name, act.name, "outlier_cols").permutation(act.K)[:n]
    return np.sort(cols.astype(np.int64))


def _draw(rng: np.random.Generator, rows: int, cols: int, dist: str) -> np.ndarray:
    if dist == "normal":
        return rng.standard_normal((rows, cols), dtype=np.float32)
    if dist == "student_t3":
        # t_3 = Z / sqrt(chi2_3 / 3), chi2_3 as the sum of three squared normals
        out = np.empty((rows, cols), dtype=np.float32)
        step = max(1, (1 << 22) // max(cols, 1))
        for r0 in range(0, rows, step):
            r1 = min(rows, r0 + step)
            z = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
            g = rng.standard_normal((3, r1 - r0, cols), dtype=np.float32)
            chi = (g * g).sum(axis=0)
            out[r0:r1] = z / np.sqrt(chi / np.float32(3.0))
        return out
    raise ValueError(dist)


def activation(cfg: Config, act_name: str, rows: int | None = None) -> np.ndarray:
    """X[M, K] as uint16 bit patterns of cfg.dtype (row = token, column = channel)."""
    act = cfg.act(act_name)
    M = cfg.M if rows is None else rows
    x = _draw(_rng(cfg.seed, cfg.name, act.name, "x"), M, act.K, act.dist)
    cols = outlier_columns(cfg, act)
    if cols.size:
        x[:, cols] *= np.float32(act.outlier_gain)
    return f32_to_storage_bits(x, cfg.dtype)


def upstream_grad(cfg: Config, proj_name: str, rows: int | None = None) -> np.ndarray:
    """dy[M, K]: synthetic gradient w.r.t. the fake-quantized activation, N(0,1), cfg.dtype bits."""
    proj = next(p for p in cfg.projs if p.name == proj_name)
    M = cfg.M if rows is None else rows
    g = _rng(cfg.seed, cfg.name, proj.name, "dy").standard_normal((M, cfg.K_of(proj)), dtype=np.float32)
    return f32_to_storage_bits(g, cfg.dtype)


def weight_fp32(cfg: Config, proj_name: str) -> np.ndarray:
    """Frozen full-precision weight W[N, K] (K contiguous), N(0, w_std), fp32."""
    proj = next(p for p in cfg.projs if p.name == proj_name)
    w = _rng(cfg.seed, cfg.name, proj.name, "w").standard_normal((proj.N, cfg.K_of(proj)), dtype=np.float32)
    w *= np.float32(cfg.w_std)
    return w


def random_bits(seed: int, name: str, shape, dtype: str, dist: str = "normal",
                gain: float = 1.0) -> np.ndarray:
    """Free-form seeded tensor for small parity cases (ragged shapes etc.)."""
    rows, cols = shape
    x = _draw(_rng(seed, "free", name), rows, cols, dist) * np.float32(gain)
    return f32_to_storage_bits(x, dtype)


def random_f32(seed: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    return (_rng(seed, "free", name).standard_normal(shape, dtype=np.float32) * np.float32(std))


def random_codes(seed: int, name: str, shape, lo: int, hi: int) -> np.ndarray:
    """Uniform integer codes in [lo, hi] as int8 (synthetic already-quantized weights)."""
    return _rng(seed, "free", name).integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int8)


def all_finite_patterns(dtype: str) -> np.ndarray:
    """Every finite 16-bit pattern of the dtype plus the two infinities (no NaN)."""
    bits = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    if dtype == F16:
        exp, man = (bits >> 10) & 0x1F, bits & 0x3FF
        keep = ~((exp == 0x1F) & (man != 0))
    elif dtype == BF16:
        exp, man = (bits >> 7) & 0xFF, bits & 0x7F
        keep = ~((exp == 0xFF) & (man != 0))
    else:
        raise ValueError(dtype)
    return bits[keep]
