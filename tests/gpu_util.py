"""Helpers for the GPU parity tests: numpy bit patterns <-> device tensors, comparisons."""
from __future__ import annotations

import numpy as np
import torch

from paper_2512_14481_amd import workloads as wl

TDT = {"f16": torch.float16, "bf16": torch.bfloat16}


def to_dev(bits: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.cuda().view(TDT[dtype])


def to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def val(bits: np.ndarray, dtype: str) -> np.ndarray:
    return wl.storage_bits_to_f32(bits, dtype).astype(np.float64)


def dev_scalar(v) -> torch.Tensor:
    return torch.tensor([float(np.float32(v))], dtype=torch.float32, device="cuda")


def assert_same_values(got_bits: np.ndarray, ref_bits: np.ndarray, dtype: str, what: str, rel: float = 0.0):
    """Equal by value (-0 == +0).  With rel > 0: max relative error bound instead of equality."""
    if np.array_equal(got_bits, ref_bits):
        return
    g, r = val(got_bits, dtype), val(ref_bits, dtype)
    if rel == 0.0:
        bad = ~((g == r) | (np.isnan(g) & np.isnan(r)))
    else:
        with np.errstate(invalid="ignore"):
            bad = ~(np.abs(g - r) <= rel * np.maximum(np.abs(r), 1e-30))
        bad &= ~((g == r))
    if bad.any():
        i = np.flatnonzero(bad)[:5]
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} differ; first at flat {i}: "
                             f"got {g.ravel()[i]} ref {r.ravel()[i]}")


def rel_err(a: float, b: float) -> float:
    return abs(a - b) / max(abs(b), 1e-30)


_PATH = {None: 0, "twopass": 1, "fused": 2}
_TILE = {None: 0, "256": 1, "128x256": 2, "128": 3}
_MFMA = {None: 0, "32x32x32": 1, "16x16x64": 2}
_BWD_TILE = {None: 0, "256": 1, "128": 2}


def set_tuning(path=None, tile=None, mfma=None, share=None, bwd_tile=None):
    """Force kernel variants through sasq_set_tuning; called without arguments it restores the
    library's own choices.  path: "twopass" | "fused"; tile: "256" | "128x256" | "128";
    mfma: "32x32x32" | "16x16x64"; share: 1..3; bwd_tile: "256" | "128"."""
    from paper_2512_14481_amd import binding as B
    B.sasq_set_tuning(B.SASQ_TUNE_LINEAR_PATH, _PATH[path])
    B.sasq_set_tuning(B.SASQ_TUNE_LINEAR_TILE, _TILE[tile])
    B.sasq_set_tuning(B.SASQ_TUNE_LINEAR_MFMA, _MFMA[mfma])
    B.sasq_set_tuning(B.SASQ_TUNE_FQ_SHARE, share or 0)
    B.sasq_set_tuning(B.SASQ_TUNE_BWD_TILE, _BWD_TILE[bwd_tile])
