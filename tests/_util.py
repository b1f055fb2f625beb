"""Shared helpers of the GPU parity tests (no method arithmetic here: the oracle does that)."""
from __future__ import annotations

import math

import numpy as np
import torch

from oracle import freqkv_oracle as orc

# Tolerances (max-abs error relative to the RMS of the oracle's retained block of that head-tensor).
# bf16 cache: fp16 operands (basis and folded span rounded to 11 significant bits), fp32
# accumulation: expected ~5e-3, required 2e-2.  fp32 cache: fp32 FMA chain over n terms: required 1e-5.
TOL_BF16 = 2e-2
TOL_F32 = 1e-5


def f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a bf16/fp32 tensor to float64 numpy."""
    return t.detach().to(torch.float32).cpu().double().numpy()


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float64 -> bfloat16 value (as float64), via torch's fp32->bf16 cast."""
    return torch.from_numpy(np.asarray(a, dtype=np.float64)).to(torch.float32).to(torch.bfloat16).double().numpy()


def bf16_ulp(a: np.ndarray) -> np.ndarray:
    """Spacing of bfloat16 numbers at |a| (8 significant bits)."""
    a = np.abs(np.asarray(a, dtype=np.float64))
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -126)))
    return 2.0 ** (e - 7)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    rms = math.sqrt(float((ref ** 2).mean()))
    return float(np.max(np.abs(got - ref))) / max(rms, 1e-300)


def oracle_span_columns(head_rows: np.ndarray, n_sink: int, window: int, lc: int, cols) -> np.ndarray:
    """Oracle result for selected channels of one head-tensor: [lc, len(cols)]."""
    x = np.ascontiguousarray(head_rows[n_sink:window][:, cols])
    return orc.compress_span(x, lc)
