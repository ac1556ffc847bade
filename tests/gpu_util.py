"""Helpers of the GPU tests: the layer object of the package plus error metrics."""
from __future__ import annotations

import numpy as np

import workloads as wl
from paper_2503_09304_amd.layer import DEV, DevWeights, DevWeightsMX, GpuLayer, to_dev, to_host  # noqa: F401


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |err| / RMS(reference)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.max(np.abs(got - ref)) / rms) if ref.size else 0.0


def bf16_y_tol(y_ref: np.ndarray, before_rounding: float = 1.2e-2, bar: float = 2e-2) -> float:
    """Bar for a bf16 y outside the named configurations (4-bit weights, small random shapes), where
    the final rounding alone can take most of 2e-2: the error before the final rounding (budget
    1.2e-2 of RMS: activation rounding to bf16, fp32 accumulation) plus the most that rounding can
    add, half an ulp in the binade of the largest |y| (2^-8 of that power of two); never below the
    2e-2 of the named configurations."""
    y = np.abs(np.asarray(y_ref, dtype=np.float64))
    rms = float(np.sqrt(np.mean(y * y))) if y.size else 0.0
    if rms == 0.0:
        return bar
    half_ulp = 2.0 ** (np.floor(np.log2(y.max())) - 8)
    return max(bar, before_rounding + half_ulp / rms)


def as_f64(a: np.ndarray) -> np.ndarray:
    return wl.as_f64(a)
