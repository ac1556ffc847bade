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


def as_f64(a: np.ndarray) -> np.ndarray:
    return wl.as_f64(a)
