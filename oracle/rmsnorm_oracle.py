"""fp64 CPU oracle for the fused RMS layer norm.  TEST INFRASTRUCTURE ONLY.

The paper's second kernel (section "Method and Investigated Kernels": RMS layernorm, fused as in the
serving stack it compares with; Table I).  It states no formula of its own and cites Zhang and
Sennrich's root-mean-square layer normalisation; this file writes that definition out in numpy fp64,
with the optional residual add in front of it:

    z[t, :]   = x[t, :] + residual[t, :]          (z = x without a residual)
    y[t, i]   = z[t, i] / sqrt(mean_i z[t, i]^2 + eps) * weight[i]
    residual' = z

Inputs are the already-rounded bf16 (or fp32) values widened exactly; nothing is rounded here.
No tiling, no fusion, no shared code with the HIP path.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def rms_norm(x: np.ndarray, weight: np.ndarray, eps: float, residual: Optional[np.ndarray] = None
             ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """x, residual: [T, H]; weight: [H]; all float64.  Returns (y, residual') in float64."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(weight, dtype=np.float64)
    if x.ndim != 2 or w.shape != (x.shape[1],):
        raise ValueError("x must be [T, H] and weight [H]")
    z = x if residual is None else x + np.asarray(residual, dtype=np.float64)
    if z.shape != x.shape:
        raise ValueError("residual must have the shape of x")
    mean_sq = np.mean(z * z, axis=1, keepdims=True) if z.shape[1] else np.zeros((z.shape[0], 1))
    y = z / np.sqrt(mean_sq + float(eps)) * w[None, :]
    return y, (None if residual is None else z)
