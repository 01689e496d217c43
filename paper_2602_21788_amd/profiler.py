"""The scheduler's Profiler (paper Sec. 5, implementation details): time the attention path of this library for
several (sequence length, CP degree) points and fit the coefficients of the compute model that fcp_plan_groups
uses (Eq. 8 with the compute terms divided by the degree):

    t(len, d) = alpha1 * len^2 / d + alpha2 * len / d + beta1

`fit_compute_coefficients` is plain linear least squares; `profile_attention` produces the samples on the GPU
(one rank's share of one sequence: forward steps + merge + backward, inputs resident).  The exchange
coefficients (Eq. 9) need more than one GPU and stay with the caller.
"""
from __future__ import annotations

import numpy as np


def fit_compute_coefficients(seq_lens, degrees, times):
    """Least-squares (alpha1, alpha2, beta1) and the largest relative error of the fit over the samples."""
    s = np.asarray(seq_lens, np.float64)
    d = np.asarray(degrees, np.float64)
    t = np.asarray(times, np.float64)
    if not (s.shape == d.shape == t.shape and s.ndim == 1 and len(s) >= 3):
        raise ValueError("need at least three (length, degree, time) samples")
    a = np.stack([s * s / d, s / d, np.ones_like(s)], axis=1)
    coef, *_ = np.linalg.lstsq(a, t, rcond=None)
    err = float(np.max(np.abs(a @ coef - t) / t))
    return (float(coef[0]), float(coef[1]), float(coef[2])), err


def profile_attention(seq_lens, degrees, hq=32, hkv=8, head_dim=128, repeats=5):
    """Seconds per forward + backward of rank 0's share of one sequence, for every (length, degree) pair given."""
    import torch
    from .rank import RankAttention

    out = []
    for length, deg in zip(seq_lens, degrees):
        ra = RankAttention([int(length)], [int(deg)], 0, hq, hkv, head_dim)
        ra.set_random_inputs(1)

        def step():
            ra.forward()
            ra.zero_grads()
            ra.backward()

        for _ in range(2):
            step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(repeats):
            step()
        e1.record()
        torch.cuda.synchronize()
        out.append(e0.elapsed_time(e1) * 1e-3 / repeats)
    return out
