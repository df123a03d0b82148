"""Helpers shared by the parity tests: dtype plumbing and error metrics (no method arithmetic)."""
from __future__ import annotations

import numpy as np

from paper_2503_12964_amd import workloads as W

# Tolerances of the target statement: forward out max-abs <= 1e-2 and relative RMS <= 5e-3;
# dq, dk, dv relative RMS <= 1.5e-2.  lse is accumulated in fp32 from exact bf16 inputs, so 1e-3
# absolute is ample; a RoPE output is the fp64 value rounded once to bf16 (half an ulp, 2^-9
# relative at most), hence a relative RMS of at most 2.5e-3.
TOL_OUT_MAXABS = 1e-2
TOL_OUT_RELRMS = 5e-3
TOL_GRAD_RELRMS = 1.5e-2
TOL_LSE_MAXABS = 1e-3
TOL_ROPE_RELRMS = 2.5e-3


def bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return W.bf16_bits_to_f32(bits).astype(np.float64)


def to_device(bits: np.ndarray):
    import torch
    return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).cuda()


def to_f64(t) -> np.ndarray:
    """Device tensor (bf16 or fp32) -> numpy float64 on the host."""
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def to_bits(t) -> np.ndarray:
    import torch
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def max_abs(a, b) -> float:
    return float(np.max(np.abs(np.asarray(a) - np.asarray(b)))) if np.size(a) else 0.0


def rel_rms(a, ref) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    d = np.asarray(a, dtype=np.float64) - ref
    den = float(np.sqrt(np.sum(ref * ref)))
    return float(np.sqrt(np.sum(d * d))) / den if den > 0 else float(np.sqrt(np.sum(d * d)))
