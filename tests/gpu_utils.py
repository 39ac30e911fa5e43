"""Test-side helpers of the GPU parity tests: the margin rule for a floating-point top-U
decision.  (The device plumbing lives in paper_2604_08971_amd.device_model.)"""
from __future__ import annotations

from typing import Optional

import numpy as np

from paper_2604_08971_amd.device_model import (ORACLE_MODE, SF_DTYPE, DeviceModel, desc_for,  # noqa: F401
                                               key_valid_host, to_dev, to_host)


def selection_report(score_oracle: np.ndarray, sel_gpu: np.ndarray, sel_oracle: np.ndarray,
                     valid: Optional[np.ndarray], eps_rel: float):
    """Margin check of one (sample, head): the GPU's active set is acceptable iff
    every chosen query scores >= tau - eps and every allowed query left out
    scores <= tau + eps, tau being the oracle's U-th largest score.
    Returns (ok, differs)."""
    L = score_oracle.shape[0]
    chosen = sel_gpu[sel_gpu >= 0]
    ref = sel_oracle[sel_oracle >= 0]
    if len(chosen) != len(ref) or len(np.unique(chosen)) != len(chosen):
        return False, True
    if len(ref) == 0:
        return True, False
    if not np.all(np.diff(chosen) > 0):
        return False, True
    allowed = np.ones(L, bool) if valid is None else valid.astype(bool)
    if not allowed[chosen].all():
        return False, True
    tau = np.min(score_oracle[ref])
    eps = eps_rel * max(1.0, abs(tau))
    mask = np.zeros(L, bool)
    mask[chosen] = True
    ok = bool(np.all(score_oracle[chosen] >= tau - eps) and
              np.all(score_oracle[allowed & ~mask] <= tau + eps))
    return ok, not np.array_equal(chosen, ref)
