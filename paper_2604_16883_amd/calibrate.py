"""Threshold calibration (host side, numpy) following Appendix A of the paper.

Per context length, the threshold that realises a target skip ratio is read off the group scores
of a calibration sample; the per-length thresholds are then fitted with a cubic in the normalised
context length, tau(x) = a x^3 + b x^2 + c x + d, whose coefficients go into
``sr_route_params.tau_coef`` (with ``len_norm`` the normaliser).  Group scores come from
``sinkrouter_probe`` on the GPU (``probe_scores``) or from any other source.

Readings: the paper does not define the normalisation; x = L / len_norm with len_norm defaulting to
the largest calibrated length.  With n scores the realised ratio is quantised to multiples of 1/n:
the threshold is placed midway between the k-th and (k+1)-th largest score, k = round(target * n),
so exactly k groups exceed it (strict comparison of Eq. 13).
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence, Tuple

import numpy as np


def threshold_for_skip_ratio(scores, target: float) -> float:
    """tau such that the fraction of scores strictly above tau is round(target*n)/n."""
    s = np.sort(np.asarray(scores, np.float64).ravel())[::-1]
    n = s.size
    if n == 0:
        raise ValueError("no scores")
    k = int(round(float(target) * n))
    k = max(0, min(n, k))
    if k == 0:
        return float(s[0])                 # nothing strictly above the maximum
    if k == n:
        return float(np.nextafter(s[-1], -np.inf))
    if s[k - 1] == s[k]:
        # a tie straddles the cut: strict '>' cannot split equal scores; cut below the run of ties
        # if that is closer to the target, else above it
        above = int(np.sum(s > s[k]))
        below = int(np.sum(s >= s[k]))
        if abs(above - target * n) <= abs(below - target * n):
            return float(s[k])
        lower = s[s < s[k]]
        return float((s[k] + lower[0]) / 2) if lower.size else float(np.nextafter(s[-1], -np.inf))
    return float((s[k - 1] + s[k]) / 2)


def skip_ratio(scores, tau: float) -> float:
    s = np.asarray(scores, np.float64).ravel()
    return float(np.mean(s > tau))


def fit_tau_cubic(lengths: Sequence[float], taus: Sequence[float], len_norm: Optional[float] = None
                  ) -> Tuple[Tuple[float, float, float, float], float]:
    """Least-squares cubic through (L/len_norm, tau).  Fewer than four distinct lengths lower the
    degree (the missing leading coefficients are 0).  Returns ((a, b, c, d), len_norm)."""
    L = np.asarray(lengths, np.float64)
    t = np.asarray(taus, np.float64)
    if L.size == 0 or L.size != t.size:
        raise ValueError("need one threshold per length")
    ln = float(len_norm) if len_norm else float(L.max())
    x = L / ln
    deg = min(3, np.unique(x).size - 1)
    coef = np.polyfit(x, t, deg) if deg > 0 else np.array([t.mean()])
    full = np.zeros(4)
    full[4 - coef.size:] = coef
    return tuple(float(c) for c in full), ln


def tau_of(coef: Sequence[float], length: float, len_norm: float) -> float:
    x = length / len_norm if len_norm > 0 else 0.0
    a, b, c, d = coef
    return ((a * x + b) * x + c) * x + d


def calibrate(scores_by_length: Dict[int, np.ndarray], target: float = 0.6, len_norm: Optional[float] = None) -> dict:
    """scores_by_length: context length -> group scores S_g of the calibration sample at that length."""
    lengths = sorted(scores_by_length)
    taus = [threshold_for_skip_ratio(scores_by_length[L], target) for L in lengths]
    coef, ln = fit_tau_cubic(lengths, taus, len_norm)
    realised = {L: skip_ratio(scores_by_length[L], tau_of(coef, L, ln)) for L in lengths}
    return {"tau_coef": coef, "len_norm": ln, "lengths": lengths, "per_length_tau": taus,
            "realised_skip_ratio": realised, "target": target}


def probe_scores(q, k_cache, seq_lens, n_kv_heads: Optional[int] = None, k0=None, k0_norm=None) -> np.ndarray:
    """Group scores S_g [B,H_kv] of device tensors through ``sinkrouter_probe`` (GPU)."""
    import torch
    from . import binding
    B, Hq, D = q.shape
    Hkv = k_cache.shape[1] if n_kv_heads is None else n_kv_heads
    Lmax = k_cache.shape[2]
    p = binding.make_route_params(B, Hq, Hkv, Lmax, head_dim=D, k0=k0, k0_norm=k0_norm)
    score = torch.empty((B, Hkv), dtype=torch.float32, device=q.device)
    mask = torch.empty((B, Hkv), dtype=torch.uint8, device=q.device)
    binding.sinkrouter_probe(q, k_cache, seq_lens, p, score, mask)
    return score.cpu().numpy().astype(np.float64)
