"""Proxy-reliability analysis of the routing signal (host side, numpy).

The paper judges the cosine proxy S_g against the target regime it stands in for: a KV group is
"sink-like" when the full-attention softmax mass on token 0 exceeds gamma = 0.65 (Section 4.2,
first paragraph), and Appendix C reports, at KV-group level, the precision-recall curve of S_g
as a score for that label (AUPRC) and precision / recall / F1 as functions of the threshold.
The inputs here are what the library emits: group scores from ``sinkrouter_probe`` and per-head
alpha_0 from ``sinkrouter_decode_diag`` run with routing disabled.

Reading: the paper does not say how the group's "full-attention BOS score" is formed from its
heads; the mean of alpha_0 over the group's heads is used, mirroring the mean in Eq. 12.
"""
from __future__ import annotations

from typing import Dict, Sequence

import numpy as np

GAMMA = 0.65   # initial-token dominance threshold of Section 4.2


def group_alpha0(alpha0: np.ndarray, group_size: int) -> np.ndarray:
    """[B,Hq] per-head alpha_0 -> [B,Hkv] mean over the heads of each KV group."""
    a = np.asarray(alpha0, np.float64)
    B, Hq = a.shape
    return a.reshape(B, Hq // group_size, group_size).mean(-1)


def sink_labels(alpha0_group: np.ndarray, gamma: float = GAMMA) -> np.ndarray:
    """Target-regime label per group: alpha_0 > gamma."""
    return np.asarray(alpha0_group) > gamma


def precision_recall_curve(scores: Sequence[float], labels: Sequence[bool]):
    """Precision and recall of "score >= t" for t running over the distinct scores, highest first.
    Returns (precision, recall, thresholds); recall is non-decreasing along the arrays."""
    s = np.asarray(scores, np.float64).ravel()
    y = np.asarray(labels, bool).ravel()
    order = np.argsort(-s, kind="stable")
    s, y = s[order], y[order]
    tp = np.cumsum(y)
    fp = np.cumsum(~y)
    last = np.r_[np.flatnonzero(np.diff(s) != 0), s.size - 1]     # last index of every run of equal scores
    tp, fp = tp[last], fp[last]
    npos = int(y.sum())
    precision = tp / np.maximum(tp + fp, 1)
    recall = tp / npos if npos else np.zeros_like(tp, dtype=np.float64)
    return precision, recall, s[last]


def average_precision(scores, labels) -> float:
    """Area under the precision-recall curve as the step-wise sum  sum_n (R_n - R_{n-1}) P_n."""
    p, r, _ = precision_recall_curve(scores, labels)
    if p.size == 0:
        return float("nan")
    return float(np.sum(np.diff(np.r_[0.0, r]) * p))


def threshold_sweep(scores, labels, taus) -> Dict[str, np.ndarray]:
    """Precision, recall, F1 and skip ratio of the decision "S_g > tau" (strict, Eq. 13) per tau."""
    s = np.asarray(scores, np.float64).ravel()
    y = np.asarray(labels, bool).ravel()
    out = {k: [] for k in ("tau", "precision", "recall", "f1", "skip_ratio")}
    for t in taus:
        pred = s > t
        tp = float(np.sum(pred & y))
        pp, ap = float(pred.sum()), float(y.sum())
        prec = tp / pp if pp else 1.0
        rec = tp / ap if ap else 0.0
        out["tau"].append(float(t))
        out["precision"].append(prec)
        out["recall"].append(rec)
        out["f1"].append(2 * prec * rec / (prec + rec) if prec + rec else 0.0)
        out["skip_ratio"].append(pp / s.size if s.size else 0.0)
    return {k: np.asarray(v) for k, v in out.items()}


def skipped_vs_active_alpha0(alpha0: np.ndarray, mask: np.ndarray, group_size: int) -> Dict[str, float]:
    """Mean alpha_0 of the heads of skipped and of active groups (the distribution-level check of
    Appendix C): alpha0 [B,Hq] from a dense run, mask [B,Hkv] from the routed decision."""
    a = np.asarray(alpha0, np.float64)
    m = np.repeat(np.asarray(mask).astype(bool), group_size, axis=1)
    return {"skipped_mean": float(a[m].mean()) if m.any() else float("nan"),
            "active_mean": float(a[~m].mean()) if (~m).any() else float("nan"),
            "skipped_frac_above_gamma": float((a[m] > GAMMA).mean()) if m.any() else float("nan"),
            "active_frac_above_gamma": float((a[~m] > GAMMA).mean()) if (~m).any() else float("nan")}


def concentration_table(alpha0, max_rest, mean_rest, regimes: Sequence[float] = (0.4, 0.6, 0.8),
                        half_width: float = 0.05) -> Dict[float, Dict[str, float]]:
    """Attention-concentration statistics by sink regime, the layout of Table 1 (Section 3).

    Inputs are the per-head outputs of ``sinkrouter_concentration`` (any shape, flattened).  For
    each regime value a, the heads with |alpha_0 - a| <= half_width are averaged: ``bos`` (mean
    alpha_0), ``max`` (mean largest non-initial weight), ``mean`` (mean non-initial weight), and
    ``ratio`` = bos / max as the table defines it; ``heads`` counts them (NaN rows when none).
    Reading: the table does not say how wide its "alpha_0 is about a" bins are; half_width is
    that free choice.
    """
    a = np.asarray(alpha0, np.float64).ravel()
    mx = np.asarray(max_rest, np.float64).ravel()
    mn = np.asarray(mean_rest, np.float64).ravel()
    ok = np.isfinite(a) & np.isfinite(mx) & np.isfinite(mn)
    table = {}
    for r in regimes:
        sel = ok & (np.abs(a - r) <= half_width)
        n = int(sel.sum())
        if n == 0:
            table[float(r)] = {"heads": 0, "bos": float("nan"), "max": float("nan"), "mean": float("nan"),
                               "ratio": float("nan")}
            continue
        bos, big = float(a[sel].mean()), float(mx[sel].mean())
        table[float(r)] = {"heads": n, "bos": bos, "max": big, "mean": float(mn[sel].mean()),
                           "ratio": bos / big if big > 0 else float("inf")}
    return table
