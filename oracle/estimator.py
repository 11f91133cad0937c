"""Exit estimation written out plainly (test infrastructure, CPU only; Sec. 5.3).

A shallow two-layer network reads the last backbone stage's features of a frame and names the
fastest exit that is still right for it, OPT_EP(x); the planner then extrapolates every exit's
true positives, false positives and false negatives on the sampled frames from OPT_EP and the
reference exit's answers (the three sums of Sec. 5.3) instead of running every exit.

Readings where the paper is silent: the features are averaged over the spatial positions before
the first layer; layer 1 is affine + ReLU, layer 2 affine; the estimate is the arg-max of the
second layer's outputs (the lowest exit on a tie), counted from 1.  All arithmetic in float64.
"""
import numpy as np

from .planner import PlannerConfig


def estimate_exit(feat, w1, b1, w2, b2):
    """feat [n, C, Hk, Wk]; w1 [hidden, C], b1 [hidden], w2 [E, hidden], b2 [E].
    Returns (OPT_EP int [n] in 1..E, logits float64 [n, E])."""
    feat = np.asarray(feat, np.float64)
    pooled = feat.mean(axis=(2, 3))
    h = np.maximum(pooled @ np.asarray(w1, np.float64).T + np.asarray(b1, np.float64), 0.0)
    logits = h @ np.asarray(w2, np.float64).T + np.asarray(b2, np.float64)
    return np.argmax(logits, axis=1) + 1, logits


def extrapolated_counts(ref_pos, opt, k):
    """TP_k, FP_k, FN_k of exit k over the sampled frames (Sec. 5.3): S = frames the reference exit
    reports positive, S^ = the others; exit k is taken to be right on x exactly when k >= OPT_EP(x)."""
    ref_pos, opt = np.asarray(ref_pos, bool), np.asarray(opt)
    tp = int(np.sum(ref_pos & (k >= opt)))
    fp = int(np.sum(~ref_pos & (k < opt)))
    fn = int(np.sum(ref_pos & (k < opt)))
    return tp, fp, fn


def pick_best_ep_estimated(ref_pos, opt, n_exits, cfg=None):
    """Estimation-based exit selection: the fastest exit whose extrapolated precision and recall meet
    the constraints; and the ratio of positive frames (reference exit)."""
    cfg = cfg or PlannerConfig()
    best = n_exits
    for k in range(1, n_exits + 1):
        tp, fp, fn = extrapolated_counts(ref_pos, opt, k)
        prec = 1.0 if tp + fp == 0 else tp / (tp + fp)
        rec = 1.0 if tp + fn == 0 else tp / (tp + fn)
        if prec >= cfg.precision and rec >= cfg.recall:
            best = k
            break
    return best, int(np.sum(np.asarray(ref_pos, bool))) / len(ref_pos)
