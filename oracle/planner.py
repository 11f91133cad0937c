"""Fine-grained query planning written out plainly (test infrastructure, CPU only).

Follows the planning section of the paper (Sec. 5.2, Algorithm 1) step by step and in its
notation: EstimateSamplingRate, GetQueryPlan (recursive), PickBestEP, the sampling-rate bound,
memoisation of inference results, and evaluation-based exit selection.  The query predicate is
the one of Table 2, Count(class) >= t per frame.  Nothing here is shared with the library's
planner; only tests (and the benchmark's CPU leg) may import it.

Where the paper leaves a quantity open this file takes one reading and names it:
  * the logarithm of the rate bound is base 2 (the rate doubles per level);
  * a chunk is divided into two halves (rate doubling + the stated maximum depth imply halving);
  * "Length is small" = the chunk cannot be halved without a half under `min_chunk` frames;
  * "sufficient" / "insufficient" positive ratio = at least `posi_enough` / at most `posi_skip`;
  * a memoised frame is "nearby" when it lies in the same chunk within `reuse_dist` frames;
  * precision (recall) of an exit that reports (is asked for) no positive frame is 1.
"""
from dataclasses import dataclass
from fractions import Fraction
import math

import numpy as np


@dataclass
class PlannerConfig:
    precision: float = 0.8     # P, Sec. 5.2 (evaluation-based exit selection)
    recall: float = 0.8        # R
    min_chunk: int = 100       # chunks hold at least this many frames (sampling-rate bound)
    final_span: int = 10       # 1 / (bound on the final sampling rate); 0.1 -> 10
    posi_enough: float = 0.1   # positive ratio from which the chunk's statistics are trusted
    posi_skip: float = 0.0     # positive ratio up to which the chunk is skipped
    reuse_dist: int = 0        # memoised frames this close (same chunk) stand in for a sample


def count_predicate(labels, scores, label, min_count, min_score=0.0):
    """Table 2: Count(class) >= t.  labels/scores [..., D] (label -1 = empty slot) -> bool [...]."""
    labels, scores = np.asarray(labels), np.asarray(scores)
    hit = (labels == label) & (scores >= np.float32(min_score))
    return hit.sum(axis=-1) >= min_count


def max_depth(n, min_chunk):
    """Maximum recursion depth, ceil(log2(|V| / min_chunk)) (text after the rate bound)."""
    if n <= min_chunk:
        return 0
    return int(math.ceil(math.log2(n / min_chunk)))


def estimate_sampling_rate(n, cfg):
    """EstimateSamplingRate: the largest initial rate with rate * 2^depth <= 1/final_span."""
    return Fraction(1, cfg.final_span * 2 ** max_depth(n, cfg.min_chunk))


def precision_recall(pred, ref):
    """Frame-level precision and recall of one exit's answers against the reference exit's."""
    pred, ref = np.asarray(pred, bool), np.asarray(ref, bool)
    tp = int(np.sum(pred & ref))
    fp = int(np.sum(pred & ~ref))
    fn = int(np.sum(~pred & ref))
    prec = 1.0 if tp + fp == 0 else tp / (tp + fp)
    rec = 1.0 if tp + fn == 0 else tp / (tp + fn)
    return prec, rec


def answer_metrics(pred, ref):
    """Sec. 6.1: frame answers of a system against the reference exit's: (TP, FP, FN, precision, recall, F-1);
    F-1 = harmonic mean of precision and recall, 0 when both are 0."""
    pred, ref = np.asarray(pred, bool), np.asarray(ref, bool)
    tp, fp, fn = int(np.sum(pred & ref)), int(np.sum(pred & ~ref)), int(np.sum(~pred & ref))
    prec, rec = precision_recall(pred, ref)
    f1 = 0.0 if prec + rec == 0 else 2 * prec * rec / (prec + rec)
    return tp, fp, fn, prec, rec, f1


def pick_best_ep(flags_sub, cfg):
    """PickBestEP: flags_sub bool [k, E] (frame answers per exit; the last exit is the
    reference).  Returns (fastest exit meeting P and R, 1-based; ratio of positive frames
    according to the reference exit)."""
    flags_sub = np.asarray(flags_sub, bool)
    k, E = flags_sub.shape
    ref = flags_sub[:, E - 1]
    best = E
    for e in range(E):
        prec, rec = precision_recall(flags_sub[:, e], ref)
        if prec >= cfg.precision and rec >= cfg.recall:
            best = e + 1
            break
    return best, int(ref.sum()) / k


class Planner:
    """evaluate(f) -> bool [E]: every exit's answer to the query on frame f (the expensive step).
    memo=False re-evaluates every sample (the paper's "no reuse" picture).
    select(rows) -> (best_ep, posi_ratio) replaces PickBestEP on the stacked results of the samples (used by
    estimation-based selection, Sec. 5.3, where evaluate returns (reference answer, OPT_EP) instead)."""

    def __init__(self, evaluate, n, cfg=None, memo=True, select=None):
        self.evaluate, self.n, self.cfg, self.use_memo = evaluate, int(n), cfg or PlannerConfig(), memo
        self.select = select or (lambda rows: pick_best_ep(rows, self.cfg))
        self.memo = {}
        self.evaluated = []      # frames passed to evaluate(), in order
        self.reused = 0
        self.depth = 0
        self.trace = []          # (a, b, span, best_ep, posi_ratio) per GetQueryPlan call, in call order

    def _result(self, f, a, b, known):
        """Answers for sample f of chunk [a, b): memoised, borrowed from a nearby memoised frame
        of the same chunk, or newly evaluated.  `known` = frames memoised when the chunk was entered."""
        if self.use_memo:
            if f in known:
                self.reused += 1
                return self.memo[f]
            near = [g for g in known if a <= g < b and abs(g - f) <= self.cfg.reuse_dist]
            if near:
                g = min(near, key=lambda g: (abs(g - f), g))
                self.reused += 1
                return self.memo[g]
        r = np.asarray(self.evaluate(f))
        self.evaluated.append(f)
        self.memo[f] = r
        return r

    def get_query_plan(self, a, b, rate, depth=0):
        """GetQueryPlan on V = frames [a, b) at sampling rate `rate` (a Fraction)."""
        cfg = self.cfg
        self.depth = max(self.depth, depth)
        span = int(1 / rate)                                   # sampling_span
        known = set(self.memo)
        sub = [self._result(f, a, b, known) for f in range(a, b, span)]   # V_sub = V[0, span, 2 span, ...]
        best_ep, posi_ratio = self.select(np.stack(sub))
        self.trace.append((a, b, span, best_ep, posi_ratio))
        small = (b - a) < 2 * cfg.min_chunk
        if (posi_ratio >= cfg.posi_enough and best_ep == 1) or small:
            return [(a, b - a, best_ep)]
        if posi_ratio <= cfg.posi_skip:
            return [(a, b - a, 0)]                             # skip
        mid = a + (b - a) // 2
        return self.get_query_plan(a, mid, 2 * rate, depth + 1) + self.get_query_plan(mid, b, 2 * rate, depth + 1)

    def plan(self):
        if self.n == 0:
            return []
        return self.get_query_plan(0, self.n, estimate_sampling_rate(self.n, self.cfg))


def plan_from_flags(flags, cfg=None, memo=True):
    """Planner run on a table of answers, flags bool [n, E] (only the sampled rows are looked at).
    Returns (plan, planner); plan = [(start, length, exit or 0 = skip), ...] in frame order."""
    flags = np.asarray(flags, bool)
    p = Planner(lambda f: flags[f], flags.shape[0], cfg, memo)
    return p.plan(), p


def accuracy_against_reference(flags, plan):
    """Frame-level precision, recall and F-1 of a plan's answers against the reference (last) exit
    on every frame (Sec. 6.1 metrics).  flags bool [n, E]."""
    flags = np.asarray(flags, bool)
    ans = np.zeros(flags.shape[0], bool)
    for a, ln, ep in plan:
        if ep > 0:
            ans[a:a + ln] = flags[a:a + ln, ep - 1]
    prec, rec = precision_recall(ans, flags[:, -1])
    f1 = 0.0 if prec + rec == 0 else 2 * prec * rec / (prec + rec)
    return prec, rec, f1


def plan_from_estimates(ref_pos, opt, n_exits, cfg=None, memo=True):
    """Planner with estimation-based exit selection (Sec. 5.3) on tables: ref_pos bool [n] (reference
    exit's answer), opt int [n] (OPT_EP per frame).  Only sampled rows are looked at."""
    from .estimator import pick_best_ep_estimated
    cfg = cfg or PlannerConfig()
    ref_pos, opt = np.asarray(ref_pos, bool), np.asarray(opt)
    p = Planner(lambda f: (int(ref_pos[f]), int(opt[f])), len(ref_pos), cfg, memo,
                select=lambda rows: pick_best_ep_estimated(rows[:, 0].astype(bool), rows[:, 1], n_exits, cfg))
    return p.plan(), p
