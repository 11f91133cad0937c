"""Pins for the planning oracle (Sec. 5.2, Algorithm 1): the rate bound's closed form, precision /
recall against a library routine, hand-worked plans, recursion invariants, memoisation.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest
from sklearn.metrics import confusion_matrix, f1_score, precision_score, recall_score

from oracle import planner as P


def _depth_by_doubling(n, mc):
    d = 0
    while mc * 2 ** d < n:
        d += 1
    return d


@pytest.mark.parametrize("mc,span", [(100, 10), (12, 2), (7, 3)])
def test_initial_rate_is_the_largest_one_within_the_bound(mc, span):
    """rate * 2^ceil(log2(|V|/min_chunk)) <= final rate, and doubling the rate breaks it (Sec. 5.2,
    sampling-rate bound).  The depth is re-derived by repeated doubling, without a logarithm."""
    cfg = P.PlannerConfig(min_chunk=mc, final_span=span)
    for n in list(range(1, 700)) + [mc * 2 ** k + o for k in range(1, 12) for o in (-1, 0, 1)]:
        d = _depth_by_doubling(n, mc)
        assert P.max_depth(n, mc) == d, n
        r = P.estimate_sampling_rate(n, cfg)
        assert r * 2 ** d <= Fraction(1, span) < 2 * r * 2 ** d


def test_paper_constants_give_rate_one_in_ten_at_the_last_level():
    """Sec. 5.2: chunks of at least 100 frames, final rate bounded by 0.1."""
    cfg = P.PlannerConfig()
    assert P.estimate_sampling_rate(100, cfg) == Fraction(1, 10)
    assert P.estimate_sampling_rate(101, cfg) == Fraction(1, 20)
    assert P.estimate_sampling_rate(800, cfg) == Fraction(1, 80)
    assert P.estimate_sampling_rate(801, cfg) == Fraction(1, 160)


def test_precision_recall_match_the_library_routine():
    rng = np.random.default_rng(5)
    for _ in range(200):
        k = int(rng.integers(1, 40))
        pred, ref = rng.random(k) < rng.random(), rng.random(k) < rng.random()
        pr, rc = P.precision_recall(pred, ref)
        assert pr == pytest.approx(precision_score(ref, pred, zero_division=1.0))
        assert rc == pytest.approx(recall_score(ref, pred, zero_division=1.0))


def test_answer_metrics_match_the_library_routines():
    rng = np.random.default_rng(8)
    for _ in range(200):
        k = int(rng.integers(1, 60))
        pred, ref = rng.random(k) < rng.random(), rng.random(k) < rng.random()
        tp, fp, fn, pr, rc, f1 = P.answer_metrics(pred, ref)
        tn_, fp_, fn_, tp_ = confusion_matrix(ref, pred, labels=[False, True]).ravel()
        assert (tp, fp, fn) == (tp_, fp_, fn_)
        if tp + fp > 0 and tp + fn > 0:                     # where nothing is empty the conventions do not matter
            assert f1 == pytest.approx(f1_score(ref, pred, zero_division=0.0))
    assert P.answer_metrics([0, 0], [0, 0])[3:] == (1.0, 1.0, 1.0)
    assert P.answer_metrics([1, 0], [0, 1])[3:] == (0.0, 0.0, 0.0)


def test_pick_best_ep_is_the_fastest_exit_meeting_both_constraints():
    rng = np.random.default_rng(6)
    cfg = P.PlannerConfig(precision=0.8, recall=0.8)
    seen = set()
    for _ in range(300):
        k, E = int(rng.integers(2, 30)), int(rng.integers(1, 6))
        ref = rng.random(k) < 0.5
        flags = np.stack([np.where(rng.random(k) < q, ref, ~ref) for q in np.sort(rng.random(E))] , axis=1)
        flags[:, -1] = ref
        best, ratio = P.pick_best_ep(flags, cfg)
        ok = [precision_score(ref, flags[:, e], zero_division=1.0) >= 0.8 and recall_score(ref, flags[:, e], zero_division=1.0) >= 0.8
              for e in range(E)]
        assert ok[-1]                                   # the reference exit always qualifies
        assert best == ok.index(True) + 1
        assert ratio == pytest.approx(ref.mean())
        seen.add(best)
    assert len(seen) >= 3


def test_count_predicate():
    labels = np.array([[1, 1, 2, -1], [1, 2, 2, 2], [-1, -1, -1, -1]])
    scores = np.array([[.9, .4, .8, 0], [.9, .9, .3, .6], [0, 0, 0, 0]], np.float32)
    assert P.count_predicate(labels, scores, 1, 2).tolist() == [True, False, False]
    assert P.count_predicate(labels, scores, 1, 2, 0.5).tolist() == [False, False, False]
    assert P.count_predicate(labels, scores, 2, 2, 0.5).tolist() == [False, True, False]
    assert P.count_predicate(labels, scores, 2, 0).tolist() == [True, True, True]


def _video(n, easy, positive):
    """Two exits; the reference (exit 2) answers `positive`; exit 1 equals it on `easy` frames and says no elsewhere."""
    f = np.zeros((n, 2), bool)
    f[:, 1] = positive
    f[:, 0] = positive & easy
    return f


def test_worked_example_easy_half_hard_half():
    """400 frames, positives everywhere, exit 1 right on frames 0..199 only.  By hand: depth 2, span 40.
    Top level: 10 samples, exit 1 finds 5 of 10 -> recall 0.5 -> best exit 2, not small -> halve.
    [0,200) at span 20: exit 1 perfect, positives -> one chunk at exit 1.  [200,400) at span 20: exit 1
    finds nothing -> exit 2, 200 frames can still be halved -> [200,300), [300,400) at span 10: small.
    New evaluations: 10 + 5 + 5 + 5 + 5 (every other sample is memoised)."""
    idx = np.arange(400)
    flags = _video(400, idx < 200, np.ones(400, bool))
    plan, pl = P.plan_from_flags(flags)
    assert plan == [(0, 200, 1), (200, 100, 2), (300, 100, 2)]
    assert [t[:3] for t in pl.trace] == [(0, 400, 40), (0, 200, 20), (200, 400, 20), (200, 300, 10), (300, 400, 10)]
    assert len(pl.evaluated) == 30 and pl.reused == 20 and pl.depth == 2
    assert sorted(pl.evaluated) == sorted(set(range(0, 200, 20)) | set(range(200, 400, 10)))
    assert P.accuracy_against_reference(flags, plan) == (1.0, 1.0, 1.0)


def test_worked_example_skip_of_an_empty_half():
    """First half holds no positive frame, second half is hard: the top level cannot settle (exit 1 misses
    every positive), the empty half is skipped, the hard half ends at the reference exit."""
    idx = np.arange(400)
    flags = _video(400, np.zeros(400, bool), idx >= 200)
    plan, pl = P.plan_from_flags(flags)
    assert plan == [(0, 200, 0), (200, 100, 2), (300, 100, 2)]
    assert P.accuracy_against_reference(flags, plan) == (1.0, 1.0, 1.0)


def test_special_cases():
    ones = np.ones(1000, bool)
    # every exit agrees and positives are frequent: the whole video runs at the fastest exit after one level
    plan, pl = P.plan_from_flags(_video(1000, ones, ones))
    assert plan == [(0, 1000, 1)] and len(pl.evaluated) == len(range(0, 1000, 160))
    # a video that cannot be halved is one chunk whatever the samples say
    plan, _ = P.plan_from_flags(_video(199, ~ones[:199], ones[:199]))
    assert plan == [(0, 199, 2)]
    # no positive frame anywhere: exit 1 trivially agrees, but positives are insufficient -> skipped
    plan, _ = P.plan_from_flags(_video(1000, ones, ~ones))
    assert plan == [(0, 1000, 0)]
    assert P.plan_from_flags(np.zeros((0, 3), bool))[0] == []


@pytest.mark.parametrize("seed", range(12))
def test_recursion_invariants_on_random_videos(seed):
    """Chunks tile the video in order, none is shorter than min_chunk (unless the video is), the depth stays
    within ceil(log2(|V|/min_chunk)), every level's rate stays within the bound, sampled frames are the
    chunk's own grid, and exact memoisation changes the cost but never the plan."""
    rng = np.random.default_rng(100 + seed)
    n, E = int(rng.integers(1, 3000)), int(rng.integers(2, 6))
    cfg = P.PlannerConfig(min_chunk=int(rng.integers(5, 120)), final_span=int(rng.integers(1, 12)),
                          posi_enough=float(rng.choice([0.0, 0.1, 0.3])), posi_skip=float(rng.choice([0.0, 0.05])))
    # piecewise-constant difficulty and event presence, like scenes in a video
    seg = np.cumsum(rng.integers(20, 400, 64))
    sid = np.searchsorted(seg, np.arange(n), side="right")
    ref = (rng.random(64) < 0.6)[sid] & (rng.random(n) < 0.9)
    need = rng.integers(1, E + 1, 64)[sid]                 # first exit that gets the frame right
    flags = np.stack([np.where(need <= e + 1, ref, rng.random(n) < 0.2) for e in range(E)], axis=1)
    flags[:, -1] = ref
    plan, pl = P.plan_from_flags(flags, cfg)
    pos = 0
    for a, ln, ep in plan:
        assert a == pos and ln > 0 and 0 <= ep <= E
        assert ln >= cfg.min_chunk or n < cfg.min_chunk or len(plan) == 1
        pos += ln
    assert pos == n
    d = _depth_by_doubling(n, cfg.min_chunk)
    assert pl.depth <= d
    for a, b, span, best, ratio in pl.trace:
        assert span >= cfg.final_span and 0 <= ratio <= 1 and 1 <= best <= E
    plan2, pl2 = P.plan_from_flags(flags, cfg, memo=False)
    assert plan2 == plan and [t for t in pl2.trace] == [t for t in pl.trace]
    assert len(pl.evaluated) == len(set(pl2.evaluated)) <= len(pl2.evaluated)
    assert len(set(pl.evaluated)) == len(pl.evaluated)


def test_nearby_reuse_borrows_only_inside_the_chunk_and_within_the_distance():
    """250 frames, min_chunk 60: depth 3 -> span0 80, top-level samples 0, 80, 160, 240.  The second half
    [125, 250) samples 125, 165, 205, 245 on span 40, off the parent's grid; the memoised frames inside it are
    160 and 240 (80 lies outside the chunk).  With reuse_dist 5: 165 borrows 160 and 245 borrows 240 (both 5
    away), 125 and 205 are evaluated.  With reuse_dist 40: 125 and 165 borrow 160, 205 and 245 borrow 240."""
    n = 250
    idx = np.arange(n)
    flags = _video(n, idx < 0, np.ones(n, bool))           # exit 1 always wrong -> recursion to the bottom
    cfg = P.PlannerConfig(min_chunk=60, final_span=10, reuse_dist=5)
    plan, pl = P.plan_from_flags(flags, cfg)
    assert [t[:3] for t in pl.trace][:3] == [(0, 250, 80), (0, 125, 40), (0, 62, 20)]
    first = [f for f in pl.evaluated]
    assert first[:4] == [0, 80, 160, 240]
    assert {125, 205} <= set(pl.evaluated) and not ({165, 245} & set(pl.evaluated))
    cfg2 = P.PlannerConfig(min_chunk=60, final_span=10, reuse_dist=40)
    plan2, pl2 = P.plan_from_flags(flags, cfg2)
    assert plan2 == plan                                    # the borrowed answers are the same here
    assert not ({125, 165, 205, 245} & set(pl2.evaluated))
    assert len(pl2.evaluated) < len(pl.evaluated)
