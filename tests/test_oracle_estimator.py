"""Pins for the exit-estimation oracle (Sec. 5.3): the two-layer network against plain loops and closed
forms, the extrapolated TP/FP/FN against the per-frame case definitions, and what follows from them.  CPU only."""
import numpy as np
import pytest

from oracle import estimator as Est
from oracle import planner as P


def test_network_matches_plain_loops_on_a_tiny_case():
    rng = np.random.default_rng(1)
    n, C, Hk, Wk, hid, E = 3, 5, 2, 3, 4, 3
    feat = rng.normal(size=(n, C, Hk, Wk))
    w1, b1, w2, b2 = rng.normal(size=(hid, C)), rng.normal(size=hid), rng.normal(size=(E, hid)), rng.normal(size=E)
    opt, logits = Est.estimate_exit(feat, w1, b1, w2, b2)
    for f in range(n):
        pooled = [sum(feat[f, c, y, x] for y in range(Hk) for x in range(Wk)) / (Hk * Wk) for c in range(C)]
        h = [max(0.0, b1[j] + sum(w1[j, c] * pooled[c] for c in range(C))) for j in range(hid)]
        lg = [b2[e] + sum(w2[e, j] * h[j] for j in range(hid)) for e in range(E)]
        assert np.allclose(logits[f], lg, rtol=1e-12, atol=1e-12)
        assert opt[f] == 1 + max(range(E), key=lambda e: (lg[e], -e))


def test_network_closed_forms():
    # features constant over space: pooling returns them; first layer picks channels; second layer is a signed copy
    feat = np.zeros((2, 3, 4, 5))
    feat[0] = np.array([1.0, -2.0, 3.0])[:, None, None]
    feat[1] = np.array([-1.0, 5.0, 0.5])[:, None, None]
    w1, b1 = np.eye(3), np.zeros(3)
    w2, b2 = np.array([[1.0, 0, 0], [0, 1.0, 0], [0, 0, 1.0]]), np.array([0.0, 0.0, 0.1])
    opt, logits = Est.estimate_exit(feat, w1, b1, w2, b2)
    assert np.allclose(logits, [[1.0, 0.0, 3.1], [0.0, 5.0, 0.6]])       # the ReLU removed -2 and -1
    assert opt.tolist() == [3, 2]
    # a tie goes to the faster exit
    opt, _ = Est.estimate_exit(feat[:1], w1, b1, np.zeros((3, 3)), np.zeros(3))
    assert opt.tolist() == [1]
    # spatial average, not sum: doubling the map size with the same values changes nothing
    big = np.repeat(feat, 2, axis=2)
    assert np.allclose(Est.estimate_exit(big, w1, b1, w2, b2)[1], logits)


def test_extrapolated_counts_follow_the_case_definitions():
    rng = np.random.default_rng(2)
    for _ in range(100):
        n, E = int(rng.integers(1, 30)), int(rng.integers(1, 6))
        ref, opt = rng.random(n) < 0.5, rng.integers(1, E + 1, n)
        for k in range(1, E + 1):
            tp = sum(1 for x in range(n) if ref[x] and k >= opt[x])          # g
            fp = sum(1 for x in range(n) if not ref[x] and k < opt[x])       # g'
            fn = sum(1 for x in range(n) if ref[x] and k < opt[x])           # g''
            assert Est.extrapolated_counts(ref, opt, k) == (tp, fp, fn)
            assert tp + fn == ref.sum()                                      # every positive frame is a TP or a FN
        # a deeper exit is never worse, and the last exit is perfect
        seq = [Est.extrapolated_counts(ref, opt, k) for k in range(1, E + 1)]
        assert all(a[0] <= b[0] and a[1] >= b[1] and a[2] >= b[2] for a, b in zip(seq, seq[1:]))
        assert seq[-1][1] == 0 and seq[-1][2] == 0


def test_estimated_selection_equals_evaluated_selection_on_the_implied_answers():
    """If exit k answers like the reference exactly when k >= OPT_EP(x) (the section's premise), evaluation-based
    selection on those answers and estimation-based selection agree."""
    rng = np.random.default_rng(3)
    for _ in range(200):
        n, E = int(rng.integers(1, 40)), int(rng.integers(1, 6))
        ref, opt = rng.random(n) < rng.random(), rng.integers(1, E + 1, n)
        cfg = P.PlannerConfig(precision=float(rng.choice([0.5, 0.8, 1.0])), recall=float(rng.choice([0.5, 0.8, 1.0])))
        implied = np.stack([np.where(k >= opt, ref, ~ref) for k in range(1, E + 1)], axis=1)
        assert Est.pick_best_ep_estimated(ref, opt, E, cfg) == P.pick_best_ep(implied, cfg)


def test_worked_example():
    """Six samples, three exits.  Positives: OPT = 1, 2, 3, 3; negatives: OPT = 1, 2.
    k=1: TP 1, FN 3, FP 1 -> precision 1/2, recall 1/4.  k=2: TP 2, FN 2, FP 0 -> 1, 1/2.  k=3: TP 4 -> 1, 1."""
    ref = np.array([1, 1, 1, 1, 0, 0], bool)
    opt = np.array([1, 2, 3, 3, 1, 2])
    assert [Est.extrapolated_counts(ref, opt, k) for k in (1, 2, 3)] == [(1, 1, 3), (2, 0, 2), (4, 0, 0)]
    assert Est.pick_best_ep_estimated(ref, opt, 3, P.PlannerConfig())[0] == 3
    assert Est.pick_best_ep_estimated(ref, opt, 3, P.PlannerConfig(precision=0.9, recall=0.5))[0] == 2
    assert Est.pick_best_ep_estimated(ref, opt, 3, P.PlannerConfig(precision=0.5, recall=0.25)) == (1, 4 / 6)


def test_planner_with_estimates_on_a_hand_worked_video():
    """400 frames, all positive; OPT_EP = 1 on frames 0..199 and 2 after: same plan as the evaluated case."""
    ref = np.ones(400, bool)
    opt = np.where(np.arange(400) < 200, 1, 2)
    plan, pl = P.plan_from_estimates(ref, opt, 2)
    assert plan == [(0, 200, 1), (200, 100, 2), (300, 100, 2)]
    assert len(pl.evaluated) == 30 and pl.reused == 20
