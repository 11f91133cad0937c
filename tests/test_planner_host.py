"""The library's planner (host logic, no device work) against the planning oracle on tables of answers:
identical plan, identical set of evaluated frames, identical reuse count.  CPU only."""
import numpy as np
import pytest

from oracle import planner as P
from paper_2102_08481_amd import ThiaError, plan_from_flags, planner_cfg


def _both(flags, **kw):
    ocfg = P.PlannerConfig(**{k: v for k, v in kw.items() if k != "eval_batch"})
    plan_o, pl = P.plan_from_flags(flags, ocfg)
    plan_l, st, ev = plan_from_flags(flags, planner_cfg(**kw))
    return plan_o, pl, plan_l, st, ev


def _random_video(rng, n, E):
    seg = np.cumsum(rng.integers(15, 300, 96))
    sid = np.searchsorted(seg, np.arange(n), side="right")
    ref = (rng.random(96) < rng.random())[sid] & (rng.random(n) < 0.95)
    need = rng.integers(1, E + 1, 96)[sid]
    flags = np.stack([np.where(need <= e + 1, ref, rng.random(n) < 0.15) for e in range(E)], axis=1)
    flags[:, -1] = ref
    return flags


def test_defaults_are_the_papers_constants():
    c = planner_cfg()
    assert (c.precision, c.recall, c.min_chunk, c.final_span) == (0.8, 0.8, 100, 10)   # Sec. 5.2
    assert (c.posi_enough, c.posi_skip, c.reuse_dist) == (P.PlannerConfig().posi_enough, P.PlannerConfig().posi_skip, 0)


@pytest.mark.parametrize("seed", range(40))
def test_library_planner_equals_oracle_on_random_videos(seed):
    rng = np.random.default_rng(7000 + seed)
    n, E = int(rng.integers(1, 6000)), int(rng.integers(1, 6))
    kw = dict(min_chunk=int(rng.integers(1, 150)), final_span=int(rng.integers(1, 14)),
              precision=float(rng.choice([0.5, 0.8, 0.95, 1.0])), recall=float(rng.choice([0.5, 0.8, 1.0])),
              posi_enough=float(rng.choice([0.0, 0.1, 0.4])), posi_skip=float(rng.choice([0.0, 0.02, 0.1])),
              reuse_dist=int(rng.choice([0, 0, 1, 3, 8])), eval_batch=int(rng.choice([0, 1, 7, 32])))
    flags = _random_video(rng, n, E)
    plan_o, pl, plan_l, st, ev = _both(flags, **kw)
    assert plan_l == plan_o
    assert np.flatnonzero(ev).tolist() == sorted(pl.evaluated)
    assert st["frames_evaluated"] == len(pl.evaluated) and st["samples_reused"] == pl.reused
    assert st["depth"] == pl.depth and st["n_chunks"] == len(plan_o)


def test_worked_examples_through_the_library():
    idx = np.arange(400)
    flags = np.stack([idx < 200, np.ones(400, bool)], axis=1)
    plan, st, ev = plan_from_flags(flags)
    assert plan == [(0, 200, 1), (200, 100, 2), (300, 100, 2)]
    assert st["frames_evaluated"] == 30 and st["samples_reused"] == 20 and st["depth"] == 2
    flags = np.stack([np.zeros(400, bool), idx >= 200], axis=1)
    assert plan_from_flags(flags)[0] == [(0, 200, 0), (200, 100, 2), (300, 100, 2)]
    assert plan_from_flags(np.zeros((0, 4), np.uint8))[0] == []


def test_bad_configurations_are_refused():
    flags = np.zeros((50, 2), np.uint8)
    for bad in (dict(precision=1.5), dict(recall=-0.1), dict(min_chunk=0), dict(final_span=0), dict(posi_enough=2.0),
                dict(reuse_dist=-1)):
        with pytest.raises(ThiaError):
            plan_from_flags(flags, planner_cfg(**bad))
    with pytest.raises(KeyError):
        planner_cfg(no_such_field=1)


@pytest.mark.parametrize("seed", range(12))
def test_estimation_based_planning_through_the_answer_table(seed):
    """Sec. 5.3: with OPT_EP per frame, exit k counts as right exactly when k >= OPT_EP.  The library plans
    estimation-based by handing its planner that implied table; the oracle evaluates the section's TP/FP/FN
    sums directly.  Same plan, same evaluated frames."""
    rng = np.random.default_rng(9000 + seed)
    n, E = int(rng.integers(1, 4000)), int(rng.integers(1, 6))
    seg = np.cumsum(rng.integers(15, 300, 96))
    sid = np.searchsorted(seg, np.arange(n), side="right")
    ref = (rng.random(96) < rng.random())[sid] & (rng.random(n) < 0.95)
    opt = np.clip(rng.integers(1, E + 1, 96)[sid] + (rng.random(n) < 0.1), 1, E)
    kw = dict(min_chunk=int(rng.integers(1, 150)), final_span=int(rng.integers(1, 14)), reuse_dist=int(rng.choice([0, 2])))
    plan_o, pl = P.plan_from_estimates(ref, opt, E, P.PlannerConfig(**kw))
    implied = np.stack([(k >= opt) == ref for k in range(1, E + 1)], axis=1)
    plan_l, st, ev = plan_from_flags(implied, planner_cfg(**kw))
    assert plan_l == plan_o
    assert np.flatnonzero(ev).tolist() == sorted(pl.evaluated) and st["samples_reused"] == pl.reused


def test_metrics_from_counts_equal_the_oracle():
    from paper_2102_08481_amd import metrics_from_counts
    rng = np.random.default_rng(4)
    cases = [(0, 0, 0), (5, 0, 0), (0, 3, 0), (0, 0, 2), (0, 3, 2)] + [tuple(int(v) for v in rng.integers(0, 50, 3)) for _ in range(50)]
    for tp, fp, fn in cases:
        pred = np.r_[np.ones(tp + fp, bool), np.zeros(fn, bool)]
        ref = np.r_[np.ones(tp, bool), np.zeros(fp, bool), np.ones(fn, bool)]
        o = P.answer_metrics(pred, ref)
        assert o[:3] == (tp, fp, fn)
        assert metrics_from_counts((tp, fp, fn)) == pytest.approx(o[3:], abs=0, rel=1e-15)
