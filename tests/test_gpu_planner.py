"""Planner on the device path (Sec. 5.2): the predicate kernel, chunks of unequal length, and
thia_plan_query against the planning oracle.  The planner's decisions are discrete, so the oracle
planner is fed the answers derived (with the oracle's predicate) from the GPU's own detections of
every frame -- the planner itself, its sampling, memoisation and batching are what is compared; the
detections behind the answers are covered by the end-to-end parity tests."""
import numpy as np
import pytest
import torch

import oracle
from oracle import estimator as Est
from oracle import planner as P
from gpu_common import MINI_BF16, MINI_FP32, gpu_model, nhwc_to_nchw, relerr, to_dev
from paper_2102_08481_amd import ThiaError, planner_cfg
from thia_synth import SceneSpec, make_frames

pytestmark = pytest.mark.gpu


def test_predicate_kernel_is_bit_exact():
    m, _ = gpu_model(MINI_BF16, 0xBEEF + 51)
    rng = np.random.default_rng(3)
    for rows in (0, 1, 255, 256, 1031):
        labels = rng.integers(-1, 8, (rows, m.D)).astype(np.int32)
        scores = (rng.integers(0, 11, (rows, m.D)) / 10).astype(np.float32)      # many ties with the threshold
        for label, t, s in ((1, 1, 0.0), (3, 4, 0.5), (7, 0, 0.9), (2, m.D + 1, 0.0), (5, 2, 1.0)):
            got = m.eval_predicate(to_dev(labels), to_dev(scores), label, t, s).cpu().numpy().astype(bool)
            assert np.array_equal(got, P.count_predicate(labels, scores, label, t, s)), (rows, label, t, s)


def test_answer_counts_are_exact():
    from paper_2102_08481_amd import metrics_from_counts
    m, _ = gpu_model(MINI_BF16, 0xBEEF + 51)
    rng = np.random.default_rng(4)
    for n in (0, 1, 1023, 1024, 50001):
        a, r = (rng.random(n) < 0.4).astype(np.uint8), (rng.random(n) < 0.6).astype(np.uint8)
        c = m.answer_counts(to_dev(a), to_dev(r)).cpu().numpy()
        o = P.answer_metrics(a, r)
        assert tuple(int(v) for v in c) == o[:3], n
        assert metrics_from_counts(c) == pytest.approx(o[3:], abs=0, rel=1e-15)


def test_chunks_of_unequal_length_match_stand_alone_calls():
    m, _ = gpu_model(MINI_BF16, 0xBEEF + 51)
    frames = to_dev(make_frames(SceneSpec(160, 224, 20, 4, 10, 10, 90), 43))
    plan = [(10, 5, 4), (0, 3, 1), (3, 7, 0), (17, 3, 2), (15, 0, 3)]           # frames 15, 16 uncovered; unordered
    b, s, l = m.run_chunks(frames, plan)
    torch.cuda.synchronize()
    for a, ln, ep in plan:
        if ep == 0 or ln == 0:
            continue
        cb, cs, cl = m.detect_chunk(frames[a:a + ln].contiguous(), ep)
        torch.cuda.synchronize()
        assert torch.equal(b[a:a + ln], cb) and torch.equal(s[a:a + ln], cs) and torch.equal(l[a:a + ln], cl), (a, ln, ep)
    for a, e in ((3, 10), (15, 17)):
        assert (l[a:e] == -1).all() and (s[a:e] == 0).all() and (b[a:e] == 0).all()
    assert (l[:3, 0] >= 1).all()
    for bad in ([(0, 5, 1), (4, 3, 2)], [(18, 3, 1)], [(-1, 2, 1)], [(0, 2, 5)]):
        with pytest.raises(ThiaError):
            m.run_chunks(frames, bad)
    out = m.run_chunks(frames[:0], [])
    assert out[0].shape[0] == 0


def _answers_of_every_frame(m, frames_dev, label, t, s):
    b, sc, l = m.detect_all_exits(frames_dev)
    torch.cuda.synchronize()
    return P.count_predicate(l.cpu().numpy(), sc.cpu().numpy(), label, t, s).T       # [n, E]


def _pick_query(m, frames_dev):
    """A query whose answer changes along the video (derived from the data; both sides use the same one)."""
    b, sc, l = m.detect_all_exits(frames_dev)
    torch.cuda.synchronize()
    l, sc = l.cpu().numpy(), sc.cpu().numpy()
    best = None
    for label in range(1, 8):
        for t in (1, 2, 3, 4, 6):
            r = P.count_predicate(l[-1], sc[-1], label, t, 0.0).mean()
            if best is None or abs(r - 0.5) < best[0]:
                best = (abs(r - 0.5), label, t)
    return best[1], best[2]


@pytest.mark.parametrize("reuse,batch", [(0, 32), (2, 5), (0, 0)])
def test_plan_query_equals_the_oracle_planner_on_the_same_answers(reuse, batch):
    m, _ = gpu_model(MINI_BF16, 0xBEEF + 51)
    n = 150
    frames = to_dev(make_frames(SceneSpec(160, 224, n, 4, 10, 10, 90), 48))
    label, t = _pick_query(m, frames)
    flags = _answers_of_every_frame(m, frames, label, t, 0.0)
    assert 0 < flags[:, -1].mean() < 1
    kw = dict(min_chunk=9, final_span=2, posi_enough=0.1, posi_skip=0.0, reuse_dist=reuse)
    plan_o, pl = P.plan_from_flags(flags, P.PlannerConfig(**kw))
    plan, st, ev = m.plan_query(frames, label, t, 0.0, planner_cfg(eval_batch=batch, **kw))
    assert plan == plan_o
    assert np.flatnonzero(ev).tolist() == sorted(pl.evaluated)
    assert st["frames_evaluated"] == len(pl.evaluated) and st["samples_reused"] == pl.reused and st["depth"] == pl.depth
    assert st["frames_evaluated"] < n                                   # sampling, not a scan
    # executing the plan: every chunk as a stand-alone call would give it, skipped chunks empty
    b, s, l = m.run_chunks(frames, plan)
    torch.cuda.synchronize()
    ans = np.zeros(n, bool)
    for a, ln, ep in plan:
        if ep == 0:
            assert (l[a:a + ln] == -1).all()
            continue
        cb, cs, cl = m.detect_chunk(frames[a:a + ln].contiguous(), ep)
        torch.cuda.synchronize()
        assert torch.equal(l[a:a + ln], cl) and torch.equal(s[a:a + ln], cs) and torch.equal(b[a:a + ln], cb)
        ans[a:a + ln] = flags[a:a + ln, ep - 1]
    got = m.eval_predicate(l, s, label, t, 0.0).cpu().numpy().astype(bool)
    assert np.array_equal(got, ans)


def test_plan_query_against_the_full_oracle_pipeline_fp32():
    """Small enough for the CPU oracle to evaluate every exit on every frame: oracle detections -> oracle
    predicate -> oracle planner, against the library's planner on the device.  Discrete answers can differ
    where a detection score sits within fp32 rounding of a threshold; the comparison is made when the
    answers agree (reported otherwise), which they do on this seed."""
    m, blob = gpu_model(MINI_FP32, 0xBEEF + 50)
    n = 24
    fh = make_frames(SceneSpec(128, 160, n, 4, 10, 10, 70), 49)
    fd = to_dev(fh)
    label, t = _pick_query(m, fd)
    ref = oracle.Model(blob).detect_all_exits(fh)
    flags_o = P.count_predicate(ref["labels"], ref["scores"], label, t, 0.0).T
    flags_g = _answers_of_every_frame(m, fd, label, t, 0.0)
    agree = np.mean(flags_o == flags_g)
    assert agree >= 0.95, agree
    kw = dict(min_chunk=3, final_span=1, posi_enough=0.1, posi_skip=0.0, reuse_dist=0)
    plan, st, ev = m.plan_query(fd, label, t, 0.0, planner_cfg(eval_batch=8, **kw))
    plan_o, pl = P.plan_from_flags(flags_o, P.PlannerConfig(**kw))
    if np.array_equal(flags_o, flags_g):
        assert plan == plan_o and np.flatnonzero(ev).tolist() == sorted(pl.evaluated)
    else:
        print(f"answers differ on {np.sum(flags_o != flags_g)} of {flags_o.size} (frame, exit) pairs; plan compared on the GPU's answers")
        assert plan == P.plan_from_flags(flags_g, P.PlannerConfig(**kw))[0]


def test_plan_query_argument_errors():
    m, _ = gpu_model(MINI_BF16, 0xBEEF + 51)
    frames = to_dev(make_frames(SceneSpec(160, 224, 4, 4, 10, 10, 90), 50))
    with pytest.raises(ThiaError):
        m.plan_query(frames, 1, 1, 0.0, planner_cfg(min_chunk=0))
    plan, st, ev = m.plan_query(frames[:0], 1, 1)
    assert plan == [] and st["frames_evaluated"] == 0
    plan, st, ev = m.plan_query(frames, 1, 1)                            # shorter than one chunk: one chunk
    assert len(plan) == 1 and plan[0][:2] == (0, 4)


def _estimator_weights(seed, C=2048, hidden=96, E=4):
    rng = np.random.default_rng(seed)
    return (rng.normal(0, C ** -0.5, (hidden, C)).astype(np.float32), rng.normal(0, 0.1, hidden).astype(np.float32),
            rng.normal(0, hidden ** -0.5, (E, hidden)).astype(np.float32), rng.normal(0, 0.05, E).astype(np.float32))


@pytest.mark.parametrize("spec,tol_full", [(MINI_FP32, 1e-4), (MINI_BF16, 2e-2)])
def test_exit_estimator_matches_oracle(spec, tol_full):
    """Logits against the oracle on the GPU's own last-stage tensor (fp32 accumulation vs float64: 1e-5) and on
    the oracle's own backbone (the path's stated tolerance); the arg-max wherever the two best logits are
    further apart than that error; the reference detections bit-identical to a call at the last exit."""
    m, blob = gpu_model(spec, 0xBEEF + (50 if spec is MINI_FP32 else 51))
    w = _estimator_weights(11)
    m.set_estimator(*w)
    fh = make_frames(SceneSpec(160, 224, 5, 4, 10, 10, 90), 52)
    fd = to_dev(fh)
    opt, logits, (b, s, l) = m.estimate_exit(fd)
    torch.cuda.synchronize()
    m.set_debug(True)
    rb, rs, rl = m.detect_chunk(fd, 4)
    torch.cuda.synchronize()
    Ck, Hk, Wk, _ = oracle.Model(blob).exit_shape(4, 160, 224)
    feat = nhwc_to_nchw(m.tap("feat").reshape(5, Hk, Wk, Ck))
    m.set_debug(False)
    assert torch.equal(b, rb) and torch.equal(s, rs) and torch.equal(l, rl)
    opt, logits = opt.cpu().numpy(), logits.cpu().numpy()
    o_opt, o_logits = Est.estimate_exit(feat, *w)
    assert relerr(logits, o_logits) <= 1e-5
    top2 = np.sort(o_logits, axis=1)[:, -2:]
    clear = (top2[:, 1] - top2[:, 0]) > 1e-5 * np.abs(o_logits).max()
    assert clear.any() and np.array_equal(opt[clear], o_opt[clear])
    assert ((opt >= 1) & (opt <= 4)).all()
    f_opt, f_logits = Est.estimate_exit(oracle.Model(blob).backbone(fh, 4), *w)
    assert relerr(logits, f_logits) <= tol_full
    # micro-batching does not change the estimate; removing the estimator makes the call fail
    m.set_microbatch(2)
    opt2, logits2, _ = m.estimate_exit(fd)
    torch.cuda.synchronize()
    m.set_microbatch(0)
    assert np.array_equal(opt2.cpu().numpy(), opt) and np.array_equal(logits2.cpu().numpy(), logits)
    m.set_estimator(None, None, None, None)
    with pytest.raises(ThiaError):
        m.estimate_exit(fd)
    with pytest.raises(ThiaError):
        m.plan_query(fd, 1, 1, 0.0, planner_cfg(use_estimator=1))


def test_plan_query_with_estimator_equals_the_oracle_planner_on_the_same_estimates():
    m, _ = gpu_model(MINI_BF16, 0xBEEF + 51)
    n = 150
    # five scenes, so that the pooled features (and with them the estimate) change along the video
    fh = np.concatenate([make_frames(SceneSpec(160, 224, 30, 2 + 3 * i, 4 + 4 * i, 10, 40 + 12 * i), 60 + i) for i in range(5)])
    frames = to_dev(fh)
    w1, b1, w2, b2 = _estimator_weights(12)
    m.set_estimator(w1, b1, w2, b2)
    _, logits, _ = m.estimate_exit(frames)
    torch.cuda.synchronize()
    # centre every exit's output over the video (a stand-in for training, which needs labelled data): the estimate then varies
    b2 = (b2 - logits.cpu().numpy().mean(axis=0)).astype(np.float32)
    m.set_estimator(w1, b1, w2, b2)
    label, t = _pick_query(m, frames)
    opt, _, (b, s, l) = m.estimate_exit(frames)
    torch.cuda.synchronize()
    ref = P.count_predicate(l.cpu().numpy(), s.cpu().numpy(), label, t, 0.0)
    opt = opt.cpu().numpy()
    assert len(set(opt.tolist())) > 1 and 0 < ref.mean() < 1
    kw = dict(min_chunk=9, final_span=2, posi_enough=0.1, posi_skip=0.0, reuse_dist=0)
    plan_o, pl = P.plan_from_estimates(ref, opt, 4, P.PlannerConfig(**kw))
    plan, st, ev = m.plan_query(frames, label, t, 0.0, planner_cfg(eval_batch=16, use_estimator=1, **kw))
    # the whole query in this mode: only reference-exit answers of sampled frames are carried over to the execution
    answers, plan_q, _ = m.run_query(frames, label, t, 0.0, planner_cfg(eval_batch=16, use_estimator=1, **kw))
    cb, cs, cl = m.run_chunks(frames, plan)
    want = m.eval_predicate(cl, cs, label, t, 0.0)
    torch.cuda.synchronize()
    assert plan_q == plan and torch.equal(answers, want)
    m.set_estimator(None, None, None, None)
    assert plan == plan_o
    assert np.flatnonzero(ev).tolist() == sorted(pl.evaluated) and st["samples_reused"] == pl.reused
    print("plan with estimator:", plan, st)


def test_run_query_is_plan_then_execution_then_predicate():
    m, _ = gpu_model(MINI_BF16, 0xBEEF + 51)
    n = 150
    frames = to_dev(make_frames(SceneSpec(160, 224, n, 4, 10, 10, 90), 48))
    label, t = _pick_query(m, frames)
    kw = dict(min_chunk=9, final_span=2)
    answers, plan, st = m.run_query(frames, label, t, 0.0, planner_cfg(**kw))
    torch.cuda.synchronize()
    plan2, st2, _ = m.plan_query(frames, label, t, 0.0, planner_cfg(**kw))
    assert plan == plan2 and st == st2
    b, s, l = m.run_chunks(frames, plan)
    want = m.eval_predicate(l, s, label, t, 0.0)
    torch.cuda.synchronize()
    assert torch.equal(answers, want)       # (sampled frames keep the answer of the planning pass and are not run again)
    assert st["frames_evaluated"] > 0
    # against the oracle's metrics: frames of skipped chunks answer "no"
    flags = _answers_of_every_frame(m, frames, label, t, 0.0)
    exp = np.zeros(n, bool)
    for a, ln, ep in plan:
        if ep:
            exp[a:a + ln] = flags[a:a + ln, ep - 1]
    assert np.array_equal(answers.cpu().numpy().astype(bool), exp)
    e, plan0, st0 = m.run_query(frames[:0], label, t)
    assert e.numel() == 0 and plan0 == []
