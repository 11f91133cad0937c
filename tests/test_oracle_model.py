"""Pins of the composed CPU oracle: the wiring of the network against an independent
float64 reconstruction with torch CPU ops, the structural facts the paper states
(exit channels of Table 4, shared prefix, early stop, plan semantics).  CPU only."""
import os
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from thia_synth import ModelSpec, SceneSpec, make_blob, make_frames, split_blob, CONFIGS
from thia_synth.weights import tensor_list

GOLD = os.path.join(os.path.dirname(__file__), "golden")

MINI = ModelSpec(precision=0, n_exits=4, blocks=(2, 1, 2, 1), stem_ch=8, base_width=8, head_ch=16, fc_dim=32,
                 sizes=(16.0, 32.0), ratios=(0.5, 1.0, 2.0), pre_nms=60, post_nms=20, n_classes=4, max_det=10)
MINI_SCENE = SceneSpec(72, 104, 3, 3, 6, 8, 40)


@pytest.fixture(scope="module")
def mini():
    blob = make_blob(MINI, 77, res_gain=0.25, pred_std=0.05)
    frames = make_frames(MINI_SCENE, 78)
    return blob, frames


def test_exit_channels_match_table4():
    rows = [l.split() for l in open(os.path.join(GOLD, "table4_exit_channels.txt")) if l.strip() and l[0] != "#"]
    table = {int(r[0]): (int(r[1]), int(r[2])) for r in rows}
    spec = CONFIGS[3].model
    assert spec.stem_ch == table[1][0]
    m = oracle.Model(make_blob(replace(spec, blocks=(1, 1, 1, 1), fc_dim=8), 1))
    for k in range(1, 5):                       # repository exit k = paper EP-(k+1)
        C, Hk, Wk, stride = m.exit_shape(k, 540, 960)
        assert C == table[k + 1][0] == spec.stage_channels(k)
        assert stride == 4 << (k - 1)
    assert [m.exit_shape(k, 540, 960)[1:3] for k in range(1, 5)] == [(135, 240), (68, 120), (34, 60), (17, 30)]
    assert all(k == 3 for _, k in table.values())          # first RPN layer is 3x3 at every exit


def torch_backbone(w, spec, frames, ep):
    """Independent float64 statement of the truncated backbone with library convolutions."""
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
    x = (t(frames.astype(np.float32)) - spec.mean) / spec.std
    x = F.relu(F.conv2d(x, t(w["stem.w"]), t(w["stem.b"]), stride=2, padding=3))
    x = F.max_pool2d(x, 3, 2, 1)
    outs = []
    for s in range(1, ep + 1):
        for b in range(spec.blocks[s - 1]):
            p = f"s{s}.b{b}"
            st = 2 if (b == 0 and s > 1) else 1
            y = F.relu(F.conv2d(x, t(w[p + ".conv1.w"]), t(w[p + ".conv1.b"])))
            y = F.relu(F.conv2d(y, t(w[p + ".conv2.w"]), t(w[p + ".conv2.b"]), stride=st, padding=1))
            y = F.conv2d(y, t(w[p + ".conv3.w"]), t(w[p + ".conv3.b"]))
            sc = F.conv2d(x, t(w[p + ".short.w"]), t(w[p + ".short.b"]), stride=st) if b == 0 else x
            x = F.relu(y + sc)
        outs.append(x)
    return outs


def relerr(a, b):
    return float(np.max(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64))) / max(np.max(np.abs(b)), 1e-30))


def test_network_wiring_matches_torch_float64(mini):
    blob, frames = mini
    w = split_blob(MINI, blob)
    m = oracle.Model(blob)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
    for ep in (1, 3, 4):
        r = m.detect(frames, ep, taps=oracle.TAP_NAMES)
        ref = torch_backbone(w, MINI, frames, ep)[-1]
        assert r["feat"].shape == tuple(ref.shape)
        assert relerr(r["feat"], ref.numpy()) < 1e-5
        e = f"e{ep}"
        hf = F.conv2d(ref, t(w[e + ".lateral.w"]), t(w[e + ".lateral.b"]))          # bias, no activation
        assert relerr(r["head_feat"], hf.numpy()) < 1e-5
        assert (r["head_feat"] < 0).any()
        h = F.relu(F.conv2d(hf, t(w[e + ".rpn.conv.w"]), t(w[e + ".rpn.conv.b"]), padding=1))
        obj = F.conv2d(h, t(w[e + ".rpn.obj.w"]), t(w[e + ".rpn.obj.b"]))              # [n,A,Hk,Wk]
        dl = F.conv2d(h, t(w[e + ".rpn.delta.w"]), t(w[e + ".rpn.delta.b"]))          # [n,4A,Hk,Wk]
        n, A = obj.shape[0], obj.shape[1]
        # anchor-index order (y, x, a); delta channel 4a + j
        assert relerr(r["rpn_logits"], obj.permute(0, 2, 3, 1).reshape(n, -1).numpy()) < 1e-5
        d = dl.reshape(n, A, 4, *dl.shape[2:]).permute(0, 3, 4, 1, 2).reshape(n, -1, 4)
        assert relerr(r["rpn_deltas"], d.numpy()) < 1e-5
        # box head on the oracle's own ROI features (flatten order c, ph, pw)
        for f in range(n):
            nr = r["roi_n"][f]
            x = t(r["roi_feat"][f, :nr])
            h1 = F.relu(x @ t(w[e + ".fc1.w"]).T + t(w[e + ".fc1.b"]))
            h2 = F.relu(h1 @ t(w[e + ".fc2.w"]).T + t(w[e + ".fc2.b"]))
            cl = h2 @ t(w[e + ".cls.w"]).T + t(w[e + ".cls.b"])
            bd = h2 @ t(w[e + ".box.w"]).T + t(w[e + ".box.b"])
            assert relerr(r["cls_logits"][f, :nr], cl.numpy()) < 1e-5
            assert relerr(r["box_deltas"][f, :nr], bd.numpy()) < 1e-5
            assert relerr(r["cand_scores"][f, :nr], torch.softmax(cl, 1).numpy()) < 1e-5


def test_detect_is_the_composition_of_the_pinned_steps(mini):
    blob, frames = mini
    m = oracle.Model(blob)
    H, W = frames.shape[2:]
    for ep in (2, 4):
        r = m.detect(frames, ep, taps=oracle.TAP_NAMES)
        Ck, Hk, Wk, stride = m.exit_shape(ep, H, W)
        for f in range(frames.shape[0]):
            idx, _ = oracle.topk(r["rpn_logits"][f], MINI.pre_nms)
            k = r["topk_n"][f]
            assert k == min(MINI.pre_nms, Hk * Wk * MINI.n_anchors)
            assert np.array_equal(idx, r["topk_idx"][f, :k])
            boxes = []
            for i in idx:
                bx, ok = oracle.decode(m.anchor(i, Wk, stride), r["rpn_deltas"][f, i], W, H)
                if ok:
                    boxes.append(bx)
            boxes = np.array(boxes, np.float32).reshape(-1, 4)
            assert r["prop_n"][f] == len(boxes) and np.array_equal(r["prop_boxes"][f, :len(boxes)], boxes)
            keep = oracle.nms(boxes, MINI.rpn_nms_thr, MINI.post_nms)
            assert r["roi_n"][f] == len(keep) and np.array_equal(r["rois"][f, :len(keep)], boxes[keep])
            rf = oracle.roialign(r["head_feat"][f], boxes[keep], stride)
            assert np.array_equal(r["roi_feat"][f, :len(keep)], rf.reshape(len(keep), -1))
            nr = len(keep)
            ob, osc, ol, nd = oracle.select_detections(r["cand_scores"][f, :nr], r["cand_boxes"][f, :nr],
                                                       MINI.score_thr, MINI.det_nms_thr, MINI.max_det)
            assert nd == r["det_n"][f]
            assert np.array_equal(ob, r["boxes"][f]) and np.array_equal(osc, r["scores"][f]) and np.array_equal(ol, r["labels"][f])
            # per-class boxes = decode of the ROI (as centre/size) with that class's deltas
            for rr in (0, nr - 1):
                q = r["rois"][f, rr]
                anc = [q[0] + 0.5 * (q[2] - q[0]), q[1] + 0.5 * (q[3] - q[1]), q[2] - q[0], q[3] - q[1]]
                for c in range(1, MINI.n_classes):
                    bx, _ = oracle.decode(anc, r["box_deltas"][f, rr, 4 * c:4 * c + 4], W, H)
                    assert np.array_equal(bx, r["cand_boxes"][f, rr, c])
        assert (r["det_n"] > 0).all()            # the synthetic recipe gives non-degenerate detections


def test_exit_k_backbone_is_prefix_of_exit_k_plus_1(mini):
    """Exits share parameters and features (Sec. 6.8 memory discussion): stage k's tensor while
    running the deepest exit is bit-identical to exit k's own backbone output."""
    blob, frames = mini
    m = oracle.Model(blob)
    full, stages = m.backbone(frames, 4, stages=True)
    assert np.array_equal(full, stages[3])
    for k in (1, 2, 3):
        assert np.array_equal(m.backbone(frames, k), stages[k - 1])


def test_early_stop_never_touches_later_stages_or_other_exits(mini):
    """Inference is short-circuited at the exit (Sec. 4.1): the result at exit 2 cannot depend
    on conv4_x/conv5_x weights nor on another exit's heads."""
    blob, frames = mini
    w = split_blob(MINI, blob.copy())
    b2 = blob.copy()
    w2 = split_blob(MINI, b2)
    for name in w2:
        if name.startswith(("s3.", "s4.", "e1.", "e3.", "e4.")):
            w2[name][...] = np.nan
    a = oracle.Model(blob).detect(frames, 2)
    b = oracle.Model(b2).detect(frames, 2)
    for key in ("boxes", "scores", "labels"):
        assert np.array_equal(a[key], b[key])
    assert (a["labels"] >= 0).any()


def test_all_exits_result_is_each_exit_alone_in_exit_major_order(mini):
    """Evaluation-based exit selection (Sec. 5.2) looks at every exit on the same sampled frames: block e
    of the all-exits result is exit e's own result, and it survives poisoning everything exit e never reads."""
    blob, frames = mini
    allx = oracle.Model(blob).detect_all_exits(frames)
    assert allx["labels"].shape[:2] == (4, frames.shape[0])
    for ep in (1, 2, 3, 4):
        one = oracle.Model(blob).detect(frames, ep)
        for key in ("boxes", "scores", "labels"):
            assert np.array_equal(allx[key][ep - 1], one[key])
    b2 = blob.copy()
    w2 = split_blob(MINI, b2)
    for name in w2:
        if name.startswith(("s4.", "e4.")):
            w2[name][...] = np.nan
    poisoned = oracle.Model(b2).detect_all_exits(frames)
    for key in ("boxes", "scores", "labels"):
        assert np.array_equal(poisoned[key][:3], allx[key][:3])
    assert (allx["labels"][:, :, 0] >= 1).all()


def test_plan_equals_per_chunk_calls_and_skip_is_empty(mini):
    """A plan is a list of chunks each with an exit or 'skip' (Sec. 3, execution engine)."""
    blob, _ = mini
    frames = make_frames(replace(MINI_SCENE, n_frames=8), 79)
    m = oracle.Model(blob)
    plan = [3, 0, 1, 4]
    out = m.run_plan(frames, 2, plan)
    for c, ep in enumerate(plan):
        one = m.detect(frames[2 * c:2 * c + 2], ep)
        for key in ("boxes", "scores", "labels"):
            assert np.array_equal(out[key][2 * c:2 * c + 2], one[key])
    assert np.all(out["labels"][2:4] == -1) and np.all(out["scores"][2:4] == 0) and np.all(out["boxes"][2:4] == 0)
    assert np.all(out["labels"][0:2, 0] >= 1)


def test_outputs_are_padded_and_sorted(mini):
    blob, frames = mini
    r = oracle.Model(blob).detect(frames, 1, taps=["det_n"])
    for f in range(frames.shape[0]):
        n = r["det_n"][f]
        assert np.all(r["labels"][f, :n] >= 1) and np.all(r["labels"][f, :n] < MINI.n_classes)
        assert np.all(r["labels"][f, n:] == -1) and np.all(r["scores"][f, n:] == 0)
        assert np.all(np.diff(r["scores"][f, :n]) <= 0) and np.all(r["scores"][f, :n] > MINI.score_thr)
        b = r["boxes"][f, :n]
        assert np.all(b[:, 0] >= 0) and np.all(b[:, 2] <= frames.shape[3]) and np.all(b[:, 3] <= frames.shape[2])


def test_bf16_mode_is_close_to_fp32_and_stores_bf16(mini):
    blob, frames = mini
    a = oracle.Model(blob, precision=0).detect(frames, 3, taps=["feat", "rpn_logits"])
    b = oracle.Model(blob, precision=1).detect(frames, 3, taps=["feat", "rpn_logits"])
    assert relerr(b["feat"], a["feat"]) < 2e-2 and relerr(b["rpn_logits"], a["rpn_logits"]) < 2e-2
    assert np.array_equal(b["feat"], torch.from_numpy(b["feat"]).to(torch.bfloat16).float().numpy())
    assert not np.array_equal(b["feat"], a["feat"])


def test_bad_blob_and_bad_exit():
    with pytest.raises(ValueError):
        oracle.Model(np.zeros(300, np.uint8))
    blob = make_blob(MINI, 1)
    with pytest.raises(ValueError):
        oracle.Model(blob[:-4])
    m = oracle.Model(blob)
    with pytest.raises(ValueError):
        m.detect(np.zeros((1, 3, 32, 32), np.uint8), 5)


STEM5 = ModelSpec(precision=0, n_exits=5, stem_exit=1, blocks=(1, 1, 1, 1), has_lateral=0, fc_dim=16, pre_nms=60, post_nms=20,
                  n_classes=4, base_width=8, stem_ch=8, sizes=(16.0, 32.0), ratios=(1.0,))


def test_five_exit_variant_with_an_exit_on_the_stem_stage():
    """The paper's case study has five exits, the first on the 64-channel stage in front of the bottleneck stages and
    each unit's first layer sized to its stage (Sec. 4.2, Table 4).  With the stem-exit flag exit 1 reads the pooled
    stem output at stride 4, exit k >= 2 reads what exit k - 1 of the four-exit numbering reads, and the same
    weights give the same detections there."""
    blob5 = make_blob(STEM5, 5)
    frames = make_frames(replace(MINI_SCENE, n_frames=2), 81)
    H, W = frames.shape[2:]
    m5 = oracle.Model(blob5)
    assert [m5.exit_shape(k, H, W)[0] for k in range(1, 6)] == [8, 32, 64, 128, 256]
    assert [m5.exit_shape(k, H, W)[3] for k in range(1, 6)] == [4, 4, 8, 16, 32]
    assert m5.exit_shape(1, H, W)[1:3] == m5.exit_shape(2, H, W)[1:3]
    # exit 1's tensor is the max-pooled stem output, computed by the step functions
    w = split_blob(STEM5, blob5)
    x = oracle.maxpool3x3s2(oracle.conv2d(oracle.normalize(frames), w["stem.w"], w["stem.b"], stride=2, pad=3, relu=True))
    r1 = m5.detect(frames, 1, taps=["feat", "head_feat"])
    assert np.array_equal(r1["feat"], x) and np.array_equal(r1["head_feat"], x)
    assert (r1["labels"][:, 0] >= 1).all()
    # the same tensors under the four-exit numbering: drop exit 1's unit from the blob
    spec4 = replace(STEM5, n_exits=4, stem_exit=0)
    names4 = [n for n, _, _ in tensor_list(spec4)]
    w4 = {n: w[n if not n.startswith("e") else f"e{int(n[1]) + 1}{n[2:]}"] for n in names4}
    blob4 = make_blob(spec4, 5)
    for n, v in split_blob(spec4, blob4).items():
        v[...] = w4[n]
    m4 = oracle.Model(blob4)
    for k in (1, 2, 3, 4):
        a, b = m4.detect(frames, k), m5.detect(frames, k + 1)
        for key in ("boxes", "scores", "labels"):
            assert np.array_equal(a[key], b[key]), (k, key)
    # prefix property with the shifted numbering, and bounds
    full, stages = m5.backbone(frames, 5, stages=True)
    assert len(stages) == 4 and np.array_equal(full, stages[3])
    assert np.array_equal(m5.backbone(frames, 3), stages[1])
    with pytest.raises(ValueError):
        m5.detect(frames, 6)
    bad = blob5.copy()
    bad[:256].view(np.int32)[38] = 0                                   # five exits need the stem exit
    with pytest.raises(ValueError):
        oracle.Model(bad)
