"""Helpers for the GPU parity tests (layout conversion, error measures, cached models)."""
import numpy as np
import torch

from conftest import get_blob
from thia_synth import CONFIGS, ModelSpec, SceneSpec, make_frames

_models = {}

# Reduced-depth bf16 detector with the real ResNet-50 channel widths (the kernels need
# channel counts that are multiples of 64), small enough for the CPU oracle.
MINI_BF16 = ModelSpec(precision=1, blocks=(1, 1, 1, 1), fc_dim=128, pre_nms=1000, post_nms=300, n_classes=8)
MINI_FP32 = ModelSpec(precision=0, blocks=(1, 1, 1, 1), fc_dim=128, pre_nms=300, post_nms=100, n_classes=5)


def gpu_model(spec, seed):
    """(Model on cuda:0, blob) cached per spec."""
    from paper_2102_08481_amd import thia_load_model
    key = (spec.header(), seed)
    if key not in _models:
        blob = get_blob(spec, seed)
        _models[key] = (thia_load_model(blob, spec.n_exits), blob)
    return _models[key]


def relerr(a, b):
    """max |a - b| / max |b| (per tensor, normalised by the reference's max-abs)."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-30)) if a.size else 0.0


def to_dev(x, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def nchw_to_nhwc(x):
    return np.ascontiguousarray(np.transpose(x, (0, 2, 3, 1)))


def nhwc_to_nchw(x):
    return np.ascontiguousarray(np.transpose(x, (0, 3, 1, 2)))


def box_iou(a, b):
    """IoU matrix of [n,4] and [m,4] (float64)."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    iw = np.clip(np.minimum(a[:, None, 2], b[None, :, 2]) - np.maximum(a[:, None, 0], b[None, :, 0]), 0, None)
    ih = np.clip(np.minimum(a[:, None, 3], b[None, :, 3]) - np.maximum(a[:, None, 1], b[None, :, 1]), 0, None)
    inter = iw * ih
    ua = (a[:, 2] - a[:, 0]) * (a[:, 3] - a[:, 1])
    ub = (b[:, 2] - b[:, 0]) * (b[:, 3] - b[:, 1])
    return inter / np.maximum(ua[:, None] + ub[None, :] - inter, 1e-30)


def match_fraction(gb, gl, rb, rl, iou_thr=0.99):
    """Fraction of reference detections (label >= 0) matched one-to-one by a GPU detection of the
    same label with IoU >= iou_thr, and the symmetric fraction of GPU detections; returns the minimum."""
    rv, gv = rl >= 0, gl >= 0
    nr, ng = int(rv.sum()), int(gv.sum())
    if nr == 0 and ng == 0:
        return 1.0, 0
    if nr == 0 or ng == 0:
        return 0.0, max(nr, ng)
    iou = box_iou(rb[rv], gb[gv])
    same = rl[rv][:, None] == gl[gv][None, :]
    ok = (iou >= iou_thr) & same
    used, hit = set(), 0
    for i in range(nr):
        for j in np.argsort(-iou[i]):
            if ok[i, j] and j not in used:
                used.add(j)
                hit += 1
                break
    return hit / max(nr, ng), max(nr, ng)


def chain_check(m, blob, spec, H, W, ep, n_frames, frame, gb, gs, gl, step_tol):
    """Stage-by-stage check INSIDE a full run: every stage of frame `frame` is recomputed by the
    oracle's step functions from the GPU's own upstream tensors (taps).  Discrete stages (top-k
    indices, NMS keeps, final selection) must then agree bit-exactly; continuous stages within
    step_tol (per tensor, max-abs normalised).  This is immune to the rank-order sensitivity of
    random-init scores, because both sides take each decision on identical numbers."""
    import oracle
    from thia_synth import split_blob
    orc = oracle.Model(blob)
    bf = spec.precision
    Ck, Hk, Wk, stride = orc.exit_shape(ep, H, W)
    Ch = spec.head_ch if spec.has_lateral else Ck
    A, pre, post, P, Kc, D = spec.n_anchors, spec.pre_nms, spec.post_nms, spec.pool, spec.n_classes, spec.max_det
    nA = Hk * Wk * A
    f = frame
    tap = lambda name, shape: m.tap(name).reshape((n_frames,) + shape)[f]
    logits, deltas = tap("rpn_logits", (nA,)), tap("rpn_deltas", (nA, 4))
    # top-k on the GPU's own logits
    ridx, _ = oracle.topk(logits, pre)
    gidx = tap("topk_idx", (pre,))
    assert np.array_equal(gidx[:len(ridx)], ridx) and np.all(gidx[len(ridx):] == -1), "top-k indices"
    # decode + clip + drop empties
    ref = []
    for i in ridx:
        bx, ok = oracle.decode(orc.anchor(i, Wk, stride), deltas[i], W, H)
        if ok:
            ref.append(bx)
    ref = np.array(ref, np.float32).reshape(-1, 4)
    pn = int(m.tap("prop_n")[f])
    pbox = tap("prop_boxes", (pre, 4))
    assert pn == len(ref), ("proposal count", pn, len(ref))
    assert np.max(np.abs(pbox[:pn] - ref)) <= 1e-5 * 4 * max(H, W), "decoded proposals"
    # NMS on the GPU's own proposals
    keep = oracle.nms(pbox[:pn], spec.rpn_nms_thr, post)
    rn = int(m.tap("roi_n")[f])
    rois = tap("rois", (post, 4))
    assert rn == len(keep) and np.array_equal(rois[:rn], pbox[keep]) and np.all(rois[rn:] == 0), "proposal NMS"
    # ROIAlign on the GPU's own head feature map and ROIs
    hf = np.ascontiguousarray(np.transpose(tap("head_feat", (Hk, Wk, Ch)), (2, 0, 1)))
    rf_ref = oracle.roialign(hf, rois[:rn], stride, P, spec.sampling, round_out=bf)          # [rn, Ch, P, P]
    rf = tap("roi_feat", (post, P * P, Ch))[:rn]
    rf_nchw = np.ascontiguousarray(np.transpose(rf, (0, 2, 1))).reshape(rn, Ch * P * P)
    e_roi = relerr(rf_nchw, rf_ref.reshape(rn, -1))
    assert e_roi <= step_tol, ("roialign", e_roi)
    # box head on the GPU's own ROI features
    w = split_blob(spec, blob)
    e = f"e{ep}"
    h1 = oracle.fc(rf_nchw, w[e + ".fc1.w"], w[e + ".fc1.b"], relu=True, bf16_weights=bf, round_out=bf)
    h2 = oracle.fc(h1, w[e + ".fc2.w"], w[e + ".fc2.b"], relu=True, bf16_weights=bf, round_out=bf)
    cl_ref = oracle.fc(h2, w[e + ".cls.w"], w[e + ".cls.b"], bf16_weights=bf)
    bd_ref = oracle.fc(h2, w[e + ".box.w"], w[e + ".box.b"], bf16_weights=bf)
    cl, bd = tap("cls_logits", (post, Kc))[:rn], tap("box_deltas", (post, 4 * Kc))[:rn]
    head_tol = 4 * step_tol if bf else step_tol      # two bf16-rounded FC layers in between
    e_cl, e_bd = relerr(cl, cl_ref), relerr(bd, bd_ref)
    assert e_cl <= head_tol and e_bd <= head_tol, ("box head", e_cl, e_bd)
    # scores and per-class boxes from the GPU's own logits / deltas
    cs, cb = tap("cand_scores", (post, Kc))[:rn], tap("cand_boxes", (post, Kc, 4))[:rn]
    assert np.max(np.abs(cs - oracle.softmax(cl))) <= 1e-5, "softmax"
    for r in (0, rn // 2, rn - 1):
        q = rois[r]
        anc = [q[0] + np.float32(0.5) * (q[2] - q[0]), q[1] + np.float32(0.5) * (q[3] - q[1]), q[2] - q[0], q[3] - q[1]]
        for c in range(1, Kc):
            bx, _ = oracle.decode(anc, bd[r, 4 * c:4 * c + 4], W, H)
            assert np.max(np.abs(bx - cb[r, c])) <= 1e-5 * 4 * max(H, W), "class boxes"
    # final selection on the GPU's own candidate scores / boxes
    ob, osc, ol, nd = oracle.select_detections(cs, cb, spec.score_thr, spec.det_nms_thr, D)
    assert int(m.tap("det_n")[f]) == nd, "detection count"
    assert np.array_equal(gl[f].cpu().numpy(), ol) and np.array_equal(gb[f].cpu().numpy(), ob) \
        and np.array_equal(gs[f].cpu().numpy(), osc), "final selection"
    return dict(roialign=e_roi, cls=e_cl, box=e_bd, n_rois=rn, n_det=nd)
