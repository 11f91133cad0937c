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
