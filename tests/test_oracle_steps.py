"""Pins of the CPU oracle's step functions against things that are not the oracle:
brute-force definitions in pure Python, closed forms, hand-computed values and
library routines (numpy / torch CPU in float64).  CPU only."""
import math

import numpy as np
import pytest
import torch

import oracle


# ------------------------------------------------------------------ conv / fc
def brute_conv(x, w, b, stride, pad):
    """7 nested loops, Python ints/floats: the definition of a zero-padded cross-correlation."""
    N, C, H, W = x.shape
    Co, _, kh, kw = w.shape
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    out = np.zeros((N, Co, Ho, Wo))
    for n in range(N):
        for co in range(Co):
            for oy in range(Ho):
                for ox in range(Wo):
                    s = float(b[co])
                    for ci in range(C):
                        for ky in range(kh):
                            for kx in range(kw):
                                iy, ix = oy * stride - pad + ky, ox * stride - pad + kx
                                if 0 <= iy < H and 0 <= ix < W:
                                    s += float(w[co, ci, ky, kx]) * float(x[n, ci, iy, ix])
                    out[n, co, oy, ox] = s
    return out


@pytest.mark.parametrize("k,stride,pad,H,W", [(7, 2, 3, 9, 11), (3, 1, 1, 6, 5), (3, 2, 1, 7, 8), (3, 2, 1, 8, 7),
                                              (1, 1, 0, 4, 5), (1, 2, 0, 5, 6)])
def test_conv_matches_brute_force_exactly_on_integers(k, stride, pad, H, W):
    rs = np.random.RandomState(k * 100 + stride * 10 + H)
    x = rs.randint(-4, 5, size=(2, 3, H, W)).astype(np.float32)
    w = rs.randint(-3, 4, size=(4, 3, k, k)).astype(np.float32)
    b = rs.randint(-2, 3, size=(4,)).astype(np.float32)
    got = oracle.conv2d(x, w, b, stride=stride, pad=pad)
    ref = brute_conv(x, w, b, stride, pad)
    assert got.shape == ref.shape
    assert np.array_equal(got.astype(np.float64), ref)       # integer sums: exact


def test_conv_residual_and_relu_order():
    # relu(conv + residual): the residual is added BEFORE the activation
    x = np.ones((1, 1, 2, 2), np.float32)
    w = np.full((1, 1, 1, 1), -3.0, np.float32)
    b = np.array([1.0], np.float32)
    res = np.array([[[[5.0, 1.0], [2.0, -7.0]]]], np.float32)
    got = oracle.conv2d(x, w, b, residual=res, relu=True)
    assert np.array_equal(got, np.array([[[[3.0, 0.0], [0.0, 0.0]]]], np.float32))
    got = oracle.conv2d(x, w, b, residual=res, relu=False)
    assert np.array_equal(got, np.array([[[[3.0, -1.0], [0.0, -9.0]]]], np.float32))


def test_conv_all_ones_counts_valid_taps():
    # all-ones input and kernel, zero padding: output = number of in-image taps
    x = np.ones((1, 2, 5, 6), np.float32)
    w = np.ones((1, 2, 3, 3), np.float32)
    got = oracle.conv2d(x, w, np.zeros(1, np.float32), stride=1, pad=1)[0, 0]
    ny = np.array([2, 3, 3, 3, 2])[:, None]
    nx = np.array([2, 3, 3, 3, 3, 2])[None, :]
    assert np.array_equal(got, (2 * ny * nx).astype(np.float32))


def test_conv_identity_kernel_and_1x1_is_matmul():
    rs = np.random.RandomState(0)
    x = rs.randn(2, 5, 4, 3).astype(np.float32)
    w = np.zeros((5, 5, 3, 3), np.float32)
    for c in range(5):
        w[c, c, 1, 1] = 1.0
    assert np.array_equal(oracle.conv2d(x, w, np.zeros(5, np.float32), pad=1), x)
    w1 = rs.randn(7, 5, 1, 1).astype(np.float32)
    b1 = rs.randn(7).astype(np.float32)
    got = oracle.conv2d(x, w1, b1)
    ref = np.einsum("oc,nchw->nohw", w1[:, :, 0, 0].astype(np.float64), x.astype(np.float64)) + b1[None, :, None, None]
    assert np.allclose(got, ref, rtol=0, atol=1e-6)
    assert np.array_equal(got, ref.astype(np.float32))     # double accumulation, rounded once


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 1, 3), (2, 3, 7), (2, 0, 1)])
def test_conv_matches_torch_float64(stride, pad, k):
    rs = np.random.RandomState(5)
    x = rs.randn(2, 6, 13, 10).astype(np.float32)
    w = rs.randn(8, 6, k, k).astype(np.float32)
    b = rs.randn(8).astype(np.float32)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     torch.from_numpy(b).double(), stride=stride, padding=pad).numpy()
    got = oracle.conv2d(x, w, b, stride=stride, pad=pad)
    assert got.shape == ref.shape
    assert np.max(np.abs(got - ref)) <= 2e-6 * np.max(np.abs(ref))


def test_fc_matches_numpy_float64():
    rs = np.random.RandomState(1)
    x = rs.randn(5, 33).astype(np.float32)
    w = rs.randn(9, 33).astype(np.float32)
    b = rs.randn(9).astype(np.float32)
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b
    assert np.array_equal(oracle.fc(x, w, b), ref.astype(np.float32))
    assert np.array_equal(oracle.fc(x, w, b, relu=True), np.maximum(ref, 0).astype(np.float32))
    # a transposed weight would fail this: non-square w
    assert oracle.fc(x, w, b).shape == (5, 9)


def test_bf16_rounding_known_values_and_torch():
    r = lambda v: float(oracle.lib().orc_round_bf16(v))
    assert r(1.0) == 1.0
    assert r(1.0 + 2.0 ** -8) == 1.0                       # tie -> even (mantissa ...0)
    assert r(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6       # tie -> even upwards
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7
    assert r(-0.0) == 0.0 and math.copysign(1, r(-0.0)) == -1
    rs = np.random.RandomState(2)
    x = (rs.randn(4000) * np.exp(rs.randn(4000) * 4)).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert np.array_equal(oracle.round_bf16(x), ref)


def test_bf16_mode_rounds_weights_and_output():
    x = np.array([[[[1.0]]]], np.float32)
    w = np.array([[[[1.0 + 3 * 2.0 ** -8]]]], np.float32)
    b = np.array([2.0 ** -9], np.float32)
    # weight -> 1 + 2^-6; + bias 2^-9 = 1.017578125 -> bf16: spacing 2^-7 -> 1.015625
    got = oracle.conv2d(x, w, b, bf16_weights=1, round_out=1)
    assert got.item() == 1.015625
    got = oracle.conv2d(x, w, b, bf16_weights=1, round_out=0)
    assert got.item() == np.float32(1.0 + 2.0 ** -6 + 2.0 ** -9)


def test_normalize():
    f = np.array([0, 114, 172, 255], np.uint8)
    got = oracle.normalize(f)
    assert np.array_equal(got, ((f.astype(np.float32) - np.float32(114)) / np.float32(58)))
    assert got[1] == 0.0 and got[2] == 1.0


# ------------------------------------------------------------------ maxpool
def test_maxpool_hand_cases():
    x = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    # windows centred at input (0,0),(0,2),(2,0),(2,2), 3x3, clipped to the image
    assert np.array_equal(oracle.maxpool3x3s2(x)[0, 0], np.array([[5, 7], [13, 15]], np.float32))
    # all-negative input: padding must never win
    xn = -np.ones((1, 1, 5, 5), np.float32) * 3
    assert np.array_equal(oracle.maxpool3x3s2(xn), -3 * np.ones((1, 1, 3, 3), np.float32))
    # odd size 5 -> 3 outputs; last window covers rows 3..4 only
    x5 = np.zeros((1, 1, 5, 5), np.float32)
    x5[0, 0, 4, 4] = 9
    assert oracle.maxpool3x3s2(x5)[0, 0, 2, 2] == 9 and oracle.maxpool3x3s2(x5)[0, 0, 1, 1] == 0


def test_maxpool_matches_torch():
    rs = np.random.RandomState(3)
    x = rs.randn(2, 3, 9, 12).astype(np.float32)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x), 3, 2, 1).numpy()
    assert np.array_equal(oracle.maxpool3x3s2(x), ref)


# ------------------------------------------------------------------ top-k
def test_topk_is_prefix_of_stable_sort_with_ties():
    rs = np.random.RandomState(4)
    s = rs.randint(-3, 4, size=500).astype(np.float32)         # many ties
    s[10] = -0.0
    s[20] = 0.0
    order = np.lexsort((np.arange(s.size), -s.astype(np.float64)))  # score desc, index asc
    for k in (1, 7, 64, 499, 500):
        idx, val = oracle.topk(s, k)
        assert np.array_equal(idx, order[:k].astype(np.int32))
        assert np.array_equal(val, s[order[:k]])
    idx, _ = oracle.topk(s, 900)                               # k > n returns all
    assert idx.size == 500 and np.array_equal(idx, order.astype(np.int32))


def test_topk_negative_zero_equals_positive_zero():
    s = np.array([0.0, -0.0, 0.0, -1.0, -0.0], np.float32)
    idx, _ = oracle.topk(s, 4)
    assert list(idx) == [0, 1, 2, 4]


# ------------------------------------------------------------------ NMS
def iou64(a, b):
    iw = max(0.0, min(a[2], b[2]) - max(a[0], b[0]))
    ih = max(0.0, min(a[3], b[3]) - max(a[1], b[1]))
    inter = iw * ih
    uni = (a[2] - a[0]) * (a[3] - a[1]) + (b[2] - b[0]) * (b[3] - b[1]) - inter
    return inter / uni if uni > 0 else 0.0


def brute_nms(boxes, thr, max_keep, labels=None):
    """The definition: i survives iff no surviving j < i (same label) has IoU > thr."""
    n = len(boxes)
    alive = [True] * n
    keep = []
    for i in range(n):
        if not alive[i]:
            continue
        if len(keep) == max_keep:
            break
        keep.append(i)
        for j in range(i + 1, n):
            if labels is not None and labels[i] != labels[j]:
                continue
            if iou64(boxes[i].astype(np.float64), boxes[j].astype(np.float64)) > thr:
                alive[j] = False
    return keep


def rand_boxes(rs, n, size=100.0):
    # coordinates on a 1/8 grid: areas, intersections and unions are exact in fp32 and fp64
    x1 = np.round(rs.rand(n) * size * 8) / 8
    y1 = np.round(rs.rand(n) * size * 8) / 8
    w = np.round((2 + rs.rand(n) * size / 2) * 8) / 8
    h = np.round((2 + rs.rand(n) * size / 2) * 8) / 8
    return np.stack([x1, y1, x1 + w, y1 + h], 1).astype(np.float32)


@pytest.mark.parametrize("thr", [0.3, 0.5, 0.7])
def test_nms_matches_quadratic_definition(thr):
    rs = np.random.RandomState(int(thr * 10))
    b = rand_boxes(rs, 300)
    assert list(oracle.nms(b, thr)) == brute_nms(b, thr, 300)
    assert list(oracle.nms(b, thr, max_keep=17)) == brute_nms(b, thr, 17)
    lab = rs.randint(1, 4, size=300).astype(np.int32)
    assert list(oracle.nms(b, thr, labels=lab)) == brute_nms(b, thr, 300, lab)


def test_iou_identities():
    a = np.array([1, 2, 5, 7], np.float32)
    b = np.array([5, 2, 9, 7], np.float32)                    # touching: zero overlap
    c = np.array([3, 2, 7, 7], np.float32)                    # half of a: inter 10, union 30
    assert oracle.iou_over(a, a, 0.999) and not oracle.iou_over(a, a, 1.0)   # IoU(a,a) = 1, strict >
    assert not oracle.iou_over(a, b, 0.0)                     # disjoint: inter 0 is not > 0
    assert oracle.iou_over(a, c, 0.33) and not oracle.iou_over(a, c, 0.34)
    assert oracle.iou_over(a, c, 0.33) == oracle.iou_over(c, a, 0.33)
    z = np.zeros(4, np.float32)
    assert not oracle.iou_over(z, z, 0.0)                     # empty union never overlaps


def test_nms_special_thresholds_and_duplicates():
    rs = np.random.RandomState(9)
    b = rand_boxes(rs, 50)
    assert list(oracle.nms(b, 1.0)) == list(range(50))        # nothing exceeds IoU 1
    k0 = list(oracle.nms(b, 0.0))                             # survivors pairwise disjoint
    for i in k0:
        for j in k0:
            if i < j:
                assert iou64(b[i], b[j]) == 0.0
    d = np.stack([b[0], b[1], b[0], b[0]])
    assert 0 in oracle.nms(d, 0.5) and 2 not in oracle.nms(d, 0.5) and 3 not in oracle.nms(d, 0.5)


def test_per_class_nms_is_independent_nms_per_label():
    rs = np.random.RandomState(11)
    b = rand_boxes(rs, 120)
    lab = rs.randint(1, 5, size=120).astype(np.int32)
    joint = set(oracle.nms(b, 0.5, labels=lab).tolist())
    sep = set()
    for c in range(1, 5):
        ids = np.nonzero(lab == c)[0]
        sep |= set(ids[oracle.nms(b[ids], 0.5)].tolist())
    assert joint == sep


# ------------------------------------------------------------------ anchors / decoding
def test_anchor_and_decode_closed_forms(tiny):
    from thia_synth import CONFIGS
    from conftest import get_blob
    cfg = CONFIGS[2]
    # only the header matters for anchors: build a header-only model via the tiny blob is not
    # possible (sizes differ), so use config 1 (sizes 32/64/128, ratio 1) and check ratios below
    _, blob, _ = tiny
    m = oracle.Model(blob)
    Wk, stride, A = 32, 4, 3
    for (x, y, a) in [(0, 0, 0), (5, 7, 1), (31, 31, 2)]:
        i = (y * Wk + x) * A + a
        cx, cy, w, h = m.anchor(i, Wk, stride)
        size = (32.0, 64.0, 128.0)[a]
        assert (cx, cy) == ((x + 0.5) * stride, (y + 0.5) * stride)
        assert w == size and h == size
        # zero deltas: proposal = anchor clipped to the image
        box, ok = oracle.decode([cx, cy, w, h], [0, 0, 0, 0], 128, 128)
        exp = np.clip([cx - size / 2, cy - size / 2, cx + size / 2, cy + size / 2], 0, 128).astype(np.float32)
        assert ok and np.array_equal(box, exp)


def test_anchor_ratios_preserve_area():
    from thia_synth import ModelSpec, make_blob
    from dataclasses import replace
    spec = ModelSpec(precision=0, n_exits=1, blocks=(1, 0, 0, 0), has_lateral=0, fc_dim=8, n_classes=2,
                     sizes=(32.0, 64.0), ratios=(0.5, 1.0, 2.0))
    m = oracle.Model(make_blob(spec, 1))
    Wk, stride, A = 10, 4, 6
    for a in range(A):
        size = (32.0, 64.0)[a // 3]                            # size-major ordering
        r = (0.5, 1.0, 2.0)[a % 3]
        cx, cy, w, h = m.anchor((3 * Wk + 4) * A + a, Wk, stride)
        assert (cx, cy) == (18.0, 14.0)
        assert abs(w * h - size * size) <= 1e-3 * size * size   # area preserved
        assert abs(h / w - r) <= 1e-6 * r                      # ratio = h / w
        assert abs(w - size / math.sqrt(r)) <= 1e-5 * size


def test_decode_shift_scale_clamp_clip_and_empty():
    anc = [50.0, 40.0, 20.0, 10.0]
    box, ok = oracle.decode(anc, [1.0, 0.0, 0.0, 0.0], 1000, 1000)       # dx = 1 shifts by w
    assert ok and np.array_equal(box, np.array([60, 35, 80, 45], np.float32))
    box, _ = oracle.decode(anc, [0.0, -2.0, 0.0, 0.0], 1000, 1000)       # dy = -2 shifts by -2h
    assert np.array_equal(box, np.array([40, 15, 60, 25], np.float32))
    box, _ = oracle.decode(anc, [0.0, 0.0, math.log(2.0), 0.0], 1000, 1000)  # dw = ln 2 doubles w
    assert np.allclose(box, [30, 35, 70, 45], atol=1e-4)
    box, _ = oracle.decode(anc, [0.0, 0.0, 0.0, math.log(3.0)], 1000, 1000)
    assert np.allclose(box, [40, 25, 60, 55], atol=1e-4)
    big, _ = oracle.decode([5000.0, 40.0, 20.0, 10.0], [0.0, 0.0, 50.0, 0.0], 1e9, 1e9)         # clamp at ln(1000/16)
    assert np.isclose(big[2] - big[0], 20.0 * 1000.0 / 16.0, rtol=1e-5)
    box, ok = oracle.decode(anc, [0.0, 0.0, 0.0, 0.0], 55, 42)           # clip to [0,W] x [0,H]
    assert ok and np.array_equal(box, np.array([40, 35, 55, 42], np.float32))
    box, ok = oracle.decode(anc, [10.0, 0.0, 0.0, 0.0], 55, 42)          # pushed outside: empty
    assert not ok and box[0] == box[2] == 55
    box, ok = oracle.decode(anc, [0.0, 0.0, -20.0, 0.0], 100, 100)       # collapsed width
    assert not ok


# ------------------------------------------------------------------ ROIAlign
def test_roialign_constant_map():
    f = np.full((3, 9, 11), 2.5, np.float32)
    rois = np.array([[4, 4, 30, 20], [0, 0, 44, 36], [10.3, 7.7, 12.1, 9.2]], np.float32)
    out = oracle.roialign(f, rois, stride=4)
    assert out.shape == (3, 3, 7, 7) and np.allclose(out, 2.5, atol=1e-6)


def test_roialign_linear_ramp_is_reproduced_at_bin_centres():
    Hk, Wk, stride = 20, 24, 8
    yy, xx = np.meshgrid(np.arange(Hk), np.arange(Wk), indexing="ij")
    # texel j has centre j + 0.5 (feature units): value = 3*X + 5*Y + 1 at the texel centre
    f = (3.0 * (xx + 0.5) + 5.0 * (yy + 0.5) + 1.0).astype(np.float32)[None]
    roi = np.array([[40.0, 24.0, 120.0, 108.0]], np.float32)      # interior, feature coords 5..15, 3..13.5
    out = oracle.roialign(f, roi, stride=stride)[0, 0]
    x1, y1, x2, y2 = roi[0] / stride
    bw, bh = (x2 - x1) / 7, (y2 - y1) / 7
    for ph in range(7):
        for pw in range(7):
            cx, cy = x1 + (pw + 0.5) * bw, y1 + (ph + 0.5) * bh   # mean of symmetric samples = centre
            assert abs(out[ph, pw] - (3 * cx + 5 * cy + 1)) < 1e-4


def test_roialign_hand_computed_2x2():
    # 2x2 map, stride 1, one bin (P=1), 2x2 samples.  ROI = [0.5,0.5,1.5,1.5]:
    # samples at (0.75|1.25, 0.75|1.25) -> u,v in {0.25, 0.75}
    f = np.array([[[1.0, 2.0], [3.0, 5.0]]], np.float32)
    roi = np.array([[0.5, 0.5, 1.5, 1.5]], np.float32)
    out = oracle.roialign(f, roi, stride=1, P=1, S=2)

    def bil(u, v):
        return (1 - v) * ((1 - u) * 1 + u * 2) + v * ((1 - u) * 3 + u * 5)
    exp = np.mean([bil(u, v) for u in (0.25, 0.75) for v in (0.25, 0.75)])
    assert abs(out.item() - exp) < 1e-6 and abs(exp - 2.75) < 1e-12
    # samples left of the first texel centre clamp to it; beyond one texel outside contribute 0
    roi = np.array([[-4.0, 0.0, -2.0, 1.0]], np.float32)      # u in [-4.5,-2.5] < -1: all zero
    assert oracle.roialign(f, roi, stride=1, P=1, S=2).item() == 0.0
    roi = np.array([[0.0, 0.0, 0.5, 0.5]], np.float32)        # u,v = -0.375, -0.125 -> clamp to texel (0,0)
    assert oracle.roialign(f, roi, stride=1, P=1, S=2).item() == 1.0


def test_roialign_channel_and_bin_layout():
    # channel c holds c; a map varying only in x must vary only along pw
    f = np.stack([np.full((8, 8), c, np.float32) for c in range(4)])
    out = oracle.roialign(f, np.array([[2, 2, 20, 20]], np.float32), stride=4)
    assert np.allclose(out[0, :, 3, 3], np.arange(4))
    g = np.tile(np.arange(8, dtype=np.float32)[None, None, :], (1, 8, 1))
    o = oracle.roialign(g, np.array([[4, 4, 28, 28]], np.float32), stride=4)[0, 0]
    assert np.allclose(o, o[0:1, :]) and np.all(np.diff(o[0]) > 0)


# ------------------------------------------------------------------ softmax / selection
def test_softmax_invariants():
    rs = np.random.RandomState(6)
    x = (rs.randn(20, 8) * 5).astype(np.float32)
    p = oracle.softmax(x)
    assert np.allclose(p.sum(1), 1.0, atol=1e-6) and np.all(p > 0)
    assert np.allclose(oracle.softmax(x + 100.0), p, atol=1e-6)
    ref = torch.softmax(torch.from_numpy(x).double(), 1).numpy()
    assert np.allclose(p, ref, atol=1e-7)
    big = np.array([[1000.0, 0.0, -1000.0]], np.float32)       # no overflow
    assert np.allclose(oracle.softmax(big), [[1, 0, 0]])


def test_select_detections_definition():
    rs = np.random.RandomState(7)
    R, Kc, D = 40, 4, 12
    scores = rs.rand(R, Kc).astype(np.float32) * 0.3
    boxes = np.stack([rand_boxes(rs, R) for _ in range(Kc)], 1)   # [R,Kc,4]
    boxes[3, 2] = [5, 5, 5, 9]                                    # empty box is never a candidate
    scores[3, 2] = 0.9
    scores[4, 0] = 0.99                                           # background never emitted
    ob, osc, ol, n = oracle.select_detections(scores, boxes, 0.05, 0.5, D)
    cand = [(-(scores[r, c].astype(np.float64)), r * Kc + c) for r in range(R) for c in range(1, Kc)
            if scores[r, c] > np.float32(0.05) and (r, c) != (3, 2)]
    cand.sort()
    cb = np.array([boxes.reshape(-1, 4)[j] for _, j in cand])
    cl = np.array([j % Kc for _, j in cand])
    keep = brute_nms(cb, 0.5, D, cl)
    assert n == len(keep) == D
    assert np.array_equal(ol[:n], cl[keep]) and np.array_equal(ob[:n], cb[keep])
    assert np.array_equal(osc[:n], np.array([-cand[k][0] for k in keep], np.float32))
    assert np.all(np.diff(osc[:n]) <= 0)
    # fewer than D: padded with score 0, label -1, box 0
    ob, osc, ol, n = oracle.select_detections(scores[:2], boxes[:2], 0.25, 0.5, D)
    assert n < D and np.all(ol[n:] == -1) and np.all(osc[n:] == 0) and np.all(ob[n:] == 0)
