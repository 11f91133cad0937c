"""Step-level parity on the GPU: every kernel of the path is fed the ORACLE's upstream
tensor through the C ABI (thia_op_*) and compared with the oracle's downstream tensor.
Orderings, indices and NMS keeps must be bit-exact; floating-point tensors within the
tolerance written next to each check."""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import MINI_BF16, MINI_FP32, gpu_model, nchw_to_nhwc, nhwc_to_nchw, relerr, to_dev
from thia_synth import CONFIGS, SceneSpec, make_frames

pytestmark = pytest.mark.gpu

# fp32 tensors: fp32 MFMA accumulation against double accumulation -> 1e-4 (the stated bar);
# bf16 tensors against the oracle in bf16-storage mode: the single bf16 rounding of an output may
# go the other way where the fp32 and the double sum straddle a rounding boundary, i.e. one bf16
# ulp; for an element just below a power of two that is 2^-7 of the tensor's max-abs.
TOL_F32 = 1e-4
TOL_BF16_STEP = 2.0 ** -7


def _model(precision):
    return gpu_model(MINI_BF16 if precision else MINI_FP32, 0xBEEF + 50 + precision)


def _bf16(x):
    return torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16).float().numpy()


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("case", [
    dict(n=2, H=13, W=17, Cin=64, Cout=64, k=1, stride=1, pad=0),        # narrow tile, ragged M (442 rows)
    dict(n=3, H=20, W=23, Cin=64, Cout=256, k=1, stride=1, pad=0),       # several M tiles + tail
    dict(n=2, H=19, W=21, Cin=64, Cout=64, k=3, stride=1, pad=1),        # 3x3 borders
    dict(n=2, H=19, W=22, Cin=128, Cout=128, k=3, stride=2, pad=1),      # strided 3x3, odd/even sizes
    dict(n=2, H=17, W=16, Cin=256, Cout=512, k=1, stride=2, pad=0),      # strided 1x1 shortcut
    dict(n=1, H=9, W=11, Cin=256, Cout=75, k=1, stride=1, pad=0),        # Cout not a multiple of 4 (scalar epilogue)
    dict(n=300, H=1, W=1, Cin=1024, Cout=40, k=1, stride=1, pad=0),      # FC-shaped, narrow
    dict(n=1, H=1, W=1, Cin=64, Cout=64, k=1, stride=1, pad=0),          # single row
    dict(n=2, H=11, W=9, Cin=128, Cout=128, k=1, stride=1, pad=0),       # two K steps
    dict(n=2, H=11, W=9, Cin=192, Cout=256, k=1, stride=1, pad=0),       # three K steps (odd count)
    dict(n=2, H=161, W=159, Cin=64, Cout=256, k=3, stride=1, pad=1),     # 256x256 tile kernel, ragged M, 3x3 borders
    dict(n=2, H=161, W=160, Cin=512, Cout=512, k=1, stride=1, pad=0),    # 256x256 tile kernel, two N tiles
    dict(n=400, H=1, W=1, Cin=8192, Cout=256, k=1, stride=1, pad=0),     # very long K, few tiles: 192-pixel tile kernel, ragged M
])
def test_conv_op_matches_oracle(precision, case):
    m, _ = _model(precision)
    c = dict(case)
    rs = np.random.RandomState(c["H"] * 31 + c["Cout"])
    x = rs.randn(c["n"], c["Cin"], c["H"], c["W"]).astype(np.float32)
    w = (rs.randn(c["Cout"], c["Cin"], c["k"], c["k"]) * np.sqrt(2.0 / (c["Cin"] * c["k"] ** 2))).astype(np.float32)
    b = rs.randn(c["Cout"]).astype(np.float32) * 0.1
    if precision:
        x = _bf16(x)
    Ho = (c["H"] + 2 * c["pad"] - c["k"]) // c["stride"] + 1
    Wo = (c["W"] + 2 * c["pad"] - c["k"]) // c["stride"] + 1
    res = rs.randn(c["n"], c["Cout"], Ho, Wo).astype(np.float32)
    if precision:
        res = _bf16(res)
    xd = to_dev(nchw_to_nhwc(x), m.elem)
    rd = to_dev(nchw_to_nhwc(res), m.elem)
    for (use_res, relu, out_f32) in [(False, False, False), (True, True, False), (False, False, True)]:
        ref = oracle.conv2d(x, w, b, stride=c["stride"], pad=c["pad"], residual=res if use_res else None, relu=relu,
                            bf16_weights=precision, round_out=int(bool(precision) and not out_f32))
        got = m.op_conv(xd, w, b, stride=c["stride"], pad=c["pad"], residual=rd if use_res else None, relu=relu, out_f32=out_f32)
        torch.cuda.synchronize()
        got = nhwc_to_nchw(got.float().cpu().numpy())
        assert got.shape == ref.shape
        tol = TOL_BF16_STEP if (precision and not out_f32) else TOL_F32
        assert relerr(got, ref) <= tol, (case, use_res, relu, out_f32, relerr(got, ref))


def test_bf16_output_rounding_is_nearest_even_bit_exact():
    """The kernels round fp32 results to bf16 with the hardware conversion; the oracle with integer
    arithmetic.  A convolution with zero weights returns round(bias): ties both ways, values next to
    ties, bf16 and fp32 subnormals, the largest finite values and signed zeros must agree bit for bit."""
    m, _ = _model(1)
    bits = [0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF, 0x3F817FFF, 0x3F818001, 0x00000001, 0x00008000, 0x00018000, 0x007FFFFF,
            0x00800000, 0x7F7F0000, 0x7F7F7FFF, 0x7F7E8000, 0x80000000, 0x00000000, 0xBF808000, 0xBF818000, 0x80008001, 0xC2F6E979]
    rs = np.random.RandomState(7)
    bits = np.array(bits + list(rs.randint(0, 2 ** 32, 64 - len(bits), dtype=np.uint64)), dtype=np.uint32)
    bits = np.where((bits & 0x7F800000) == 0x7F800000, bits & 0x3FFFFFFF, bits).astype(np.uint32)   # no inf / nan
    b = bits.view(np.float32)
    x = np.zeros((1, 64, 3, 5), np.float32)
    w = np.zeros((64, 64, 1, 1), np.float32)
    ref = oracle.conv2d(x, w, b, bf16_weights=1, round_out=1)
    got = m.op_conv(to_dev(nchw_to_nhwc(x), m.elem), w, b)
    torch.cuda.synchronize()
    got = nhwc_to_nchw(got.float().cpu().numpy())
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), np.flatnonzero(got.view(np.uint32) != ref.view(np.uint32))[:8]


@pytest.mark.parametrize("variant", [(64, False), (64, True), (128, False)])
@pytest.mark.parametrize("shape", [(2, 21, 37), (1, 5, 7), (3, 41, 50), (1, 8, 16)])
def test_bottleneck_op_matches_oracle(shape, variant):
    """Single-kernel bottleneck (identity and projection shortcut) against the oracle's convolutions in
    bf16 storage mode.  Three roundings are chained, so besides the one-ulp flip of the output (2^-7, see
    above) a flipped intermediate element can move an output by a fraction of an ulp more: the bound is
    2^-6, and the share of elements that differ at all is bounded too."""
    m, _ = _model(1)
    n, H, W = shape
    wd, first = variant
    cin = wd if first else 4 * wd
    rs = np.random.RandomState(H * 131 + W + int(first) + wd)
    x = _bf16(np.abs(rs.randn(n, cin, H, W)).astype(np.float32))
    w1 = (rs.randn(wd, cin, 1, 1) * np.sqrt(2.0 / cin)).astype(np.float32)
    w2 = (rs.randn(wd, wd, 3, 3) * np.sqrt(2.0 / (9 * wd))).astype(np.float32)
    w3 = (rs.randn(4 * wd, wd, 1, 1) * np.sqrt(2.0 / wd)).astype(np.float32)
    ws = (rs.randn(4 * wd, cin, 1, 1) * np.sqrt(1.0 / cin)).astype(np.float32)
    b1, b2, b3, bs = [(rs.randn(c) * 0.1).astype(np.float32) for c in (wd, wd, 4 * wd, 4 * wd)]
    t1 = oracle.conv2d(x, w1, b1, relu=True, bf16_weights=1, round_out=1)
    t2 = oracle.conv2d(t1, w2, b2, pad=1, relu=True, bf16_weights=1, round_out=1)
    if first:
        sc = oracle.conv2d(x, ws, bs, bf16_weights=1, round_out=0)      # the projection is not rounded before the sum
        ref = oracle.conv2d(t2, w3, b3, residual=sc, relu=True, bf16_weights=1, round_out=1)
        got = m.op_bottleneck(to_dev(nchw_to_nhwc(x), m.elem), w1, b1, w2, b2, w3, b3, ws, bs)
    else:
        ref = oracle.conv2d(t2, w3, b3, residual=x, relu=True, bf16_weights=1, round_out=1)
        got = m.op_bottleneck(to_dev(nchw_to_nhwc(x), m.elem), w1, b1, w2, b2, w3, b3)
    torch.cuda.synchronize()
    got = nhwc_to_nchw(got.float().cpu().numpy())
    assert got.shape == ref.shape
    differ = float(np.mean(got != ref))
    assert relerr(got, ref) <= 2.0 ** -6, (shape, relerr(got, ref), differ)
    assert differ <= 0.02, (shape, differ)


@pytest.mark.parametrize("tail_n,relu", [(128, True), (256, False)])
@pytest.mark.parametrize("shape", [(2, 21, 37), (1, 5, 7), (1, 8, 16)])
def test_bottleneck_tail_layer_matches_oracle(shape, tail_n, relu):
    """The 1x1 layer applied by the block to its own output tile (next stage's first 1x1 with ReLU, or an exit's lateral
    without): the block output is unchanged by the extra phase, and the tail equals the oracle's 1x1 convolution of that
    very output (bf16 storage) up to one-ulp flips of the rounded result."""
    m, _ = _model(1)
    n, H, W = shape
    wd = 64
    rs = np.random.RandomState(H * 17 + W + tail_n)
    x = _bf16(np.abs(rs.randn(n, 4 * wd, H, W)).astype(np.float32))
    w1 = (rs.randn(wd, 4 * wd, 1, 1) * np.sqrt(2.0 / (4 * wd))).astype(np.float32)
    w2 = (rs.randn(wd, wd, 3, 3) * np.sqrt(2.0 / (9 * wd))).astype(np.float32)
    w3 = (rs.randn(4 * wd, wd, 1, 1) * np.sqrt(2.0 / wd)).astype(np.float32)
    wt = (rs.randn(tail_n, 4 * wd, 1, 1) * np.sqrt(2.0 / (4 * wd))).astype(np.float32)
    b1, b2, b3, bt = [(rs.randn(c) * 0.1).astype(np.float32) for c in (wd, wd, 4 * wd, tail_n)]
    xd = to_dev(nchw_to_nhwc(x), m.elem)
    y0 = m.op_bottleneck(xd, w1, b1, w2, b2, w3, b3)
    y, z = m.op_bottleneck_tail(xd, w1, b1, w2, b2, w3, b3, wt, bt, relu)
    torch.cuda.synchronize()
    assert torch.equal(y, y0)
    yh = nhwc_to_nchw(y.float().cpu().numpy())
    ref = oracle.conv2d(yh, wt, bt, relu=relu, bf16_weights=1, round_out=1)
    got = nhwc_to_nchw(z.float().cpu().numpy())
    assert got.shape == ref.shape == (n, tail_n, H, W)
    assert relerr(got, ref) <= 2.0 ** -7, relerr(got, ref)
    assert float(np.mean(got != ref)) <= 0.02


def test_bottleneck_op_rejects_unsupported():
    from paper_2102_08481_amd import ThiaError
    m, _ = _model(1)
    x = torch.zeros((1, 8, 8, 128), dtype=torch.bfloat16, device="cuda")
    z = lambda *s: np.zeros(s, np.float32)
    with pytest.raises(ThiaError) as e:
        m.op_bottleneck(x, z(32, 128, 1, 1), z(32), z(32, 32, 3, 3), z(32), z(128, 32, 1, 1), z(128))
    assert e.value.code == -3
    with pytest.raises(ThiaError) as e:       # the 128-wide variant has no projection form
        m.op_bottleneck(x, z(128, 128, 1, 1), z(128), z(128, 128, 3, 3), z(128), z(512, 128, 1, 1), z(512), z(512, 128, 1, 1), z(512))
    assert e.value.code == -3
    m32, _ = _model(0)
    with pytest.raises(ThiaError):
        m32.op_bottleneck(torch.zeros((1, 8, 8, 256), dtype=torch.float32, device="cuda"), z(64, 256, 1, 1), z(64), z(64, 64, 3, 3), z(64),
                          z(256, 64, 1, 1), z(256))


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("size", [(70, 93), (64, 128), (131, 252), (33, 37)])
def test_stem_op_matches_oracle(precision, size):
    """Normalisation + 7x7 stem + ReLU + 3x3 max-pool (one kernel for bf16 models): odd and even sizes,
    widths that are and are not multiples of 4, several tiles with ragged right and bottom edges."""
    m, blob = _model(precision)
    spec = MINI_BF16 if precision else MINI_FP32
    from thia_synth import split_blob
    w = split_blob(spec, blob)
    frames = make_frames(SceneSpec(size[0], size[1], 3, 3, 6, 8, 40), 5)
    x = oracle.normalize(frames, spec.mean, spec.std, bf16=precision)
    y = oracle.conv2d(x, w["stem.w"], w["stem.b"], stride=2, pad=3, relu=True, bf16_weights=precision, round_out=precision)
    ref = oracle.maxpool3x3s2(y)
    got = m.op_stem(to_dev(frames))
    torch.cuda.synchronize()
    got = nhwc_to_nchw(got.float().cpu().numpy())
    assert got.shape == ref.shape
    assert relerr(got, ref) <= (TOL_BF16_STEP if precision else TOL_F32), relerr(got, ref)


def _rand_boxes(rs, n, size):
    x1 = rs.rand(n) * size
    y1 = rs.rand(n) * size
    w = 2 + rs.rand(n) * size / 3
    h = 2 + rs.rand(n) * size / 3
    return np.stack([x1, y1, x1 + w, y1 + h], 1).astype(np.float32)


def test_nms_op_is_bit_exact():
    m, _ = _model(0)
    rs = np.random.RandomState(3)
    cap = 1000
    counts = np.array([1000, 0, 1, 64, 65, 999, 513, 128], np.int32)
    boxes = np.zeros((len(counts), cap, 4), np.float32)
    for f, c in enumerate(counts):
        boxes[f, :c] = _rand_boxes(rs, c, 120.0 if f % 2 == 0 else 400.0)
    boxes[5, 10:20] = boxes[5, 0]                      # exact duplicates: lowest index wins
    for thr, max_keep in [(0.7, 300), (0.5, 1000), (0.3, 7)]:
        keep, cnt = m.op_nms(to_dev(boxes), to_dev(counts), thr, max_keep)
        torch.cuda.synchronize()
        keep, cnt = keep.cpu().numpy(), cnt.cpu().numpy()
        for f, c in enumerate(counts):
            ref = oracle.nms(boxes[f, :c], thr, max_keep)
            assert cnt[f] == len(ref), (thr, f)
            assert np.array_equal(keep[f, :len(ref)], ref), (thr, f)
            assert np.all(keep[f, len(ref):] == -1)


def test_nms_op_large_cap():
    m, _ = _model(0)
    rs = np.random.RandomState(4)
    cap = 2000
    counts = np.array([2000, 1937], np.int32)
    boxes = np.zeros((2, cap, 4), np.float32)
    for f, c in enumerate(counts):
        boxes[f, :c] = _rand_boxes(rs, c, 300.0)
    keep, cnt = m.op_nms(to_dev(boxes), to_dev(counts), 0.7, 1000)
    torch.cuda.synchronize()
    for f, c in enumerate(counts):
        ref = oracle.nms(boxes[f, :c], 0.7, 1000)
        assert cnt[f].item() == len(ref) and np.array_equal(keep[f, :len(ref)].cpu().numpy(), ref)


def test_nms_op_maximum_cap():
    """The largest proposal count the step accepts (4096 boxes: 64 words per mask row, 16 staged words per thread)."""
    m, _ = _model(0)
    rs = np.random.RandomState(6)
    cap = 4096
    counts = np.array([4096, 4095, 3000], np.int32)
    boxes = np.zeros((3, cap, 4), np.float32)
    for f, c in enumerate(counts):
        boxes[f, :c] = _rand_boxes(rs, c, 500.0)
    for thr, max_keep in [(0.7, 4096), (0.5, 1000)]:
        keep, cnt = m.op_nms(to_dev(boxes), to_dev(counts), thr, max_keep)
        torch.cuda.synchronize()
        for f, c in enumerate(counts):
            ref = oracle.nms(boxes[f, :c], thr, max_keep)
            assert cnt[f].item() == len(ref) and np.array_equal(keep[f, :len(ref)].cpu().numpy(), ref), (thr, f)
            assert (keep[f, len(ref):] == -1).all()


@pytest.mark.parametrize("precision,H,W,ep", [(0, 160, 224, 2), (1, 160, 224, 2), (1, 320, 352, 1), (1, 324, 348, 1)])
def test_rpn_proposals_op_matches_oracle(precision, H, W, ep):
    """Top-k indices are bit-exact on identical logits (including ties and signed zeros);
    decoded boxes differ only by the exp() implementation.  The small map takes the one-block-per-frame kernel, the large
    ones (105 600 anchors; 105 705, whose frames do not start on 16-byte boundaries) the multi-block radix passes, whose
    later digits only run for the tied frames."""
    m, blob = _model(precision)
    spec = MINI_BF16 if precision else MINI_FP32
    orc = oracle.Model(blob)
    Ck, Hk, Wk, stride = orc.exit_shape(ep, H, W)
    nA = Hk * Wk * spec.n_anchors
    rs = np.random.RandomState(7)
    n = 6
    logits = rs.randn(n, nA).astype(np.float32)
    logits[5] = 3.0 + 1e-3 * logits[5]                # narrow spread on an offset: thousands share the cut's leading digits
    logits[1] = np.round(logits[1] * 2) / 2          # heavy ties across the cut
    logits[2] = 0.0                                   # all equal: the first k indices win
    logits[2, ::3] = -0.0
    logits[3, : nA // 2] = -5.0                       # ties below the cut only
    deltas = (rs.randn(n, nA, 4) * 0.5).astype(np.float32)
    deltas[4, :, 2:] = -30.0                          # every box collapses: all dropped
    deltas[0, ::5, 0] = 50.0                          # pushed outside the frame: dropped
    idx, boxes, cnt = m.op_rpn_proposals(to_dev(logits), to_dev(deltas), H, W, ep)
    torch.cuda.synchronize()
    idx, boxes, cnt = idx.cpu().numpy(), boxes.cpu().numpy(), cnt.cpu().numpy()
    for f in range(n):
        ridx, _ = oracle.topk(logits[f], spec.pre_nms)
        assert np.array_equal(idx[f, :len(ridx)], ridx), f
        assert np.all(idx[f, len(ridx):] == -1)
        ref = []
        for i in ridx:
            bx, ok = oracle.decode(orc.anchor(i, Wk, stride), deltas[f, i], W, H)
            if ok:
                ref.append(bx)
        ref = np.array(ref, np.float32).reshape(-1, 4)
        assert cnt[f] == len(ref), (f, cnt[f], len(ref))
        if len(ref):
            assert np.max(np.abs(boxes[f, :len(ref)] - ref)) <= 1e-5 * max(H, W) * 4
        assert np.all(boxes[f, len(ref):] == 0)
    assert cnt[4] == 0 and cnt[2] > 0


def test_rpn_proposals_fewer_anchors_than_k():
    m, blob = _model(0)                                # pre_nms 300, smallest map: 1x1..: use ep 4 on a 64x64 frame
    orc = oracle.Model(blob)
    H = W = 64
    Ck, Hk, Wk, stride = orc.exit_shape(4, H, W)
    nA = Hk * Wk * MINI_FP32.n_anchors
    assert nA < MINI_FP32.pre_nms
    rs = np.random.RandomState(8)
    logits = rs.randn(2, nA).astype(np.float32)
    deltas = (rs.randn(2, nA, 4) * 0.1).astype(np.float32)
    idx, boxes, cnt = m.op_rpn_proposals(to_dev(logits), to_dev(deltas), H, W, 4)
    torch.cuda.synchronize()
    for f in range(2):
        ridx, _ = oracle.topk(logits[f], MINI_FP32.pre_nms)
        assert len(ridx) == nA and np.array_equal(idx[f, :nA].cpu().numpy(), ridx)
        assert np.all(idx[f, nA:].cpu().numpy() == -1)


@pytest.mark.parametrize("precision", [0, 1])
def test_roialign_op_matches_oracle(precision):
    m, _ = _model(precision)
    spec = MINI_BF16 if precision else MINI_FP32
    rs = np.random.RandomState(9)
    n, Hk, Wk, Ch, stride = 2, 23, 31, spec.head_ch, 8
    feat = rs.randn(n, Ch, Hk, Wk).astype(np.float32)
    if precision:
        feat = _bf16(feat)
    post = spec.post_nms
    rois = np.zeros((n, post, 4), np.float32)
    rois[:, : post - 5] = _rand_boxes(rs, n * (post - 5), Wk * stride * 0.8).reshape(n, post - 5, 4)
    rois[0, 0] = [0, 0, Wk * stride, Hk * stride]                   # whole map, samples at the borders
    rois[0, 1] = [Wk * stride - 1.5, Hk * stride - 2.5, Wk * stride, Hk * stride]
    rois[0, 2] = [3.3, 4.4, 3.9, 5.0]                                # tiny box inside one texel
    out = m.op_roialign(to_dev(nchw_to_nhwc(feat), m.elem), to_dev(rois), stride)
    torch.cuda.synchronize()
    out = out.float().cpu().numpy()                                  # [n, post, P*P, Ch]
    P = spec.pool
    for f in range(n):
        ref = oracle.roialign(feat[f], rois[f], stride, P, 2, round_out=precision)     # [post, Ch, P, P]
        ref = np.transpose(ref.reshape(post, Ch, P * P), (0, 2, 1))
        assert relerr(out[f], ref) <= (TOL_BF16_STEP if precision else 1e-5), relerr(out[f], ref)


def test_select_detections_op_is_bit_exact():
    m, _ = _model(1)
    spec = MINI_BF16
    rs = np.random.RandomState(10)
    n, post, Kc, D = 4, spec.post_nms, spec.n_classes, spec.max_det
    scores = rs.dirichlet(np.ones(Kc) * 0.7, size=(n, post)).astype(np.float32)
    scores[1] = np.round(scores[1] * 16) / 16                        # many equal scores: index order decides
    boxes = _rand_boxes(rs, n * post * Kc, 500.0).reshape(n, post, Kc, 4)
    boxes[0, :40, 3] = boxes[0, :40, 3]
    boxes[2, ::7, 2, 2] = boxes[2, ::7, 2, 0]                        # empty boxes are never candidates
    roi_n = np.array([post, post - 17, 3, 0], np.int32)
    ob, osc, ol, cnt = m.op_select_detections(to_dev(scores), to_dev(boxes), to_dev(roi_n))
    torch.cuda.synchronize()
    ob, osc, ol, cnt = ob.cpu().numpy(), osc.cpu().numpy(), ol.cpu().numpy(), cnt.cpu().numpy()
    for f in range(n):
        rb, rs_, rl, rn = oracle.select_detections(scores[f, :roi_n[f]], boxes[f, :roi_n[f]], spec.score_thr, spec.det_nms_thr, D)
        assert cnt[f] == rn, f
        assert np.array_equal(ol[f], rl) and np.array_equal(ob[f], rb) and np.array_equal(osc[f], rs_), f
    assert cnt[0] == D and cnt[3] == 0
