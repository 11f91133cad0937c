"""The image classifier with exits (the paper's generalisation of early inference, Sec. 4.2) on the GPU against its CPU
oracle, through the C ABI: single steps on identical inputs, every exit of a reduced network element by element, and the
full VGG-16-style network (thirteen 3x3 layers, eight exits, 102 classes) at 224 x 224."""
import numpy as np
import pytest
import torch

from gpu_common import nchw_to_nhwc, relerr, to_dev
from oracle import classifier as oc
from thia_synth import ClassifierSpec, VGG16_EXITS, SceneSpec, make_classifier_blob, make_frames, split_classifier_blob

pytestmark = pytest.mark.gpu

TOL = {0: 1e-4, 1: 2e-2}      # logits, per tensor max |gpu - ref| / max |ref|: fp32 path; bf16 path vs the fp32 oracle
SMALL = {p: ClassifierSpec(precision=p, channels=(64, 64, 128, 128, 192), pool_after=(2, 4), taps=(1, 2, 4, 5), n_classes=11) for p in (0, 1)}
_cache = {}


def _clf(spec, seed):
    from paper_2102_08481_amd import thia_classifier_load
    key = (spec.header(), seed)
    if key not in _cache:
        blob = make_classifier_blob(spec, seed)
        _cache[key] = (thia_classifier_load(blob, spec.n_exits), blob)
    return _cache[key]


def _check_answers(labels, conf, logits, ref, tol):
    """Logits within tol; where the reference's best class leads the runner-up by more than the error bound both sides must
    name it (the decision is then not a matter of rounding); elsewhere the GPU's label must be one of the near-tied classes."""
    g_lab, g_conf, g_log = labels.cpu().numpy(), conf.cpu().numpy(), logits.cpu().numpy()
    err = relerr(g_log, ref["logits"])
    assert err <= tol, err
    bound = 2 * tol * np.max(np.abs(ref["logits"]))
    srt = np.sort(ref["logits"], axis=1)
    clear = srt[:, -1] - srt[:, -2] > bound
    assert np.array_equal(g_lab[clear], ref["labels"][clear])
    for f in np.flatnonzero(~clear):
        assert ref["logits"][f, g_lab[f]] >= srt[f, -1] - bound
    assert np.array_equal(g_lab, np.argmax(g_log, axis=1))            # the GPU's own decision: first maximum of its own logits
    assert np.max(np.abs(g_conf[clear] - ref["conf"][clear])) <= 4 * bound + 1e-5
    return err, int(clear.sum())


@pytest.mark.parametrize("precision", [0, 1])
def test_pool_step_matches_oracle(precision):
    c, _ = _clf(SMALL[precision], 70)
    rs = np.random.RandomState(1)
    for (n, H, W, C) in [(2, 8, 8, 64), (3, 9, 11, 64), (1, 33, 20, 192)]:
        x = rs.randn(n, C, H, W).astype(np.float32)
        if precision:
            x = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
        y = c.op_pool(to_dev(nchw_to_nhwc(x), c.elem))
        torch.cuda.synchronize()
        assert np.array_equal(y.float().cpu().numpy(), nchw_to_nhwc(oc.maxpool2x2(x)))       # a maximum is exact


@pytest.mark.parametrize("precision", [0, 1])
def test_unit_step_matches_oracle(precision):
    """Global average pooling + FC + soft-max + arg-max on the oracle's tapped tensor (teacher forcing)."""
    spec = SMALL[precision]
    c, blob = _clf(spec, 70)
    fr = make_frames(SceneSpec(45, 61, 3, 2, 4, 8, 30, "gradient"), 5)
    for ep in (1, 4):
        ref = oc.classify(blob, fr, ep)
        n, C, h, w = ref["feat"].shape
        feat = to_dev(nchw_to_nhwc(ref["feat"]).reshape(n, h * w, C), c.elem)
        lab, conf, log = c.op_unit(feat, ep)
        torch.cuda.synchronize()
        _check_answers(lab, conf, log, ref, 1e-5)


@pytest.mark.parametrize("precision", [0, 1])
@pytest.mark.parametrize("ep", [0, 1, 2, 3, 4])
def test_small_classifier_every_exit(precision, ep):
    spec = SMALL[precision]
    c, blob = _clf(spec, 70)
    fr = make_frames(SceneSpec(45, 61, 5, 2, 4, 8, 30, "gradient"), 6)       # odd sizes: ragged tiles, dropped pool rows
    lab, conf, log = c.classify_chunk(to_dev(fr), ep, want_logits=True)
    torch.cuda.synchronize()
    if ep == 0:
        assert (lab == -1).all() and (conf == 0).all()
        return
    ref = oc.classify(blob, fr, ep, precision=0)
    err, n_clear = _check_answers(lab, conf, log, ref, TOL[precision])
    print(f"small classifier precision {precision} exit {ep}: logits max rel err {err:.2e}, {n_clear}/5 decisions beyond rounding")
    # the same call again is bit-identical, and a frame's answer does not depend on its chunk
    lab2, conf2, log2 = c.classify_chunk(to_dev(fr[1:3]), ep, want_logits=True)
    torch.cuda.synchronize()
    assert torch.equal(log2, log[1:3]) and torch.equal(lab2, lab[1:3]) and torch.equal(conf2, conf[1:3])


def test_exits_stop_early_and_share_the_prefix():
    """Layers behind the tapped one are not run (changed weights there change nothing), which is early inference."""
    spec = SMALL[1]
    blob = make_classifier_blob(spec, 70)
    poisoned = blob.copy()
    t = split_classifier_blob(spec, poisoned)
    for i in range(spec.taps[1] + 1, spec.n_layers + 1):
        t[f"conv{i}.w"][...] = 0.5
    from paper_2102_08481_amd import thia_classifier_load
    c, _ = _clf(spec, 70)
    cp = thia_classifier_load(poisoned, spec.n_exits)
    fr = to_dev(make_frames(SceneSpec(45, 61, 2, 2, 4, 8, 30, "gradient"), 8))
    a = c.classify_chunk(fr, 2, want_logits=True)
    b = cp.classify_chunk(fr, 2, want_logits=True)
    torch.cuda.synchronize()
    assert torch.equal(a[2], b[2]) and torch.equal(a[0], b[0])
    a3 = c.classify_chunk(fr, 3, want_logits=True)[2]
    b3 = cp.classify_chunk(fr, 3, want_logits=True)[2]
    torch.cuda.synchronize()
    assert not torch.equal(a3, b3)                     # (the changed layers do matter one exit further on)
    cp.close()


@pytest.mark.parametrize("ep", [1, 4, 8])
def test_vgg16_eight_exits_at_224(ep):
    """The paper's generalisation case at its real shape: VGG-16's thirteen layers, eight exits, 102 classes, 224 x 224 frames,
    bf16; the oracle is run on the first two frames of an 8-frame chunk."""
    spec = VGG16_EXITS
    c, blob = _clf(spec, 71)
    fr = make_frames(SceneSpec(224, 224, 8, 3, 8, 16, 120, "gradient"), 9)
    lab, conf, log = c.classify_chunk(to_dev(fr), ep, want_logits=True)
    torch.cuda.synchronize()
    assert ((lab >= 0) & (lab < 102)).all() and ((conf > 0) & (conf <= 1)).all()
    ref = oc.classify(blob, fr[:2], ep, precision=0)
    err, n_clear = _check_answers(lab[:2], conf[:2], log[:2], ref, TOL[1])
    print(f"VGG-16-style exit {ep}: logits max rel err vs fp32 oracle {err:.2e}, {n_clear}/2 decisions beyond rounding")


def test_classifier_argument_errors():
    from paper_2102_08481_amd import ThiaError, thia_classifier_load
    spec = SMALL[1]
    c, blob = _clf(spec, 70)
    fr = to_dev(make_frames(SceneSpec(45, 61, 1, 2, 4, 8, 30, "gradient"), 8))
    with pytest.raises(ThiaError) as e:
        c.classify_chunk(fr, 5)
    assert e.value.code == -2
    with pytest.raises(ThiaError) as e:
        thia_classifier_load(blob[:-4], spec.n_exits)
    assert e.value.code == -4
    with pytest.raises(ThiaError) as e:
        thia_classifier_load(blob, spec.n_exits + 1)
    assert e.value.code == -4
    tiny = to_dev(np.zeros((1, 3, 1, 1), np.uint8))
    with pytest.raises(ThiaError) as e:
        c.classify_chunk(tiny, 4)                      # two pools in front of exit 4 leave no position
    assert e.value.code == -3
    lab, conf = c.classify_chunk(tiny, 1)              # exit 1 has no pool in front of it
    torch.cuda.synchronize()
    assert 0 <= int(lab[0]) < spec.n_classes
