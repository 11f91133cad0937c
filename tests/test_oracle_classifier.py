"""Pins of the classifier oracle (oracle/classifier.py) against something other than itself: torch's float64 operators
for the whole stack, hand cases for the pooling, and the structural invariants the paper states for exits (an exit reads
a prefix of the next exit's computation; nothing after the tapped layer is evaluated)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import classifier as oc
from thia_synth import ClassifierSpec, make_classifier_blob, split_classifier_blob

SPEC = ClassifierSpec(precision=0, channels=(8, 8, 16, 16, 24), pool_after=(2, 4), taps=(1, 2, 4, 5), n_classes=7)


def _frames(n=3, H=21, W=26, seed=0):
    return np.random.RandomState(seed).randint(0, 256, (n, 3, H, W)).astype(np.uint8)


def _torch_reference(spec, blob, frames, ep):
    w = {k: torch.from_numpy(np.array(v)).double() for k, v in split_classifier_blob(spec, blob).items()}
    x = (torch.from_numpy(frames).double() - spec.mean) / spec.std
    tap = spec.taps[ep - 1]
    for i in range(1, tap + 1):
        x = F.relu(F.conv2d(x, w[f"conv{i}.w"], w[f"conv{i}.b"], padding=1))
        if i in spec.pool_after and i < tap:
            x = F.max_pool2d(x, 2, 2)
    g = F.adaptive_avg_pool2d(x, 1).flatten(1)
    logits = F.linear(g, w[f"exit{ep}.w"], w[f"exit{ep}.b"])
    p = F.softmax(logits, dim=1)
    return x.numpy(), logits.numpy(), p.numpy()


@pytest.mark.parametrize("ep", [1, 2, 3, 4])
def test_classifier_matches_torch_float64(ep):
    blob = make_classifier_blob(SPEC, 3)
    fr = _frames()
    r = oc.classify(blob, fr, ep)
    feat, logits, p = _torch_reference(SPEC, blob, fr, ep)
    assert r["feat"].shape == feat.shape
    assert np.max(np.abs(r["feat"] - feat)) <= 1e-5 * np.max(np.abs(feat))
    assert np.max(np.abs(r["logits"] - logits)) <= 1e-5 * np.max(np.abs(logits))
    assert np.array_equal(r["labels"], np.argmax(logits, axis=1))
    assert np.allclose(r["conf"], p.max(axis=1), rtol=1e-5)


def test_maxpool2x2_hand_cases():
    x = np.arange(2 * 1 * 5 * 4, dtype=np.float32).reshape(2, 1, 5, 4)
    y = oc.maxpool2x2(x)
    assert y.shape == (2, 1, 2, 2)                                   # the odd fifth row is dropped
    assert np.array_equal(y[0, 0], np.array([[5, 7], [13, 15]], np.float32))
    z = oc.maxpool2x2(-x)
    assert np.array_equal(z[0, 0], -np.array([[0, 2], [8, 10]], np.float32))   # the maximum, not the last or the largest magnitude


def test_exit_reads_a_prefix_and_later_layers_are_not_evaluated():
    blob = make_classifier_blob(SPEC, 4)
    fr = _frames(2)
    ref = oc.classify(blob, fr, 2)
    poisoned = blob.copy()
    t = split_classifier_blob(SPEC, poisoned)
    for i in range(SPEC.taps[1] + 1, SPEC.n_layers + 1):
        t[f"conv{i}.w"][...] = np.nan
    for k in (1, 3, 4):
        t[f"exit{k}.w"][...] = np.nan
    got = oc.classify(poisoned, fr, 2)
    assert np.array_equal(got["logits"], ref["logits"]) and np.array_equal(got["labels"], ref["labels"])
    # exit 3 continues from exit 2's tensor: pool (layer 2 is flagged) then layers 3, 4
    f3 = oc.backbone(blob, fr, 3)
    x = oc.maxpool2x2(ref["feat"])
    w = split_classifier_blob(SPEC, blob)
    import oracle
    for i in (3, 4):
        x = oracle.conv2d(x, w[f"conv{i}.w"], w[f"conv{i}.b"], stride=1, pad=1, relu=True)
    assert np.array_equal(x, f3)


def test_tie_goes_to_the_lowest_class_and_pooling_is_a_mean():
    spec = ClassifierSpec(precision=0, channels=(4,), pool_after=(), taps=(1,), n_classes=3)
    blob = make_classifier_blob(spec, 5)
    t = split_classifier_blob(spec, blob)
    t["conv1.w"][...] = 0.0
    t["conv1.b"][...] = np.array([1.0, 2.0, 3.0, 4.0], np.float32)     # every position holds (1, 2, 3, 4) after ReLU
    t["exit1.w"][...] = np.array([[0, 0, 0, 1], [0, 0, 0, 1], [1, 0, 0, 0]], np.float32)
    t["exit1.b"][...] = 0.0
    r = oc.classify(blob, _frames(2, 9, 11), 1)
    assert np.allclose(r["logits"], [[4, 4, 1]] * 2)                    # a mean (not a sum over the 99 positions)
    assert np.array_equal(r["labels"], [0, 0])
    e = np.exp(np.array([4.0, 4.0, 1.0]) - 4.0)
    assert np.allclose(r["conf"], (e / e.sum())[0])


def test_bf16_storage_rounds_weights_and_activations():
    spec = ClassifierSpec(precision=1, channels=(8, 8), pool_after=(1,), taps=(2,), n_classes=5)
    blob = make_classifier_blob(spec, 6)
    fr = _frames(1, 12, 12)
    f16 = oc.backbone(blob, fr, 1)
    as_bf16 = torch.from_numpy(f16).to(torch.bfloat16).float().numpy()
    assert np.array_equal(f16, as_bf16)                                 # stored activations are bf16 values
    f32 = oc.backbone(blob, fr, 1, precision=0)
    assert not np.array_equal(f16, f32) and np.max(np.abs(f16 - f32)) <= 2e-2 * np.max(np.abs(f32))
