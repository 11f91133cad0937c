"""CPU oracle of the image classifier with exits (the paper's generalisation of early inference, Sec. 4.2, "Generalization"
paragraph and its figure): TEST INFRASTRUCTURE ONLY, like the rest of oracle/.

The paper names the network (VGG-16: a stack of 3x3 convolutions with ReLU, 2x2 max-pools in between) and says exits are
added as for the detector (Sec. 4.1: a unit with the structure of the last one, its first layer sized to the tapped
layer's channels; inference stops at the chosen exit).  It does not define the unit.  Reading taken here and in the
library: the unit is global average pooling over the tapped layer's output followed by one fully connected layer to the
class logits; the answer is the arg-max class (the lowest class on a tie) and its softmax probability.

Steps, in order, for exit k of an image:
  x = (u8 - mean) / std
  for conv layer i = 1 .. tap[k]:  x = relu(conv3x3(x, W_i) + b_i)  (zero padding 1, stride 1);
                                   a 2x2 / stride-2 max-pool follows layer i if flagged AND i < tap[k]
  g[c] = mean over positions of x[c]
  logits = V_k g + c_k;  label = argmax;  confidence = softmax(logits)[label]
Convolutions use the oracle's pinned C step (double accumulation, one rounding); everything after them is float64 here.
With bf16 storage (precision 1) weights and stored activations are rounded to bf16 as in the detector; the unit is fp32.
"""
import numpy as np

import oracle


def parse_header(blob):
    hi = np.ascontiguousarray(blob[:256]).view(np.int32)
    hf = np.ascontiguousarray(blob[:256]).view(np.float32)
    assert hi[0] == 0x43494854 and hi[1] == 1, "not a classifier blob"
    L, E = int(hi[4]), int(hi[3])
    return dict(precision=int(hi[2]), n_exits=E, n_layers=L, in_ch=int(hi[5]), n_classes=int(hi[6]), mean=float(hf[7]), std=float(hf[8]),
                channels=[int(v) for v in hi[9:9 + L]], pool=[int(v) for v in hi[25:25 + L]], taps=[int(v) for v in hi[41:41 + E]])


def tensors(blob, h):
    body = np.ascontiguousarray(blob[256:]).view(np.float32)
    out, off, cin = {}, 0, h["in_ch"]

    def take(shape):
        nonlocal off
        n = int(np.prod(shape))
        v = body[off:off + n].reshape(shape)
        off += n
        return v
    for i, c in enumerate(h["channels"]):
        out[f"conv{i + 1}.w"], out[f"conv{i + 1}.b"] = take((c, cin, 3, 3)), take((c,))
        cin = c
    for k, t in enumerate(h["taps"]):
        out[f"exit{k + 1}.w"], out[f"exit{k + 1}.b"] = take((h["n_classes"], h["channels"][t - 1])), take((h["n_classes"],))
    assert off == body.size
    return out


def maxpool2x2(x):
    """2x2 windows, stride 2, no padding; a trailing odd row / column is dropped.  x [n, C, H, W]."""
    n, c, H, W = x.shape
    return x[:, :, :H // 2 * 2, :W // 2 * 2].reshape(n, c, H // 2, 2, W // 2, 2).max(axis=(3, 5))


def backbone(blob, frames, ep, precision=None):
    """Output of the conv layer exit ep taps: float32 [n, C, h, w]."""
    h = parse_header(blob)
    bf = h["precision"] if precision is None else precision
    w = tensors(blob, h)
    x = oracle.normalize(frames, h["mean"], h["std"], bf16=bf)
    tap = h["taps"][ep - 1]
    for i in range(1, tap + 1):
        x = oracle.conv2d(x, w[f"conv{i}.w"], w[f"conv{i}.b"], stride=1, pad=1, relu=True, bf16_weights=bf, round_out=bf)
        if h["pool"][i - 1] and i < tap:
            x = maxpool2x2(x)
    return x


def classify(blob, frames, ep, precision=None):
    """-> dict(labels int32 [n], conf float32 [n], logits float32 [n, classes], feat float32 [n, C, h, w])."""
    h = parse_header(blob)
    w = tensors(blob, h)
    x = backbone(blob, frames, ep, precision)
    g = x.astype(np.float64).mean(axis=(2, 3))
    logits = (g @ w[f"exit{ep}.w"].astype(np.float64).T + w[f"exit{ep}.b"].astype(np.float64)).astype(np.float32)
    z = logits.astype(np.float64)
    z = np.exp(z - z.max(axis=1, keepdims=True))
    p = z / z.sum(axis=1, keepdims=True)
    labels = np.argmax(logits, axis=1).astype(np.int32)          # numpy's arg-max returns the first maximum
    conf = p[np.arange(len(labels)), labels].astype(np.float32)
    return dict(labels=labels, conf=conf, logits=logits, feat=x)
