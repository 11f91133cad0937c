"""Seeded weights blob: header (configs.ModelSpec.header) + fp32 tensors.

Tensor order (conv weights [Cout, Cin, kh, kw]; FC weights [out, in]; every
weight is followed by its bias [Cout]):

  stem 7x7
  for stage s = 1 .. n_stages (= n_exits, or n_exits - 1 with a stem exit), block b = 0 .. blocks[s-1]-1:
      conv1 1x1 (Cin -> w), conv2 3x3 (w -> w), conv3 1x1 (w -> 4w),
      and for b == 0 only: shortcut 1x1 (Cin -> 4w)          with w = base_width * 2**(s-1)
  for exit e = 1 .. n_exits:
      [lateral 1x1 (C_e -> head_ch)]  if has_lateral
      rpn.conv 3x3 (head_ch -> head_ch), rpn.obj 1x1 (-> A), rpn.delta 1x1 (-> 4A)
      fc1 (head_ch*pool*pool -> fc), fc2 (fc -> fc), cls (fc -> Kc), box (fc -> 4 Kc)

FC1's input index is c*pool*pool + ph*pool + pw.  RPN delta channel is 4*a + j
(j = dx, dy, dw, dh); box output is 4*c + j.

Values: normal with std sqrt(2 / fan_in) (fan_in = Cin*kh*kw), biases zero.
Optional gains change only the *data* (never the detector): `res_gain` multiplies the
last conv of every residual branch, `pred_std` replaces the std of the two score
predictors (rpn.obj, cls) and `delta_std` (default: `pred_std`) that of the two box-delta
predictors (rpn.delta, box).
"""
import numpy as np

from . import rng
from .configs import ModelSpec, HEADER_BYTES


def tensor_list(spec: ModelSpec):
    """[(name, shape, role)] in blob order; role in {'conv','res_last','pred','pred_delta','bias'}."""
    out = []

    def conv(name, co, ci, k, role="conv"):
        out.append((name + ".w", (co, ci, k, k), role))
        out.append((name + ".b", (co,), "bias"))

    def fc(name, co, ci, role="conv"):
        out.append((name + ".w", (co, ci), role))
        out.append((name + ".b", (co,), "bias"))

    conv("stem", spec.stem_ch, 3, 7)
    cin = spec.stem_ch
    for s in range(1, spec.n_stages + 1):
        w = spec.base_width << (s - 1)
        for b in range(spec.blocks[s - 1]):
            p = f"s{s}.b{b}"
            conv(p + ".conv1", w, cin, 1)
            conv(p + ".conv2", w, w, 3)
            conv(p + ".conv3", 4 * w, w, 1, "res_last")
            if b == 0:
                conv(p + ".short", 4 * w, cin, 1)
            cin = 4 * w
    A = spec.n_anchors
    for e in range(1, spec.n_exits + 1):
        p = f"e{e}"
        ce = spec.stage_channels(e)
        if spec.has_lateral:
            conv(p + ".lateral", spec.head_ch, ce, 1)
            hc = spec.head_ch
        else:
            hc = ce
        conv(p + ".rpn.conv", hc, hc, 3)
        conv(p + ".rpn.obj", A, hc, 1, "pred")
        conv(p + ".rpn.delta", 4 * A, hc, 1, "pred_delta")
        fc(p + ".fc1", spec.fc_dim, hc * spec.pool * spec.pool)
        fc(p + ".fc2", spec.fc_dim, spec.fc_dim)
        fc(p + ".cls", spec.n_classes, spec.fc_dim, "pred")
        fc(p + ".box", 4 * spec.n_classes, spec.fc_dim, "pred_delta")
    return out


def blob_floats(spec: ModelSpec):
    return sum(int(np.prod(s)) for _, s, _ in tensor_list(spec))


def make_blob(spec: ModelSpec, seed: int, res_gain: float = 1.0, pred_std=None, delta_std=None) -> np.ndarray:
    """uint8 array: header + tensors.  Tensor t draws from rng stream t."""
    tl = tensor_list(spec)
    total = sum(int(np.prod(s)) for _, s, _ in tl)
    blob = np.empty(HEADER_BYTES + 4 * total, dtype=np.uint8)
    blob[:HEADER_BYTES] = np.frombuffer(spec.header(), dtype=np.uint8)
    body = blob[HEADER_BYTES:].view(np.float32)
    off = 0
    for t, (name, shape, role) in enumerate(tl):
        n = int(np.prod(shape))
        if role == "bias":
            body[off:off + n] = 0.0
        else:
            fan_in = int(np.prod(shape[1:]))
            std = np.sqrt(2.0 / fan_in)
            if role == "pred" and pred_std is not None:
                std = pred_std
            if role == "pred_delta" and (delta_std is not None or pred_std is not None):
                std = delta_std if delta_std is not None else pred_std
            if role == "res_last":
                std *= res_gain
            # generate in slabs to bound temporary memory
            step = 1 << 22
            for s0 in range(0, n, step):
                m = min(step, n - s0)
                body[off + s0:off + s0 + m] = (std * rng.normal(seed, t, m, s0)).astype(np.float32)
        off += n
    return blob


def split_blob(spec: ModelSpec, blob: np.ndarray):
    """{name: fp32 array view} — for tests that want to look at individual tensors."""
    body = blob[HEADER_BYTES:].view(np.float32)
    out, off = {}, 0
    for name, shape, _ in tensor_list(spec):
        n = int(np.prod(shape))
        out[name] = body[off:off + n].reshape(shape)
        off += n
    return out
