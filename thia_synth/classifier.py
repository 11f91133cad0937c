"""Seeded blob of an image classifier with exits (the paper's generalisation of early inference to a VGG-16-style
network, Sec. 4.2): data only, no classifier arithmetic.

Blob = 256-byte little-endian header (64 four-byte words) + fp32 tensors.

Header words (i = int32, f = float32):
  0 i magic 0x43494854 ("THIC")   1 i version (1)
  2 i precision: 0 fp32, 1 bf16 storage with fp32 accumulation
  3 i n_exits (1..8)              4 i n_layers: 3x3 convolutions in the backbone (1..16)
  5 i input channels (3)          6 i classes
  7 f pixel mean                  8 f pixel std
  9-24  i output channels of conv layer 1..16 (0 beyond n_layers)
  25-40 i 1 if a 2x2 / stride 2 max-pool follows conv layer 1..16
  41-48 i exit k (1..8) reads the output of conv layer tap[k] (after its ReLU, before any pooling); strictly increasing
  49-63 reserved, zero

Tensors, in order: conv i weight [Cout, Cin, 3, 3] and bias [Cout] for i = 1..n_layers; then for exit k = 1..n_exits the
classifier unit's weight [classes, C_tap(k)] and bias [classes].  Values: normal, std sqrt(2 / fan_in), biases zero,
tensor t from rng stream t (the unit's weight with std `pred_std` if given).
"""
from dataclasses import dataclass
import struct

import numpy as np

from . import rng
from .configs import HEADER_BYTES

CLS_MAGIC = 0x43494854


@dataclass(frozen=True)
class ClassifierSpec:
    precision: int = 1
    channels: tuple = (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512)     # VGG-16's thirteen 3x3 layers
    pool_after: tuple = (2, 4, 7, 10, 13)                                                  # 1-based layer indices
    taps: tuple = (2, 4, 6, 7, 9, 10, 12, 13)                                              # eight exits
    in_ch: int = 3
    n_classes: int = 102
    mean: float = 114.0
    std: float = 58.0

    @property
    def n_exits(self):
        return len(self.taps)

    @property
    def n_layers(self):
        return len(self.channels)

    def header(self):
        w = [0] * 64
        f = lambda x: struct.unpack("<i", struct.pack("<f", float(x)))[0]
        w[0], w[1], w[2], w[3], w[4], w[5], w[6] = CLS_MAGIC, 1, self.precision, self.n_exits, self.n_layers, self.in_ch, self.n_classes
        w[7], w[8] = f(self.mean), f(self.std)
        for i, c in enumerate(self.channels):
            w[9 + i] = c
            w[25 + i] = 1 if (i + 1) in self.pool_after else 0
        for k, t in enumerate(self.taps):
            w[41 + k] = t
        return struct.pack("<64i", *w)


VGG16_EXITS = ClassifierSpec()


def classifier_tensor_list(spec: ClassifierSpec):
    out, cin = [], spec.in_ch
    for i, c in enumerate(spec.channels):
        out.append((f"conv{i + 1}.w", (c, cin, 3, 3), "conv"))
        out.append((f"conv{i + 1}.b", (c,), "bias"))
        cin = c
    for k, t in enumerate(spec.taps):
        out.append((f"exit{k + 1}.w", (spec.n_classes, spec.channels[t - 1]), "pred"))
        out.append((f"exit{k + 1}.b", (spec.n_classes,), "bias"))
    return out


def make_classifier_blob(spec: ClassifierSpec, seed: int, pred_std=None) -> np.ndarray:
    tl = classifier_tensor_list(spec)
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
            std = np.sqrt(2.0 / int(np.prod(shape[1:])))
            if role == "pred" and pred_std is not None:
                std = pred_std
            body[off:off + n] = (std * rng.normal(seed, t, n)).astype(np.float32)
        off += n
    return blob


def split_classifier_blob(spec: ClassifierSpec, blob: np.ndarray):
    body = blob[HEADER_BYTES:].view(np.float32)
    out, off = {}, 0
    for name, shape, _ in classifier_tensor_list(spec):
        n = int(np.prod(shape))
        out[name] = body[off:off + n].reshape(shape)
        off += n
    return out
