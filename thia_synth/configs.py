"""Hyper-parameters of the five benchmark configurations and the weights-blob
header that carries them.

The blob is the only thing a detector implementation needs besides frames:
a 256-byte little-endian header (64 four-byte words, layout below) followed by
fp32 tensors in a fixed order (see weights.tensor_list).  This module only
describes data; it holds no detector arithmetic.

Header words (i = int32, f = float32):
  0 i magic 0x41494854 ("THIA")     1 i version (1)
  2 i precision: 0 fp32, 1 bf16 storage with fp32 accumulation
  3 i n_exits (1..4, or 1..5 with a stem exit)   4-7 i bottleneck blocks in conv2_x..conv5_x
  8 i stem channels                 9 i has_lateral (0/1)
 10 i head channels (lateral / RPN width, ROI feature channels)
 11 i n_sizes  12 i n_ratios        13-20 f anchor sizes (px)   21-24 f ratios h/w
 25 i pre-NMS top-k                 26 i post-NMS proposals
 27 f RPN NMS IoU threshold         28 i ROIAlign output size (7)
 29 i ROIAlign sampling ratio (2)   30 i FC width (1024)
 31 i classes incl. background      32 f score threshold
 33 f detection NMS IoU threshold   34 i max detections per frame D
 35 f pixel mean                    36 f pixel std
 37 i bottleneck base width (64)
 38 i stem exit (0/1): 1 = exit 1 reads the pooled stem output (stem channels, stride 4) and exit k >= 2 reads
      conv(k)_x, as in the paper's five-exit case study; 0 = exit k reads conv(k+1)_x
 39-63 reserved, zero
"""
from dataclasses import dataclass, field, replace
import struct

MAGIC = 0x41494854
VERSION = 1
HEADER_BYTES = 256


@dataclass(frozen=True)
class ModelSpec:
    precision: int = 0                 # 0 fp32, 1 bf16
    n_exits: int = 4
    blocks: tuple = (3, 4, 6, 3)
    stem_ch: int = 64
    has_lateral: int = 1
    head_ch: int = 256
    sizes: tuple = (32.0, 64.0, 128.0, 256.0, 512.0)
    ratios: tuple = (0.5, 1.0, 2.0)
    pre_nms: int = 1000
    post_nms: int = 300
    rpn_nms_thr: float = 0.7
    pool: int = 7
    sampling: int = 2
    fc_dim: int = 1024
    n_classes: int = 8
    score_thr: float = 0.05
    det_nms_thr: float = 0.5
    max_det: int = 100
    mean: float = 114.0
    std: float = 58.0
    base_width: int = 64
    stem_exit: int = 0                 # 1: exit 1 sits on the pooled stem output (paper's EP-1, Table 4)

    @property
    def n_stages(self):
        """Bottleneck stages the deepest exit needs."""
        return self.n_exits - self.stem_exit

    @property
    def n_anchors(self):
        return len(self.sizes) * len(self.ratios)

    def stage_channels(self, k):
        """Channels of the tensor exit k (1-based) reads: 256, 512, 1024, 2048 (with a stem exit: 64 first)."""
        k -= self.stem_exit
        return self.stem_ch if k == 0 else 4 * self.base_width * (1 << (k - 1))

    def stride(self, k):
        k -= self.stem_exit
        return 4 if k == 0 else 4 << (k - 1)

    def header(self):
        w = [0] * 64
        f = lambda x: struct.unpack("<i", struct.pack("<f", float(x)))[0]
        w[0], w[1], w[2], w[3] = MAGIC, VERSION, self.precision, self.n_exits
        for i in range(4):
            w[4 + i] = self.blocks[i] if i < len(self.blocks) else 0
        w[8], w[9], w[10] = self.stem_ch, self.has_lateral, self.head_ch
        w[11], w[12] = len(self.sizes), len(self.ratios)
        for i, s in enumerate(self.sizes):
            w[13 + i] = f(s)
        for i, r in enumerate(self.ratios):
            w[21 + i] = f(r)
        w[25], w[26], w[27] = self.pre_nms, self.post_nms, f(self.rpn_nms_thr)
        w[28], w[29], w[30], w[31] = self.pool, self.sampling, self.fc_dim, self.n_classes
        w[32], w[33], w[34] = f(self.score_thr), f(self.det_nms_thr), self.max_det
        w[35], w[36], w[37], w[38] = f(self.mean), f(self.std), self.base_width, self.stem_exit
        return struct.pack("<64i", *w)


@dataclass(frozen=True)
class SceneSpec:
    """Recipe of the synthetic frames of one configuration."""
    height: int
    width: int
    n_frames: int
    rect_min: int
    rect_max: int
    side_min: int
    side_max: int
    style: str = "road"          # "road" (gray road + shading) or "gradient"
    noise: int = 0               # per-pixel, per-channel sensor noise: uniform integers in -noise .. +noise added before clipping


@dataclass(frozen=True)
class Config:
    name: str
    model: ModelSpec
    scene: SceneSpec
    frame_seed: int
    weight_seed: int
    exits: tuple = (1,)


_R50 = ModelSpec(precision=1)
_R101 = replace(_R50, blocks=(3, 4, 23, 3), pre_nms=2000, post_nms=1000, n_classes=20)
_TINY = ModelSpec(precision=0, n_exits=1, blocks=(3, 0, 0, 0), has_lateral=0,
                  sizes=(32.0, 64.0, 128.0), ratios=(1.0,), pre_nms=200, post_nms=50, n_classes=3)

_ROAD540 = SceneSpec(540, 960, 16, 5, 40, 16, 300, noise=16)

CONFIGS = {
    1: Config("tiny-fp32", _TINY, SceneSpec(128, 128, 4, 3, 6, 12, 64, "gradient"),
              0x7414A + 1, 0xBEEF + 1, (1,)),
    2: Config("r50-ep2-b16", _R50, _ROAD540, 0x7414A + 2, 0xBEEF + 2, (2,)),
    3: Config("r50-sweep-b32", _R50, replace(_ROAD540, n_frames=32), 0x7414A + 3, 0xBEEF + 2, (1, 2, 3, 4)),
    4: Config("r50-plan-8x32", _R50, replace(_ROAD540, n_frames=256), 0x7414A + 4, 0xBEEF + 2, (1, 4, 2, 2, 3, 1, 4, 3)),
    5: Config("r101-1080p-b8", _R101, SceneSpec(1080, 1920, 8, 20, 150, 8, 400, noise=16), 0x7414A + 5, 0xBEEF + 5, (1, 2, 3, 4)),
}


def small_variant(cfg, height, width, n_frames, **model_overrides):
    """Same architecture on smaller frames: used where the CPU oracle must finish in seconds."""
    return replace(cfg, scene=replace(cfg.scene, height=height, width=width, n_frames=n_frames),
                   model=replace(cfg.model, **model_overrides))
