"""Seeded synthetic inputs (frames and weights blobs) shared, as data only, by the
CPU oracle's tests and the GPU library's tests.  No detector arithmetic lives here."""
from .configs import CONFIGS, ModelSpec, SceneSpec, Config, small_variant, HEADER_BYTES
from .frames import make_frames
from .weights import make_blob, tensor_list, split_blob, blob_floats
from .classifier import ClassifierSpec, VGG16_EXITS, make_classifier_blob, split_classifier_blob, classifier_tensor_list


def recipe_for(spec):
    """Data-only gains every test, the smoke check and the benchmark apply to the synthetic weights of `spec`
    (keyword arguments of weights.make_blob).  Literal He-normal weights without normalisation layers give degenerate
    proposals, so the last convolution of every residual branch is scaled by 1 / sqrt(number of bottleneck blocks), at
    most 0.25 (0.25 for the 16-block ResNet-50 layout, 0.174 for the 33-block ResNet-101 layout), the two score
    predictors get std 0.01, and the two box-delta predictors std 0.001: deltas as strong as the scores let bf16
    rounding noise move every box by a visible fraction of its size."""
    n_blocks = sum(spec.blocks[:spec.n_stages])
    return dict(res_gain=min(0.25, float(n_blocks) ** -0.5) if n_blocks else 0.25, pred_std=0.01, delta_std=0.001)
