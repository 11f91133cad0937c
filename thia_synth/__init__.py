"""Seeded synthetic inputs (frames and weights blobs) shared, as data only, by the
CPU oracle's tests and the GPU library's tests.  No detector arithmetic lives here."""
from .configs import CONFIGS, ModelSpec, SceneSpec, Config, small_variant, HEADER_BYTES
from .frames import make_frames
from .weights import make_blob, tensor_list, split_blob, blob_floats
