import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from thia_synth import recipe_for   # data-only gains of the synthetic weights (see thia_synth.recipe_for)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs an MI355X (runs through the C-ABI library)")


_blob_cache = {}


def get_blob(spec, seed):
    """Weights blob for a ModelSpec; cached in memory and under /tmp (generation takes seconds)."""
    from thia_synth import make_blob
    import hashlib
    key = hashlib.sha1(spec.header() + seed.to_bytes(8, "little") + repr(sorted(recipe_for(spec).items())).encode()).hexdigest()[:16]
    if key in _blob_cache:
        return _blob_cache[key]
    path = f"/tmp/thia_blob_{key}.npy"
    if os.path.exists(path):
        blob = np.load(path)
    else:
        blob = make_blob(spec, seed, **recipe_for(spec))
        tmp = path + f".{os.getpid()}.npy"
        np.save(tmp, blob)
        os.replace(tmp, path)
    _blob_cache[key] = blob
    return blob


@pytest.fixture(scope="session")
def tiny():
    """Config 1 (tiny single-exit fp32 detector): (config, blob, frames)."""
    from thia_synth import CONFIGS, make_frames
    cfg = CONFIGS[1]
    return cfg, get_blob(cfg.model, cfg.weight_seed), make_frames(cfg.scene, cfg.frame_seed)
