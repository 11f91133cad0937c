"""MI355X-native execution engine of a multi-exit two-stage detector (THIA, arXiv
2102.08481): a C-ABI HIP library (libthia.so, see include/thia.h) and this thin binding.

The names below mirror the C entry points; they only marshal arguments.
"""
from .binding import Model, ThiaError, ThiaInfo, lib, EXPORTS, TAPS, KERNEL_CLASSES, LIB_PATH


def thia_load_model(weights, n_exits, device="cuda:0"):
    """weights: uint8 numpy blob (header + fp32 tensors).  Returns the resident model."""
    return Model(weights, n_exits, device)


def thia_detect_chunk(model, frames, ep, out=None):
    """frames: cuda uint8 [n,3,H,W]; ep in 1..n_exits or 0 (skip).  Returns (boxes, scores, labels)."""
    return model.detect_chunk(frames, ep, out)


def thia_run_plan(model, frames, chunk_len, chunk_ep, out=None):
    """frames: cuda uint8 [n_chunks*chunk_len,3,H,W]; chunk_ep: exit per chunk (0 = skip)."""
    return model.run_plan(frames, chunk_len, chunk_ep, out)


def thia_free_model(model):
    model.close()
