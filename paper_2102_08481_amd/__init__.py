"""MI355X-native execution engine of a multi-exit two-stage detector (THIA, arXiv
2102.08481): a C-ABI HIP library (libthia.so, see include/thia.h) and this thin binding.

The names below mirror the C entry points; they only marshal arguments.
"""
from .binding import (Model, Classifier, ThiaError, ThiaInfo, ThiaQuery, ThiaPlannerCfg, ThiaPlanStats, lib, planner_cfg, plan_from_flags, metrics_from_counts,
                      EXPORTS, TAPS, KERNEL_CLASSES, LIB_PATH)


def thia_load_model(weights, n_exits, device="cuda:0"):
    """weights: uint8 numpy blob (header + fp32 tensors).  Returns the resident model."""
    return Model(weights, n_exits, device)


def thia_detect_chunk(model, frames, ep, out=None):
    """frames: cuda uint8 [n,3,H,W]; ep in 1..n_exits or 0 (skip).  Returns (boxes, scores, labels)."""
    return model.detect_chunk(frames, ep, out)


def thia_run_plan(model, frames, chunk_len, chunk_ep, out=None):
    """frames: cuda uint8 [n_chunks*chunk_len,3,H,W]; chunk_ep: exit per chunk (0 = skip)."""
    return model.run_plan(frames, chunk_len, chunk_ep, out)


def thia_detect_all_exits(model, frames, out=None):
    """frames: cuda uint8 [n,3,H,W]; every exit in one backbone pass.  Returns exit-major (boxes, scores, labels)."""
    return model.detect_all_exits(frames, out)


def thia_run_chunks(model, frames, plan, out=None):
    """plan: [(start, len, exit or 0 = skip), ...] over frames cuda uint8 [n,3,H,W]."""
    return model.run_chunks(frames, plan, out)


def thia_plan_query(model, frames, label, min_count, min_score=0.0, cfg=None):
    """Plan for the query Count(label) >= min_count.  Returns (plan, stats, evaluated mask)."""
    return model.plan_query(frames, label, min_count, min_score, cfg)


def thia_run_query(model, frames, label, min_count, min_score=0.0, cfg=None):
    """Plan, execute and apply the predicate: returns (answers cuda uint8 [n], plan, stats)."""
    return model.run_query(frames, label, min_count, min_score, cfg)


def thia_plan_from_flags(flags, cfg=None):
    """The planner on a host table of per-frame, per-exit answers [n, E]."""
    return plan_from_flags(flags, cfg)


def thia_free_model(model):
    model.close()


def thia_classifier_load(weights, n_exits, device="cuda:0"):
    """weights: uint8 numpy blob of an image classifier with exits.  Returns the resident classifier."""
    return Classifier(weights, n_exits, device)


def thia_classify_chunk(classifier, frames, ep, want_logits=False):
    """frames: cuda uint8 [n,3,H,W]; ep in 1..n_exits or 0 (skip).  Returns (labels, confidence[, logits])."""
    return classifier.classify_chunk(frames, ep, want_logits)
