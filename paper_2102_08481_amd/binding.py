"""Thin Python binding of libthia.so (include/thia.h): argument marshalling only.

Device buffers are torch tensors on the current HIP device; every step of the
detector runs inside the library's kernels.  If the shared library is missing or a
symbol cannot be resolved this module raises: there is no fallback path.
"""
import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libthia.so")

THIA_OK = 0
ERRORS = {-1: "THIA_E_BADARG", -2: "THIA_E_BADEP", -3: "THIA_E_SHAPE", -4: "THIA_E_BLOB", -5: "THIA_E_NOMEM", -6: "THIA_E_HIP"}

TAPS = {"feat": 0, "head_feat": 1, "rpn_logits": 2, "rpn_deltas": 3, "topk_idx": 4, "prop_boxes": 5, "prop_n": 6,
        "rois": 7, "roi_n": 8, "roi_feat": 9, "cls_logits": 10, "box_deltas": 11, "cand_scores": 12, "cand_boxes": 13,
        "det_n": 14}
_TAP_ELEM = {"feat": "T", "head_feat": "T", "roi_feat": "T", "topk_idx": "i", "prop_n": "i", "roi_n": "i", "det_n": "i"}
KERNEL_CLASSES = ["stem", "pool", "conv", "fc", "topk", "nms", "roialign", "post", "rpn"]

EXPORTS = ["thia_load_model", "thia_free_model", "thia_set_stream", "thia_set_microbatch", "thia_get_info",
           "thia_detect_chunk", "thia_detect_all_exits", "thia_run_plan", "thia_run_chunks",
           "thia_planner_defaults", "thia_eval_predicate", "thia_plan_from_flags", "thia_plan_query",
           "thia_set_estimator", "thia_estimate_exit", "thia_run_query", "thia_answer_counts", "thia_metrics_from_counts", "thia_last_error", "thia_set_debug", "thia_debug_tap",
           "thia_debug_tap_bytes", "thia_profile_begin", "thia_profile_read", "thia_profile_end",
           "thia_op_rpn_proposals", "thia_op_nms", "thia_op_nms_noalloc", "thia_op_roialign", "thia_op_select_detections", "thia_op_conv",
           "thia_op_stem", "thia_op_bottleneck", "thia_op_bottleneck_tail", "thia_set_fusion", "thia_set_lanes",
           "thia_classifier_load", "thia_classifier_free", "thia_classifier_set_stream", "thia_classifier_last_error",
           "thia_classify_chunk", "thia_classifier_op_pool", "thia_classifier_op_unit"]


class ThiaInfo(C.Structure):
    _fields_ = [("precision", C.c_int32), ("n_exits", C.c_int32), ("blocks", C.c_int32 * 4), ("head_ch", C.c_int32),
                ("n_anchors", C.c_int32), ("pre_nms", C.c_int32), ("post_nms", C.c_int32), ("pool", C.c_int32),
                ("fc_dim", C.c_int32), ("n_classes", C.c_int32), ("max_det", C.c_int32), ("microbatch", C.c_int32),
                ("has_lateral", C.c_int32)]


class ThiaQuery(C.Structure):
    _fields_ = [("label", C.c_int32), ("min_count", C.c_int32), ("min_score", C.c_float)]


class ThiaPlannerCfg(C.Structure):
    _fields_ = [("precision", C.c_double), ("recall", C.c_double), ("min_chunk", C.c_int32), ("final_span", C.c_int32),
                ("posi_enough", C.c_double), ("posi_skip", C.c_double), ("reuse_dist", C.c_int32), ("eval_batch", C.c_int32),
                ("use_estimator", C.c_int32)]


class ThiaPlanStats(C.Structure):
    _fields_ = [("n_chunks", C.c_int32), ("frames_evaluated", C.c_int32), ("samples_reused", C.c_int32), ("depth", C.c_int32),
                ("eval_batches", C.c_int32)]


class ThiaError(RuntimeError):
    def __init__(self, code, msg=""):
        super().__init__(f"{ERRORS.get(code, code)}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load libthia.so (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    L.thia_load_model.argtypes = [vp, sz, i32, C.POINTER(vp)]
    L.thia_free_model.argtypes = [vp]
    L.thia_free_model.restype = None
    L.thia_set_stream.argtypes = [vp, vp]
    L.thia_set_microbatch.argtypes = [vp, i32]
    L.thia_get_info.argtypes = [vp, C.POINTER(ThiaInfo)]
    L.thia_detect_chunk.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp]
    L.thia_detect_all_exits.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    L.thia_run_plan.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
    L.thia_run_chunks.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    L.thia_planner_defaults.argtypes = [C.POINTER(ThiaPlannerCfg)]
    L.thia_planner_defaults.restype = None
    L.thia_eval_predicate.argtypes = [vp, vp, vp, i32, C.POINTER(ThiaQuery), vp]
    L.thia_plan_from_flags.argtypes = [vp, i32, i32, C.POINTER(ThiaPlannerCfg), i32, vp, vp, vp, C.POINTER(ThiaPlanStats), vp]
    L.thia_plan_query.argtypes = [vp, vp, i32, i32, i32, C.POINTER(ThiaQuery), C.POINTER(ThiaPlannerCfg), i32, vp, vp, vp,
                                  C.POINTER(ThiaPlanStats), vp]
    L.thia_set_estimator.argtypes = [vp, i32, vp, vp, vp, vp]
    L.thia_estimate_exit.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp]
    L.thia_answer_counts.argtypes = [vp, vp, vp, i32, vp]
    L.thia_metrics_from_counts.argtypes = [vp, vp]
    L.thia_metrics_from_counts.restype = None
    L.thia_run_query.argtypes = [vp, vp, i32, i32, i32, C.POINTER(ThiaQuery), C.POINTER(ThiaPlannerCfg), vp, i32, vp, vp, vp,
                                 C.POINTER(ThiaPlanStats)]
    L.thia_last_error.argtypes = [vp]
    L.thia_last_error.restype = C.c_char_p
    L.thia_set_debug.argtypes = [vp, i32]
    L.thia_debug_tap.argtypes = [vp, i32, vp, sz]
    L.thia_debug_tap_bytes.argtypes = [vp, i32]
    L.thia_debug_tap_bytes.restype = sz
    L.thia_profile_begin.argtypes = [vp]
    L.thia_profile_read.argtypes = [vp, vp, vp]
    L.thia_profile_end.argtypes = [vp]
    L.thia_op_rpn_proposals.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
    L.thia_op_nms.argtypes = [vp, vp, vp, i32, i32, C.c_float, i32, vp, vp]
    L.thia_op_nms_noalloc.argtypes = [vp, vp, vp, i32, i32, C.c_float, i32, vp, vp]
    L.thia_op_roialign.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
    L.thia_op_select_detections.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp, vp]
    L.thia_op_conv.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, i32, i32, i32, i32, vp, i32, i32, vp]
    L.thia_op_stem.argtypes = [vp, vp, i32, i32, i32, vp]
    L.thia_op_bottleneck.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.thia_op_bottleneck_tail.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp]
    L.thia_set_fusion.argtypes = [vp, i32]
    L.thia_set_lanes.argtypes = [vp, i32]
    L.thia_classifier_load.argtypes = [vp, sz, i32, C.POINTER(vp)]
    L.thia_classifier_free.argtypes = [vp]
    L.thia_classifier_free.restype = None
    L.thia_classifier_set_stream.argtypes = [vp, vp]
    L.thia_classifier_last_error.argtypes = [vp]
    L.thia_classifier_last_error.restype = C.c_char_p
    L.thia_classify_chunk.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp]
    L.thia_classifier_op_pool.argtypes = [vp, vp, i32, i32, i32, i32, vp]
    L.thia_classifier_op_unit.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    for name in EXPORTS:
        getattr(L, name)
    _lib = L
    return L


def planner_cfg(**overrides):
    """thia_planner_cfg with the library's defaults, fields overridden by keyword."""
    cfg = ThiaPlannerCfg()
    lib().thia_planner_defaults(C.byref(cfg))
    for k, v in overrides.items():
        if k not in dict(ThiaPlannerCfg._fields_):
            raise KeyError(k)
        setattr(cfg, k, v)
    return cfg


def _plan_buffers(n, cfg):
    cap = max(1, 2 * (n // max(1, cfg.min_chunk)) + 2)
    return cap, [np.zeros(cap, np.int32) for _ in range(3)], ThiaPlanStats(), np.zeros(max(n, 1), np.uint8)


def _plan_result(bufs, stats, evaluated, n):
    k = stats.n_chunks
    plan = [(int(bufs[0][i]), int(bufs[1][i]), int(bufs[2][i])) for i in range(k)]
    st = {name: int(getattr(stats, name)) for name, _ in ThiaPlanStats._fields_}
    return plan, st, evaluated[:n].astype(bool)


def plan_from_flags(flags, cfg=None):
    """thia_plan_from_flags: flags [n, E] (host) -> (plan [(start, len, exit or 0)], stats dict, evaluated mask [n])."""
    flags = np.ascontiguousarray(flags, dtype=np.uint8)
    n, E = flags.shape
    cfg = cfg or planner_cfg()
    cap, bufs, stats, ev = _plan_buffers(n, cfg)
    rc = lib().thia_plan_from_flags(flags.ctypes.data, n, E, C.byref(cfg), cap, bufs[0].ctypes.data, bufs[1].ctypes.data,
                                    bufs[2].ctypes.data, C.byref(stats), ev.ctypes.data)
    if rc:
        raise ThiaError(rc, "thia_plan_from_flags")
    return _plan_result(bufs, stats, ev, n)


def metrics_from_counts(counts):
    """thia_metrics_from_counts: (TP, FP, FN) -> (precision, recall, F-1)."""
    c = np.ascontiguousarray(counts, dtype=np.int32)
    out = np.zeros(3, np.float64)
    lib().thia_metrics_from_counts(c.ctypes.data, out.ctypes.data)
    return tuple(float(x) for x in out)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dev(t, dtype):
    assert t.is_cuda and t.dtype == dtype and t.is_contiguous(), (t.device, t.dtype, dtype)
    return t


class Model:
    """One resident multi-exit detector (thia_model*)."""

    def __init__(self, blob, n_exits, device="cuda:0"):
        blob = np.ascontiguousarray(blob, dtype=np.uint8)
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        torch.zeros(1, device=self.device)          # make sure the HIP context exists
        self._h = C.c_void_p()
        rc = lib().thia_load_model(blob.ctypes.data, blob.nbytes, n_exits, C.byref(self._h))
        if rc:
            self._h = None
            raise ThiaError(rc, "thia_load_model")
        self.info = ThiaInfo()
        self._check(lib().thia_get_info(self._h, C.byref(self.info)))
        self.precision = self.info.precision
        self.n_exits = self.info.n_exits
        self.elem = torch.bfloat16 if self.precision else torch.float32
        self.D = self.info.max_det
        self.set_stream(torch.cuda.current_stream(self.device))

    # -- lifetime
    def close(self):
        if getattr(self, "_h", None):
            lib().thia_free_model(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc:
            raise ThiaError(rc, lib().thia_last_error(self._h).decode())

    def refresh_info(self):
        self._check(lib().thia_get_info(self._h, C.byref(self.info)))
        return self.info

    # -- the boundary calls
    def set_stream(self, stream):
        self._check(lib().thia_set_stream(self._h, C.c_void_p(stream.cuda_stream if stream is not None else 0)))

    def set_microbatch(self, frames):
        self._check(lib().thia_set_microbatch(self._h, frames))

    def alloc_outputs(self, n):
        D = self.D
        return (torch.empty((n, D, 4), dtype=torch.float32, device=self.device),
                torch.empty((n, D), dtype=torch.float32, device=self.device),
                torch.empty((n, D), dtype=torch.int32, device=self.device))

    def detect_chunk(self, frames, ep, out=None):
        """frames: cuda uint8 [n,3,H,W]; returns (boxes [n,D,4], scores [n,D], labels [n,D]) on the device."""
        _dev(frames, torch.uint8)
        n, c, H, W = frames.shape
        assert c == 3
        out = out or self.alloc_outputs(n)
        self._check(lib().thia_detect_chunk(self._h, _ptr(frames), n, H, W, ep, _ptr(out[0]), _ptr(out[1]), _ptr(out[2])))
        return out

    def detect_all_exits(self, frames, out=None):
        """frames: cuda uint8 [n,3,H,W]; returns (boxes [E,n,D,4], scores [E,n,D], labels [E,n,D]), E = n_exits."""
        _dev(frames, torch.uint8)
        n, c, H, W = frames.shape
        assert c == 3
        if out is None:
            b, s, l = self.alloc_outputs(self.n_exits * n)
            out = (b.view(self.n_exits, n, self.D, 4), s.view(self.n_exits, n, self.D), l.view(self.n_exits, n, self.D))
        self._check(lib().thia_detect_all_exits(self._h, _ptr(frames), n, H, W, _ptr(out[0]), _ptr(out[1]), _ptr(out[2])))
        return out

    def run_plan(self, frames, chunk_len, chunk_ep, out=None):
        _dev(frames, torch.uint8)
        n, c, H, W = frames.shape
        ce = np.ascontiguousarray(chunk_ep, dtype=np.int32)
        assert c == 3 and n == chunk_len * ce.size
        out = out or self.alloc_outputs(n)
        self._check(lib().thia_run_plan(self._h, _ptr(frames), ce.size, chunk_len, H, W, ce.ctypes.data, _ptr(out[0]),
                                        _ptr(out[1]), _ptr(out[2])))
        return out

    def run_chunks(self, frames, plan, out=None):
        """plan: [(start, len, exit or 0 = skip), ...]; outputs as for detect_chunk on all frames."""
        _dev(frames, torch.uint8)
        n, c, H, W = frames.shape
        assert c == 3
        st, ln, ep = (np.ascontiguousarray([p[i] for p in plan], dtype=np.int32) for i in range(3))
        out = out or self.alloc_outputs(n)
        self._check(lib().thia_run_chunks(self._h, _ptr(frames), n, H, W, len(plan), st.ctypes.data, ln.ctypes.data, ep.ctypes.data,
                                          _ptr(out[0]), _ptr(out[1]), _ptr(out[2])))
        return out

    def eval_predicate(self, labels, scores, label, min_count, min_score=0.0):
        """Count(label) >= min_count per row of detection slots: labels int32 [..., D], scores float32 [..., D] -> uint8 [...]."""
        _dev(labels, torch.int32)
        _dev(scores, torch.float32)
        assert labels.shape == scores.shape and labels.shape[-1] == self.D
        rows = labels.numel() // self.D
        flags = torch.empty(labels.shape[:-1], dtype=torch.uint8, device=self.device)
        q = ThiaQuery(label, min_count, min_score)
        self._check(lib().thia_eval_predicate(self._h, _ptr(labels), _ptr(scores), rows, C.byref(q), _ptr(flags)))
        return flags

    def answer_counts(self, answers, reference):
        """(TP, FP, FN) of answers against reference answers (cuda uint8 [n] each), as a device int32 [3] tensor."""
        _dev(answers, torch.uint8)
        _dev(reference, torch.uint8)
        assert answers.shape == reference.shape
        counts = torch.empty(3, dtype=torch.int32, device=self.device)
        self._check(lib().thia_answer_counts(self._h, _ptr(answers), _ptr(reference), answers.numel(), _ptr(counts)))
        return counts

    def set_estimator(self, w1, b1, w2, b2):
        """Two-layer exit estimator: w1 [hidden, C_last], b1 [hidden], w2 [n_exits, hidden], b2 [n_exits] (host); None removes it."""
        if w1 is None:
            self._check(lib().thia_set_estimator(self._h, 0, None, None, None, None))
            return
        a = [np.ascontiguousarray(x, dtype=np.float32) for x in (w1, b1, w2, b2)]
        hidden = a[0].shape[0]
        assert a[1].shape == (hidden,) and a[2].shape == (self.n_exits, hidden) and a[3].shape == (self.n_exits,)
        self._check(lib().thia_set_estimator(self._h, hidden, *[x.ctypes.data for x in a]))

    def estimate_exit(self, frames, out=None):
        """Returns (opt_ep int32 [n], logits float32 [n, E], (boxes, scores, labels) of the last exit)."""
        _dev(frames, torch.uint8)
        n, c, H, W = frames.shape
        assert c == 3
        opt = torch.empty(n, dtype=torch.int32, device=self.device)
        logits = torch.empty((n, self.n_exits), dtype=torch.float32, device=self.device)
        out = out or self.alloc_outputs(n)
        self._check(lib().thia_estimate_exit(self._h, _ptr(frames), n, H, W, _ptr(opt), _ptr(logits), _ptr(out[0]), _ptr(out[1]),
                                             _ptr(out[2])))
        return opt, logits, out

    def plan_query(self, frames, label, min_count, min_score=0.0, cfg=None):
        """thia_plan_query on resident frames -> (plan, stats dict, evaluated mask [n])."""
        _dev(frames, torch.uint8)
        n, c, H, W = frames.shape
        assert c == 3
        cfg = cfg or planner_cfg()
        cap, bufs, stats, ev = _plan_buffers(n, cfg)
        q = ThiaQuery(label, min_count, min_score)
        self._check(lib().thia_plan_query(self._h, _ptr(frames), n, H, W, C.byref(q), C.byref(cfg), cap, bufs[0].ctypes.data,
                                          bufs[1].ctypes.data, bufs[2].ctypes.data, C.byref(stats), ev.ctypes.data))
        return _plan_result(bufs, stats, ev, n)

    def run_query(self, frames, label, min_count, min_score=0.0, cfg=None):
        """thia_run_query -> (answers cuda uint8 [n], plan, stats dict)."""
        _dev(frames, torch.uint8)
        n, c, H, W = frames.shape
        assert c == 3
        cfg = cfg or planner_cfg()
        cap, bufs, stats, _ = _plan_buffers(n, cfg)
        answers = torch.zeros(n, dtype=torch.uint8, device=self.device)
        q = ThiaQuery(label, min_count, min_score)
        self._check(lib().thia_run_query(self._h, _ptr(frames), n, H, W, C.byref(q), C.byref(cfg), _ptr(answers), cap,
                                         bufs[0].ctypes.data, bufs[1].ctypes.data, bufs[2].ctypes.data, C.byref(stats)))
        plan, st, _ = _plan_result(bufs, stats, np.zeros(max(n, 1), np.uint8), n)
        return answers, plan, st

    # -- inspection
    def set_debug(self, on):
        self._check(lib().thia_set_debug(self._h, int(on)))

    def tap(self, name):
        """Flat numpy array of a recorded intermediate (float32 / int32; bf16 taps are widened to float32)."""
        which = TAPS[name]
        nbytes = lib().thia_debug_tap_bytes(self._h, which)
        kind = _TAP_ELEM.get(name, "f")
        if kind == "T" and self.precision:
            raw = np.empty(nbytes // 2, np.uint16)
        elif kind == "i":
            raw = np.empty(nbytes // 4, np.int32)
        else:
            raw = np.empty(nbytes // 4, np.float32)
        self._check(lib().thia_debug_tap(self._h, which, raw.ctypes.data, nbytes))
        if raw.dtype == np.uint16:
            return (raw.astype(np.uint32) << 16).view(np.float32)
        return raw

    def profile_begin(self):
        self._check(lib().thia_profile_begin(self._h))

    def profile_read(self):
        ms = np.zeros(len(KERNEL_CLASSES), np.float32)
        cnt = np.zeros(len(KERNEL_CLASSES), np.int32)
        self._check(lib().thia_profile_read(self._h, ms.ctypes.data, cnt.ctypes.data))
        return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(KERNEL_CLASSES)}

    def profile_end(self):
        self._check(lib().thia_profile_end(self._h))

    # -- single steps
    def op_rpn_proposals(self, logits, deltas, H, W, ep):
        _dev(logits, torch.float32), _dev(deltas, torch.float32)
        n, pre = logits.shape[0], self.info.pre_nms
        idx = torch.empty((n, pre), dtype=torch.int32, device=self.device)
        boxes = torch.empty((n, pre, 4), dtype=torch.float32, device=self.device)
        cnt = torch.empty((n,), dtype=torch.int32, device=self.device)
        self._check(lib().thia_op_rpn_proposals(self._h, _ptr(logits), _ptr(deltas), n, H, W, ep, _ptr(idx), _ptr(boxes), _ptr(cnt)))
        return idx, boxes, cnt

    def op_nms(self, boxes, counts, thr, max_keep):
        _dev(boxes, torch.float32), _dev(counts, torch.int32)
        n, cap = boxes.shape[0], boxes.shape[1]
        keep = torch.empty((n, max_keep), dtype=torch.int32, device=self.device)
        cnt = torch.empty((n,), dtype=torch.int32, device=self.device)
        self._check(lib().thia_op_nms(self._h, _ptr(boxes), _ptr(counts), n, cap, thr, max_keep, _ptr(keep), _ptr(cnt)))
        return keep, cnt

    def op_nms_noalloc(self, boxes, counts, thr, max_keep, keep, cnt):
        """Same as op_nms, into caller tensors keep int32 [n,max_keep] and cnt int32 [n]; the library allocates nothing."""
        _dev(boxes, torch.float32), _dev(counts, torch.int32), _dev(keep, torch.int32), _dev(cnt, torch.int32)
        n, cap = boxes.shape[0], boxes.shape[1]
        if tuple(keep.shape) != (n, max_keep) or tuple(cnt.shape) != (n,):
            raise ValueError("keep must be [n, max_keep] and cnt [n]")
        self._check(lib().thia_op_nms_noalloc(self._h, _ptr(boxes), _ptr(counts), n, cap, thr, max_keep, _ptr(keep), _ptr(cnt)))
        return keep, cnt

    def op_roialign(self, feat, rois, stride):
        _dev(feat, self.elem), _dev(rois, torch.float32)
        n, Hk, Wk, Ch = feat.shape
        P = self.info.pool
        out = torch.empty((n, self.info.post_nms, P * P, Ch), dtype=self.elem, device=self.device)
        self._check(lib().thia_op_roialign(self._h, _ptr(feat), _ptr(rois), n, Hk, Wk, stride, _ptr(out)))
        return out

    def op_select_detections(self, scores, boxes, roi_n):
        _dev(scores, torch.float32), _dev(boxes, torch.float32), _dev(roi_n, torch.int32)
        n = scores.shape[0]
        out = self.alloc_outputs(n)
        cnt = torch.empty((n,), dtype=torch.int32, device=self.device)
        self._check(lib().thia_op_select_detections(self._h, _ptr(scores), _ptr(boxes), _ptr(roi_n), n, _ptr(out[0]),
                                                    _ptr(out[1]), _ptr(out[2]), _ptr(cnt)))
        return out + (cnt,)

    def op_conv(self, x, w, b, stride=1, pad=0, residual=None, relu=False, out_f32=False):
        """x: cuda [n,H,W,Cin] in the model's element type; w: numpy [Cout,Cin,k,k]; b: numpy [Cout]."""
        _dev(x, self.elem)
        n, H, W, Cin = x.shape
        w = np.ascontiguousarray(w, dtype=np.float32)
        b = np.ascontiguousarray(b, dtype=np.float32)
        Cout, _, k, _ = w.shape
        Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
        out = torch.empty((n, Ho, Wo, Cout), dtype=torch.float32 if out_f32 else self.elem, device=self.device)
        if residual is not None:
            _dev(residual, self.elem)
        self._check(lib().thia_op_conv(self._h, _ptr(x), n, H, W, Cin, w.ctypes.data, b.ctypes.data, Cout, k, stride, pad,
                                       _ptr(residual), int(relu), int(out_f32), _ptr(out)))
        return out

    def set_fusion(self, on):
        self._check(lib().thia_set_fusion(self._h, int(on)))   # 0 off, 1 where it pays (default), 2 wherever it applies

    def set_lanes(self, lanes):
        self._check(lib().thia_set_lanes(self._h, int(lanes)))   # 2 (default): micro-batches alternate between two streams

    def op_bottleneck(self, x, w1, b1, w2, b2, w3, b3, ws=None, bs=None):
        """x: cuda bf16 [n,H,W,Cin]; weights numpy fp32 in [Cout,Cin,k,k] order; ws/bs: projection shortcut."""
        _dev(x, self.elem)
        n, H, W, _ = x.shape
        width = np.asarray(w2).shape[0]
        arrs = [None if v is None else np.ascontiguousarray(v, dtype=np.float32) for v in (w1, b1, w2, b2, w3, b3, ws, bs)]
        out = torch.empty((n, H, W, 4 * width), dtype=self.elem, device=self.device)
        self._check(lib().thia_op_bottleneck(self._h, _ptr(x), n, H, W, width, *[None if v is None else v.ctypes.data for v in arrs],
                                             _ptr(out)))
        return out

    def op_bottleneck_tail(self, x, w1, b1, w2, b2, w3, b3, wt, bt, relu):
        """64-wide identity block plus the 1x1 tail layer wt [N,256,1,1] (N = 128 or 256) on its output: returns (y, z)."""
        _dev(x, self.elem)
        n, H, W, _ = x.shape
        arrs = [np.ascontiguousarray(v, dtype=np.float32) for v in (w1, b1, w2, b2, w3, b3, wt, bt)]
        tail_n = arrs[6].shape[0]
        out = torch.empty((n, H, W, 256), dtype=self.elem, device=self.device)
        out_tail = torch.empty((n, H, W, tail_n), dtype=self.elem, device=self.device)
        self._check(lib().thia_op_bottleneck_tail(self._h, _ptr(x), n, H, W, *[v.ctypes.data for v in arrs], tail_n, int(relu),
                                                  _ptr(out), _ptr(out_tail)))
        return out, out_tail

    def op_stem(self, frames):
        _dev(frames, torch.uint8)
        n, _, H, W = frames.shape
        Hs, Ws = (H - 1) // 2 + 1, (W - 1) // 2 + 1
        Hp, Wp = (Hs - 1) // 2 + 1, (Ws - 1) // 2 + 1
        out = torch.empty((n, Hp, Wp, 64), dtype=self.elem, device=self.device)
        self._check(lib().thia_op_stem(self._h, _ptr(frames), n, H, W, _ptr(out)))
        return out


class Classifier:
    """One resident image classifier with exits (thia_classifier*): argument marshalling only."""

    def __init__(self, blob, n_exits, device="cuda:0"):
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        blob = np.ascontiguousarray(blob, dtype=np.uint8)
        h = C.c_void_p()
        rc = lib().thia_classifier_load(blob.ctypes.data, blob.nbytes, n_exits, C.byref(h))
        if rc:
            raise ThiaError(rc, "thia_classifier_load")
        self._h = h
        hi = blob[:256].view(np.int32)
        self.precision, self.n_exits, self.n_classes = int(hi[2]), int(hi[3]), int(hi[6])
        self.elem = torch.bfloat16 if self.precision else torch.float32
        lib().thia_classifier_set_stream(self._h, C.c_void_p(torch.cuda.current_stream().cuda_stream))

    def _check(self, rc):
        if rc:
            raise ThiaError(rc, (lib().thia_classifier_last_error(self._h) or b"").decode())

    def classify_chunk(self, frames, ep, want_logits=False):
        """frames cuda uint8 [n,3,H,W] -> (labels int32 [n], confidence float32 [n][, logits float32 [n,classes]])."""
        _dev(frames, torch.uint8)
        n, c, H, W = frames.shape
        assert c == 3
        labels = torch.empty((n,), dtype=torch.int32, device=self.device)
        conf = torch.empty((n,), dtype=torch.float32, device=self.device)
        logits = torch.empty((n, self.n_classes), dtype=torch.float32, device=self.device) if want_logits else None
        self._check(lib().thia_classify_chunk(self._h, _ptr(frames), n, H, W, ep, _ptr(labels), _ptr(conf), _ptr(logits)))
        return (labels, conf, logits) if want_logits else (labels, conf)

    def op_pool(self, x):
        _dev(x, self.elem)
        n, H, W, Cc = x.shape
        out = torch.empty((n, H // 2, W // 2, Cc), dtype=self.elem, device=self.device)
        self._check(lib().thia_classifier_op_pool(self._h, _ptr(x), n, H, W, Cc, _ptr(out)))
        return out

    def op_unit(self, feat, ep):
        """feat cuda [n,HW,C_tap] -> (labels, confidence, logits)."""
        _dev(feat, self.elem)
        n, HW = feat.shape[0], feat.shape[1]
        labels = torch.empty((n,), dtype=torch.int32, device=self.device)
        conf = torch.empty((n,), dtype=torch.float32, device=self.device)
        logits = torch.empty((n, self.n_classes), dtype=torch.float32, device=self.device)
        self._check(lib().thia_classifier_op_unit(self._h, _ptr(feat), n, HW, ep, _ptr(labels), _ptr(conf), _ptr(logits)))
        return labels, conf, logits

    def close(self):
        if self._h:
            lib().thia_classifier_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
