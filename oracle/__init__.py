"""ctypes access to the CPU oracle (oracle/thia_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The GPU package never imports this module.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None

_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")

TAP_NAMES = ["feat", "head_feat", "rpn_logits", "rpn_deltas", "topk_idx", "topk_n", "prop_boxes", "prop_n",
             "rois", "roi_n", "roi_feat", "cls_logits", "box_deltas", "cand_scores", "cand_boxes", "det_n"]
_INT_TAPS = {"topk_idx", "topk_n", "prop_n", "roi_n", "det_n"}


class _Taps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in TAP_NAMES]


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        L.orc_load.restype = C.c_void_p
        L.orc_load.argtypes = [C.c_void_p, C.c_size_t, C.c_int]
        L.orc_free.argtypes = [C.c_void_p]
        L.orc_round_bf16.restype = C.c_float
        L.orc_round_bf16.argtypes = [C.c_float]
        L.orc_exit_shape.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int] + [C.POINTER(C.c_int)] * 4
        L.orc_normalize.argtypes = [_u8p, C.c_long, C.c_float, C.c_float, C.c_int, _f32p]
        L.orc_conv2d.argtypes = [_f32p] + [C.c_int] * 4 + [_f32p, _f32p] + [C.c_int] * 5 + [C.c_void_p] + [C.c_int] * 3 + [_f32p]
        L.orc_maxpool3x3s2.argtypes = [_f32p] + [C.c_int] * 4 + [_f32p]
        L.orc_fc.argtypes = [_f32p, C.c_int, C.c_int, _f32p, _f32p] + [C.c_int] * 4 + [_f32p]
        L.orc_topk.restype = C.c_int
        L.orc_topk.argtypes = [_f32p, C.c_long, C.c_int, _i32p, _f32p]
        L.orc_anchor.argtypes = [C.c_void_p, C.c_int32, C.c_int, C.c_int, _f32p]
        L.orc_decode.restype = C.c_int
        L.orc_decode.argtypes = [_f32p, _f32p, C.c_float, C.c_float, _f32p]
        L.orc_iou_over.restype = C.c_int
        L.orc_iou_over.argtypes = [_f32p, _f32p, C.c_float]
        L.orc_nms.restype = C.c_int
        L.orc_nms.argtypes = [_f32p, C.c_int, C.c_float, C.c_int, C.c_void_p, _i32p]
        L.orc_roialign.argtypes = [_f32p] + [C.c_int] * 3 + [_f32p] + [C.c_int] * 5 + [_f32p]
        L.orc_softmax.argtypes = [_f32p, C.c_int, C.c_int, _f32p]
        L.orc_select_detections.restype = C.c_int
        L.orc_select_detections.argtypes = [_f32p, _f32p, C.c_int, C.c_int, C.c_float, C.c_float, C.c_int, _f32p, _f32p, _i32p]
        L.orc_backbone.restype = C.POINTER(C.c_float)
        L.orc_backbone.argtypes = [C.c_void_p, _u8p] + [C.c_int] * 4 + [C.c_void_p]
        L.orc_detect.restype = C.c_int
        L.orc_detect.argtypes = [C.c_void_p, _u8p] + [C.c_int] * 4 + [_f32p, _f32p, _i32p, C.c_void_p]
        L.orc_run_plan.restype = C.c_int
        L.orc_detect_all_exits.restype = C.c_int
        L.orc_detect_all_exits.argtypes = [C.c_void_p, _u8p] + [C.c_int] * 3 + [_f32p, _f32p, _i32p]
        L.orc_run_plan.argtypes = [C.c_void_p, _u8p] + [C.c_int] * 4 + [_i32p, _f32p, _f32p, _i32p]
        L.orc_num_threads.restype = C.c_int
        L.free.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def num_threads():
    return int(lib().orc_num_threads())


# ------------------------------------------------------------------ steps
def round_bf16(x):
    x = np.asarray(x, dtype=np.float32)
    return np.vectorize(lambda v: lib().orc_round_bf16(float(v)), otypes=[np.float32])(x)


def normalize(frames, mean=114.0, std=58.0, bf16=0):
    f = _c(frames, np.uint8)
    out = np.empty(f.shape, np.float32)
    lib().orc_normalize(f.reshape(-1), f.size, mean, std, bf16, out.reshape(-1))
    return out


def conv2d(x, w, b, stride=1, pad=0, residual=None, relu=False, bf16_weights=0, round_out=0):
    x, w, b = _c(x, np.float32), _c(w, np.float32), _c(b, np.float32)
    N, Cc, H, W = x.shape
    Co, Ci, kh, kw = w.shape
    assert Ci == Cc
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    out = np.empty((N, Co, Ho, Wo), np.float32)
    res = None
    if residual is not None:
        residual = _c(residual, np.float32)
        assert residual.shape == out.shape
        res = residual.ctypes.data
    lib().orc_conv2d(x, N, Cc, H, W, w, b, Co, kh, kw, stride, pad, res, int(relu), bf16_weights, round_out, out)
    return out


def maxpool3x3s2(x):
    x = _c(x, np.float32)
    N, Cc, H, W = x.shape
    out = np.empty((N, Cc, (H - 1) // 2 + 1, (W - 1) // 2 + 1), np.float32)
    lib().orc_maxpool3x3s2(x, N, Cc, H, W, out)
    return out


def fc(x, w, b, relu=False, bf16_weights=0, round_out=0):
    x, w, b = _c(x, np.float32), _c(w, np.float32), _c(b, np.float32)
    M, K = x.shape
    Nn = w.shape[0]
    out = np.empty((M, Nn), np.float32)
    lib().orc_fc(x, M, K, w, b, Nn, int(relu), bf16_weights, round_out, out)
    return out


def topk(score, k):
    s = _c(score, np.float32).reshape(-1)
    idx = np.empty(max(k, 1), np.int32)
    val = np.empty(max(k, 1), np.float32)
    kk = lib().orc_topk(s, s.size, k, idx, val)
    return idx[:kk].copy(), val[:kk].copy()


def decode(cxcywh, deltas, W, H):
    a, d = _c(cxcywh, np.float32), _c(deltas, np.float32)
    box = np.empty(4, np.float32)
    ok = lib().orc_decode(a, d, float(W), float(H), box)
    return box, bool(ok)


def iou_over(a, b, thr):
    return bool(lib().orc_iou_over(_c(a, np.float32), _c(b, np.float32), float(thr)))


def nms(boxes, thr, max_keep=None, labels=None):
    bx = _c(boxes, np.float32).reshape(-1, 4)
    n = bx.shape[0]
    if max_keep is None:
        max_keep = n
    keep = np.empty(max(max_keep, 1), np.int32)
    lab = None
    if labels is not None:
        labels = _c(labels, np.int32)
        lab = labels.ctypes.data
    nk = lib().orc_nms(bx, n, float(thr), max_keep, lab, keep)
    return keep[:nk].copy()


def roialign(feat, rois, stride, P=7, S=2, round_out=0):
    f, r = _c(feat, np.float32), _c(rois, np.float32).reshape(-1, 4)
    Cc, Hk, Wk = f.shape
    out = np.empty((r.shape[0], Cc, P, P), np.float32)
    lib().orc_roialign(f, Cc, Hk, Wk, r, r.shape[0], stride, P, S, round_out, out)
    return out


def softmax(x):
    x = _c(x, np.float32)
    out = np.empty_like(x)
    lib().orc_softmax(x, x.shape[0], x.shape[1], out)
    return out


def select_detections(scores, boxes, score_thr, nms_thr, D):
    s, b = _c(scores, np.float32), _c(boxes, np.float32)
    R, Kc = s.shape
    ob, osc, ol = np.empty((D, 4), np.float32), np.empty(D, np.float32), np.empty(D, np.int32)
    n = lib().orc_select_detections(s, b, R, Kc, float(score_thr), float(nms_thr), D, ob, osc, ol)
    return ob, osc, ol, n


# ------------------------------------------------------------------ model
class Model:
    def __init__(self, blob, precision=-1):
        blob = np.ascontiguousarray(blob, dtype=np.uint8)
        self._h = lib().orc_load(blob.ctypes.data, blob.nbytes, precision)
        if not self._h:
            raise ValueError("oracle: bad weights blob")
        hi = blob[:256].view(np.int32)
        hf = blob[:256].view(np.float32)
        self.n_exits, self.head_ch, self.has_lateral = int(hi[3]), int(hi[10]), int(hi[9])
        self.A = int(hi[11]) * int(hi[12])
        self.pre, self.post, self.P = int(hi[25]), int(hi[26]), int(hi[28])
        self.Kc, self.D = int(hi[31]), int(hi[34])
        self.precision = int(hi[2]) if precision < 0 else precision
        self.stem_exit = 1 if hi[38] else 0

    def close(self):
        if self._h:
            lib().orc_free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def exit_shape(self, ep, H, W):
        v = [C.c_int() for _ in range(4)]
        lib().orc_exit_shape(self._h, ep, H, W, *[C.byref(x) for x in v])
        return tuple(x.value for x in v)      # C, Hk, Wk, stride

    def anchor(self, i, Wk, stride):
        out = np.empty(4, np.float32)
        lib().orc_anchor(self._h, int(i), Wk, stride, out)
        return out

    def backbone(self, frames, ep, stages=False):
        f = _c(frames, np.uint8)
        n, _, H, W = f.shape
        so = (C.POINTER(C.c_float) * 4)()
        p = lib().orc_backbone(self._h, f, n, H, W, ep, C.cast(so, C.c_void_p) if stages else None)
        Ck, Hk, Wk, _ = self.exit_shape(ep, H, W)
        out = np.ctypeslib.as_array(p, shape=(n, Ck, Hk, Wk)).copy()
        lib().free(p)
        if not stages:
            return out
        st = []
        for s in range(ep - self.stem_exit):
            Cs, Hs, Ws, _ = self.exit_shape(s + 1 + self.stem_exit, H, W)
            st.append(np.ctypeslib.as_array(so[s], shape=(n, Cs, Hs, Ws)).copy())
            lib().free(so[s])
        return out, st

    def detect(self, frames, ep, taps=()):
        f = _c(frames, np.uint8)
        n, _, H, W = f.shape
        D = self.D
        boxes, scores = np.zeros((n, D, 4), np.float32), np.zeros((n, D), np.float32)
        labels = np.full((n, D), -1, np.int32)
        t = _Taps()
        bufs = {}
        if taps and ep > 0:
            Ck, Hk, Wk, _ = self.exit_shape(ep, H, W)
            Ch = self.head_ch if self.has_lateral else Ck
            nA = Hk * Wk * self.A
            shapes = {
                "feat": (n, Ck, Hk, Wk), "head_feat": (n, Ch, Hk, Wk), "rpn_logits": (n, nA),
                "rpn_deltas": (n, nA, 4), "topk_idx": (n, self.pre), "topk_n": (n,),
                "prop_boxes": (n, self.pre, 4), "prop_n": (n,), "rois": (n, self.post, 4), "roi_n": (n,),
                "roi_feat": (n, self.post, Ch * self.P * self.P), "cls_logits": (n, self.post, self.Kc),
                "box_deltas": (n, self.post, 4 * self.Kc), "cand_scores": (n, self.post, self.Kc),
                "cand_boxes": (n, self.post, self.Kc, 4), "det_n": (n,),
            }
            for name in taps:
                dt = np.int32 if name in _INT_TAPS else np.float32
                bufs[name] = np.zeros(shapes[name], dt)
                setattr(t, name, bufs[name].ctypes.data)
        rc = lib().orc_detect(self._h, f, n, H, W, ep, boxes, scores, labels, C.byref(t) if bufs else None)
        if rc:
            raise ValueError("oracle: bad arguments")
        bufs.update(boxes=boxes, scores=scores, labels=labels)
        return bufs

    def detect_all_exits(self, frames):
        f = _c(frames, np.uint8)
        n, _, H, W = f.shape
        E, D = self.n_exits, self.D
        boxes, scores = np.zeros((E, n, D, 4), np.float32), np.zeros((E, n, D), np.float32)
        labels = np.full((E, n, D), -1, np.int32)
        rc = lib().orc_detect_all_exits(self._h, f, n, H, W, boxes, scores, labels)
        if rc:
            raise ValueError("oracle: bad arguments")
        return dict(boxes=boxes, scores=scores, labels=labels)

    def run_plan(self, frames, chunk_len, chunk_ep):
        f = _c(frames, np.uint8)
        n, _, H, W = f.shape
        ce = _c(chunk_ep, np.int32)
        assert n == chunk_len * ce.size
        D = self.D
        boxes, scores = np.zeros((n, D, 4), np.float32), np.zeros((n, D), np.float32)
        labels = np.full((n, D), -1, np.int32)
        rc = lib().orc_run_plan(self._h, f, ce.size, chunk_len, H, W, ce, boxes, scores, labels)
        if rc:
            raise ValueError("oracle: bad plan")
        return dict(boxes=boxes, scores=scores, labels=labels)
