"""ctypes face of the CPU oracle (oracle/cnnc_oracle.c) plus the few steps that
are plain array bookkeeping (flat window index <-> (level, y, x), score
quantiles, running the stages one after another).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; never by the product package.
"""
import ctypes as C
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import build as _build

WINDOW = 12          # side of the stage-1 window (benchmark's default cascade)
MAX_LEVELS = 64


class _Layer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("cin", C.c_int32), ("cout", C.c_int32),
                ("k", C.c_int32), ("act", C.c_int32)]


class _RLayer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("cin", C.c_int32), ("cout", C.c_int32),
                ("kw", C.c_int32), ("kh", C.c_int32), ("act", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        L.orc_rational_tanh.restype = C.c_double
        L.orc_rational_tanh.argtypes = [C.c_double]
        L.orc_activation.restype = C.c_double
        L.orc_activation.argtypes = [C.c_double, C.c_int]
        L.orc_survivors.restype = C.c_int64
        L.orc_merge.restype = C.c_int32
        L.orc_merge_rect.restype = C.c_int32
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _layers(stage):
    arr = (_Layer * len(stage.layers))()
    for i, l in enumerate(stage.layers):
        arr[i] = _Layer(l.kind, l.cin, l.cout, l.k, l.act)
    return arr


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    """Threads of the oracle's parallel loops from now on (timing reports only; results do not depend on it)."""
    lib().orc_set_num_threads(C.c_int(int(n)))


def rational_tanh(y: float) -> float:
    return lib().orc_rational_tanh(float(y))


def activation(x: float, act: int) -> float:
    return lib().orc_activation(float(x), int(act))


# --------------------------------------------------------------------------
@dataclass
class Pyramid:
    width: int
    height: int
    lvl_w: List[int]
    lvl_h: List[int]
    scale: List[float]
    levels: List[np.ndarray] = field(default_factory=list)

    @property
    def n_levels(self) -> int:
        return len(self.lvl_w)

    @property
    def windows_per_level(self) -> List[int]:
        return [(w - WINDOW + 1) * (h - WINDOW + 1) for w, h in zip(self.lvl_w, self.lvl_h)]

    @property
    def score_off(self) -> List[int]:
        """Start of each level in the flat window index (level, then y, then x); last entry = total."""
        off = [0]
        for n in self.windows_per_level:
            off.append(off[-1] + n)
        return off

    def decode(self, idx: np.ndarray):
        """Flat window indices -> (level, y, x) arrays."""
        idx = np.asarray(idx, np.int64)
        off = np.asarray(self.score_off, np.int64)
        lvl = np.searchsorted(off, idx, side="right") - 1
        rem = idx - off[lvl]
        ow = np.asarray(self.lvl_w, np.int64)[lvl] - WINDOW + 1
        return lvl.astype(np.int32), (rem // ow).astype(np.int32), (rem % ow).astype(np.int32)


def pyramid_layout(width: int, height: int, min_face: float, scale_step: float) -> Pyramid:
    lw = np.zeros(MAX_LEVELS, np.int32)
    lh = np.zeros(MAX_LEVELS, np.int32)
    sc = np.zeros(MAX_LEVELS, np.float64)
    n = lib().orc_pyramid_layout(C.c_int(width), C.c_int(height), C.c_double(min_face),
                                 C.c_double(scale_step), C.c_int(WINDOW), C.c_int(MAX_LEVELS),
                                 _p(lw), _p(lh), _p(sc))
    if n < 0:
        raise ValueError("bad pyramid arguments")
    return Pyramid(width, height, lw[:n].tolist(), lh[:n].tolist(), sc[:n].tolist())


def resample_level(frame: np.ndarray, scale: float, lw: int, lh: int) -> np.ndarray:
    assert frame.dtype == np.uint8 and frame.ndim == 2 and frame.strides[1] == 1
    out = np.empty((lh, lw), np.uint8)
    lib().orc_resample_level(_p(frame), C.c_int(frame.shape[1]), C.c_int(frame.shape[0]),
                             C.c_int(frame.strides[0]), C.c_double(scale), C.c_int(lw), C.c_int(lh),
                             _p(out))
    return out


def build_pyramid(frame: np.ndarray, min_face: float, scale_step: float) -> Pyramid:
    pyr = pyramid_layout(frame.shape[1], frame.shape[0], min_face, scale_step)
    pyr.levels = [resample_level(frame, s, w, h) for s, w, h in zip(pyr.scale, pyr.lvl_w, pyr.lvl_h)]
    return pyr


# --------------------------------------------------------------------------
def net_forward(stage, weights: np.ndarray, window: np.ndarray) -> np.ndarray:
    """One network on one already normalised window (in_size x in_size float64)."""
    window = np.ascontiguousarray(window, np.float64)
    assert window.shape == (stage.in_size, stage.in_size)
    weights = np.ascontiguousarray(weights, np.float32)
    assert weights.size == stage.n_params
    last = [l for l in stage.layers][-1]
    out = np.zeros(last.cout, np.float64)
    rc = lib().orc_net_forward(_layers(stage), C.c_int(len(stage.layers)), _p(weights),
                               C.c_int(stage.in_size), _p(window), _p(out))
    if rc != 0:
        raise ValueError("layer list does not fit the input")
    return out


def stage1_level(level: np.ndarray, stage, weights: np.ndarray, form: str = "dense") -> np.ndarray:
    """Score map of one pyramid level, (H-11) x (W-11) float64."""
    level = np.ascontiguousarray(level, np.uint8)
    weights = np.ascontiguousarray(weights, np.float32)
    assert weights.size == stage.n_params
    lh, lw = level.shape
    out = np.zeros((lh - stage.in_size + 1, lw - stage.in_size + 1), np.float64)
    fn = {"dense": lib().orc_stage1_dense, "windows": lib().orc_stage1_windows}[form]
    rc = fn(_p(level), C.c_int(lw), C.c_int(lh), _layers(stage), C.c_int(len(stage.layers)),
            _p(weights), C.c_int(stage.in_size), _p(out))
    if rc != 0:
        raise ValueError("stage-1 evaluation failed")
    return out


def _rlayers(net):
    arr = (_RLayer * len(net.layers))()
    for i, l in enumerate(net.layers):
        arr[i] = _RLayer(l.kind, l.cin, l.cout, l.kw, l.kh, l.act)
    return arr


def scan_window(net, weights: np.ndarray, window: np.ndarray) -> float:
    """The scanning network on one normalised window (win_h x win_w float64): its single response."""
    window = np.ascontiguousarray(window, np.float64)
    assert window.shape == (net.win_h, net.win_w)
    weights = np.ascontiguousarray(weights, np.float32)
    assert weights.size == net.n_params
    out = np.zeros(1, np.float64)
    rc = lib().orc_rnet_forward(_rlayers(net), C.c_int(len(net.layers)), _p(weights), C.c_int(net.win_w),
                                C.c_int(net.win_h), _p(window), _p(out))
    if rc != 0:
        raise ValueError("layer list does not take the window to one response")
    return float(out[0])


def scan_level(level: np.ndarray, net, weights: np.ndarray, form: str = "fcn") -> np.ndarray:
    """Responses of the scanning network on one level: ((H - win_h) // step + 1) x ((W - win_w) // step + 1)
    float64; an empty array when the level is smaller than the window."""
    level = np.ascontiguousarray(level, np.uint8)
    weights = np.ascontiguousarray(weights, np.float32)
    assert weights.size == net.n_params
    lh, lw = level.shape
    if lw < net.win_w or lh < net.win_h:
        return np.zeros((0, 0), np.float64)
    out = np.zeros(((lh - net.win_h) // net.step + 1, (lw - net.win_w) // net.step + 1), np.float64)
    if form == "fcn":
        rc = lib().orc_scan_fcn(_p(level), C.c_int(lw), C.c_int(lh), _rlayers(net), C.c_int(len(net.layers)),
                                _p(weights), C.c_int(net.win_w), C.c_int(net.win_h), _p(out))
    else:
        rc = lib().orc_scan_windows(_p(level), C.c_int(lw), C.c_int(lh), _rlayers(net), C.c_int(len(net.layers)),
                                    _p(weights), C.c_int(net.win_w), C.c_int(net.win_h), C.c_int(net.step), _p(out))
    if rc != 0:
        raise ValueError("scan failed")
    return out


def scan_scores(pyr: Pyramid, net, weights: np.ndarray, form: str = "fcn") -> np.ndarray:
    """All responses of a frame's pyramid, flat in (level, row, column) order."""
    return np.concatenate([scan_level(l, net, weights, form).ravel() for l in pyr.levels] + [np.zeros(0)])


def region(frame: np.ndarray, x0: int, y0: int, scale: float, rw: int, rh: int) -> np.ndarray:
    """rh x rw uint8 region whose corner is (x0, y0) in level coordinates, resampled from the frame."""
    frame = np.ascontiguousarray(frame, np.uint8)
    out = np.zeros((rh, rw), np.uint8)
    lib().orc_region(_p(frame), C.c_int(frame.shape[1]), C.c_int(frame.shape[0]), C.c_int(frame.strides[0]), C.c_int(int(x0)),
                     C.c_int(int(y0)), C.c_double(float(scale)), C.c_int(rw), C.c_int(rh), _p(out))
    return out


def histeq(img: np.ndarray) -> np.ndarray:
    out = np.ascontiguousarray(img, np.uint8).copy()
    lib().orc_histeq(_p(out), C.c_int(out.size))
    return out


def select_region(reg: np.ndarray, net2, w2: np.ndarray, net3, w3: np.ndarray, t2: float, t3: float, t_nn: int,
                  rule: int = 2):
    """One equalised region through CNN_2 / CNN_3 and the decision rule (2) or (3): (K2, K3, face, r2, r3)."""
    reg = np.ascontiguousarray(reg, np.uint8)
    w2 = np.ascontiguousarray(w2, np.float32)
    w3 = np.ascontiguousarray(w3, np.float32)
    assert w2.size == net2.n_params and w3.size == net3.n_params
    rh, rw = reg.shape
    nh, nw = (rh - net2.win_h) // net2.step + 1, (rw - net2.win_w) // net2.step + 1
    k2, k3, face = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    r2 = np.zeros((nh, nw), np.float64)
    r3 = np.zeros((nh, nw), np.float64)
    rc = lib().orc_select_region(_p(reg), C.c_int(rw), C.c_int(rh), _rlayers(net2), C.c_int(len(net2.layers)), _p(w2),
                                 _rlayers(net3), C.c_int(len(net3.layers)), _p(w3), C.c_int(net2.win_w), C.c_int(net2.win_h),
                                 C.c_float(t2), C.c_float(t3), C.c_int(t_nn), C.c_int(rule), C.byref(k2), C.byref(k3), C.byref(face),
                                 _p(r2), _p(r3))
    if rc != 0:
        raise ValueError("a network does not fit the region")
    return k2.value, k3.value, bool(face.value), r2, r3


def select_unit(frame: np.ndarray, pyr: Pyramid, scan_idx: np.ndarray, net1, net2, w2, net3, w3, t2: float, t3: float,
                t_nn: int, rw: int = 51, rh: int = 55, margin: int = 12, rule: int = 2):
    """The selective unit for the scan responses with flat indices scan_idx: list of dicts (index, level, i, j, k2, k3,
    face, r2, r3) in that order.  The region of window (i, j) of a level is the window plus `margin` level pixels."""
    sizes = [((l.shape[0] - net1.win_h) // net1.step + 1, (l.shape[1] - net1.win_w) // net1.step + 1)
             if l.shape[0] >= net1.win_h and l.shape[1] >= net1.win_w else (0, 0) for l in pyr.levels]
    off = np.concatenate([[0], np.cumsum([a * b for a, b in sizes])])
    out = []
    for g in np.asarray(scan_idx, np.int64):
        lvl = int(np.searchsorted(off, g, side="right") - 1)
        rel = int(g - off[lvl])
        j, i = divmod(rel, sizes[lvl][1])
        reg = histeq(region(frame, net1.step * i - margin, net1.step * j - margin, pyr.scale[lvl], rw, rh))
        k2, k3, face, r2, r3 = select_region(reg, net2, w2, net3, w3, t2, t3, t_nn, rule)
        out.append(dict(index=int(g), level=lvl, i=i, j=j, k2=k2, k3=k3, face=face, r2=r2, r3=r3))
    return out


def stage1_scores(pyr: Pyramid, stage, weights: np.ndarray, form: str = "dense") -> np.ndarray:
    """All stage-1 scores of a frame, flat in (level, y, x) order."""
    return np.concatenate([stage1_level(l, stage, weights, form).ravel() for l in pyr.levels])


def threshold_from_quantile(scores: np.ndarray, q: float) -> np.float32:
    """Threshold that lets the top floor(q N) scores through (benchmark rule: thresholds
    sit at score quantiles): midway between the k-th and (k+1)-th largest fp32 score."""
    s = np.sort(np.asarray(scores).astype(np.float32))[::-1]
    k = int(np.floor(q * s.size))
    if k <= 0:
        return np.float32(s[0]) if s.size else np.float32(0)
    if k >= s.size:
        return np.float32(-np.inf)
    return np.float32((float(s[k - 1]) + float(s[k])) / 2.0)


def survivors(scores: np.ndarray, thr) -> np.ndarray:
    scores = np.ascontiguousarray(scores, np.float64)
    idx = np.zeros(scores.size, np.int64)
    n = lib().orc_survivors(_p(scores), C.c_int64(scores.size), C.c_float(float(thr)),
                            C.c_int64(scores.size), _p(idx))
    return idx[:n].copy()


def crop(frame: np.ndarray, x: int, y: int, scale: float, n: int) -> np.ndarray:
    out = np.zeros((n, n), np.float64)
    lib().orc_crop(_p(frame), C.c_int(frame.shape[1]), C.c_int(frame.shape[0]), C.c_int(frame.strides[0]),
                   C.c_int(int(x)), C.c_int(int(y)), C.c_double(scale), C.c_int(WINDOW), C.c_int(n), _p(out))
    return out


def eval_stage(frame: np.ndarray, pyr: Pyramid, idx: np.ndarray, stage, weights: np.ndarray) -> np.ndarray:
    """Stage 2 / 3 score of every listed window (flat stage-1 indices)."""
    lvl, ys, xs = pyr.decode(idx)
    scales = np.asarray(pyr.scale, np.float64)[lvl]
    xs = np.ascontiguousarray(xs, np.int32)
    ys = np.ascontiguousarray(ys, np.int32)
    weights = np.ascontiguousarray(weights, np.float32)
    assert weights.size == stage.n_params
    out = np.zeros(len(idx), np.float64)
    rc = lib().orc_eval_crops(_p(frame), C.c_int(frame.shape[1]), C.c_int(frame.shape[0]),
                              C.c_int(frame.strides[0]), _p(xs), _p(ys), _p(np.ascontiguousarray(scales)),
                              C.c_int64(len(idx)), C.c_int(WINDOW), _layers(stage), C.c_int(len(stage.layers)),
                              _p(weights), C.c_int(stage.in_size), _p(out))
    if rc != 0:
        raise ValueError("stage evaluation failed")
    return out


def window_boxes(pyr: Pyramid, idx: np.ndarray):
    """Frame-pixel boxes (x, y, size) of flat window indices."""
    lvl, ys, xs = pyr.decode(idx)
    bx = np.zeros(len(idx), np.int32)
    by = np.zeros(len(idx), np.int32)
    bs = np.zeros(len(idx), np.int32)
    a, b, c = C.c_int32(), C.c_int32(), C.c_int32()
    for i in range(len(idx)):
        lib().orc_window_box(C.c_int(int(xs[i])), C.c_int(int(ys[i])), C.c_double(pyr.scale[lvl[i]]),
                             C.c_int(WINDOW), C.byref(a), C.byref(b), C.byref(c))
        bx[i], by[i], bs[i] = a.value, b.value, c.value
    return bx, by, bs


def merge(bx, by, bs, score, order, iou: float = 0.3, min_neighbors: int = 1):
    """Greedy merge; returns (positions of kept boxes in kept order, neighbour counts)."""
    n = len(bx)
    bx = np.ascontiguousarray(bx, np.int32)
    by = np.ascontiguousarray(by, np.int32)
    bs = np.ascontiguousarray(bs, np.int32)
    score = np.ascontiguousarray(score, np.float32)
    order = np.ascontiguousarray(order, np.int64)
    oi = np.zeros(max(n, 1), np.int32)
    on = np.zeros(max(n, 1), np.int32)
    k = lib().orc_merge(_p(bx), _p(by), _p(bs), _p(score), _p(order), C.c_int32(n), C.c_float(iou),
                        C.c_int32(min_neighbors), _p(oi), _p(on))
    return oi[:k].copy(), on[:k].copy()


def merge_rect(bx, by, bw, bh, score, order, iou: float = 0.3, min_neighbors: int = 1):
    """Greedy merge of rectangles; returns (positions of kept boxes in kept order, neighbour counts)."""
    n = len(bx)
    bx, by, bw, bh = (np.ascontiguousarray(a, np.int32) for a in (bx, by, bw, bh))
    score = np.ascontiguousarray(score, np.float32)
    order = np.ascontiguousarray(order, np.int64)
    oi = np.zeros(max(n, 1), np.int32)
    on = np.zeros(max(n, 1), np.int32)
    k = lib().orc_merge_rect(_p(bx), _p(by), _p(bw), _p(bh), _p(score), _p(order), C.c_int32(n), C.c_float(iou),
                             C.c_int32(min_neighbors), _p(oi), _p(on))
    return oi[:k].copy(), on[:k].copy()


def region_box(i: int, j: int, scale: float, net1):
    """Frame-pixel rectangle (x, y, w, h) of the scan window (i, j) of a level with the given scale."""
    v = [C.c_int32() for _ in range(4)]
    lib().orc_region_box(C.c_int(int(i)), C.c_int(int(j)), C.c_double(float(scale)), C.c_int(net1.step),
                         C.c_int(net1.win_w), C.c_int(net1.win_h), *[C.byref(a) for a in v])
    return tuple(a.value for a in v)


def select_merge(pyr: Pyramid, records, net1, iou: float = 0.3, min_neighbors: int = 1):
    """Merge of the regions a selective-unit pass accepted (records from select_unit): list of dicts
    (index, x, y, w, h, score, level, neighbors) in kept order."""
    faces = [r for r in records if r["face"]]
    box = [region_box(r["i"], r["j"], pyr.scale[r["level"]], net1) for r in faces]
    sc = np.array([np.float32(r["r3"].max()) for r in faces], np.float32)
    kept, nb = merge_rect([b[0] for b in box], [b[1] for b in box], [b[2] for b in box], [b[3] for b in box], sc,
                          [r["index"] for r in faces], iou, min_neighbors)
    return [dict(index=faces[p]["index"], x=box[p][0], y=box[p][1], w=box[p][2], h=box[p][3], score=float(sc[p]),
                 level=faces[p]["level"], neighbors=int(k)) for p, k in zip(kept, nb)]


# --------------------------------------------------------------------------
@dataclass
class Trace:
    """Every intermediate of one frame through the cascade."""
    pyramid: Pyramid
    score1: np.ndarray            # all stage-1 scores, flat
    thr: List[float]
    idx1: np.ndarray              # flat indices surviving stage 1
    score2: np.ndarray            # stage-2 score of idx1
    idx2: np.ndarray              # flat indices surviving stage 2
    score3: np.ndarray            # stage-3 score of idx2
    idx3: np.ndarray              # flat indices surviving stage 3
    score3_kept: np.ndarray       # stage-3 score of idx3
    det: List[Dict]               # merged detections


def detect(frame: np.ndarray, cascade, weights: Sequence[np.ndarray], min_face: float, scale_step: float,
           thr: Optional[Sequence[float]] = None, quantiles=(0.02, 0.2), thr3: float = 0.0,
           iou: float = 0.3, min_neighbors: int = 1, form: str = "dense") -> Trace:
    """The whole cascade on one frame.  With `thr=None` the stage-1 / stage-2 thresholds are set at
    the given survival quantiles of this frame's scores and the stage-3 threshold is `thr3`."""
    pyr = build_pyramid(frame, min_face, scale_step)
    s1 = stage1_scores(pyr, cascade[0], weights[0], form)
    t1 = np.float32(thr[0]) if thr is not None else threshold_from_quantile(s1, quantiles[0])
    idx1 = survivors(s1, t1)
    s2 = eval_stage(frame, pyr, idx1, cascade[1], weights[1])
    t2 = np.float32(thr[1]) if thr is not None else threshold_from_quantile(s2, quantiles[1])
    idx2 = idx1[survivors(s2, t2)]
    s3 = eval_stage(frame, pyr, idx2, cascade[2], weights[2])
    t3 = np.float32(thr[2]) if thr is not None else np.float32(thr3)
    keep3 = survivors(s3, t3)
    idx3 = idx2[keep3]
    s3k = s3[keep3]
    bx, by, bs = window_boxes(pyr, idx3)
    kept, nb = merge(bx, by, bs, s3k, idx3, iou, min_neighbors)
    lvl, _, _ = pyr.decode(idx3)
    det = [dict(x=int(bx[p]), y=int(by[p]), size=int(bs[p]), score=float(np.float32(s3k[p])),
                level=int(lvl[p]), neighbors=int(n), index=int(idx3[p])) for p, n in zip(kept, nb)]
    return Trace(pyr, s1, [float(t1), float(t2), float(t3)], idx1, s2, idx2, s3, idx3, s3k, det)
