"""ctypes binding of libcnnc.so: argument marshalling only.

Frames are torch uint8 CUDA (ROCm) tensors; streams are torch streams (or None for the default
stream).  Every method maps to the C entry point of the same name in include/cnnc.h.
"""
import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcnnc.so")

# every symbol include/cnnc.h declares
EXPORTS = [
    "cnnc_create", "cnnc_destroy", "cnnc_set_params", "cnnc_pyramid_layout", "cnnc_build_pyramid",
    "cnnc_stage1_scoremap", "cnnc_compact_survivors", "cnnc_eval_stage", "cnnc_merge_detections",
    "cnnc_detect", "cnnc_detect_async", "cnnc_fetch_detections", "cnnc_get_pyramid", "cnnc_get_scoremap",
    "cnnc_get_survivors", "cnnc_get_stage_scores", "cnnc_survivor_count", "cnnc_set_timing",
    "cnnc_get_timings", "cnnc_set_eval_impl", "cnnc_executed_mfma", "cnnc_measure_peaks", "cnnc_last_error", "cnnc_version",
    "cnnc_stage1_survivors", "cnnc_set_fused_stage1", "cnnc_set_async_chunks", "cnnc_compact_noalloc",
    "cnnc_set_literal_weights", "cnnc_literal_weights", "cnnc_measure_issue_rates", "cnnc_measure_lds_read",
    "cnnc_scan_set_weights", "cnnc_scan_layout", "cnnc_scan_scoremap", "cnnc_get_scan_scoremap", "cnnc_scan_set_tile", "cnnc_scan_tile",
    "cnnc_select_set_weights", "cnnc_select_set_rule", "cnnc_select_run", "cnnc_select_fetch", "cnnc_select_merge", "cnnc_abi_sizes",
    "cnnc_detect_paper", "cnnc_detect_paper_async", "cnnc_fetch_paper",
    "cnnc_pipe_create", "cnnc_pipe_destroy", "cnnc_pipe_set_params", "cnnc_pipe_frame_buffer", "cnnc_pipe_submit", "cnnc_pipe_submit_device",
    "cnnc_pipe_fetch", "cnnc_pipe_set_paper", "cnnc_pipe_fetch_paper", "cnnc_pipe_last_error",
]
STEP_NAMES = ["pyramid", "stage1", "compact1", "stage2", "compact2", "stage3", "compact3", "merge",
              "stage2_conv", "stage3_conv", "scan", "select"]
MAX_LEVELS = 64
E_OVERFLOW = -3


class CnncError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("cnnc error %d: %s" % (code, msg))
        self.code = code


class _Layer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("cin", C.c_int32), ("cout", C.c_int32), ("k", C.c_int32), ("act", C.c_int32)]


class _StageDesc(C.Structure):
    _fields_ = [("in_size", C.c_int32), ("n_layers", C.c_int32), ("layers", C.POINTER(_Layer)),
                ("weights", C.POINTER(C.c_float))]


class _PaperParams(C.Structure):
    _fields_ = [("t1", C.c_float), ("t2", C.c_float), ("t3", C.c_float), ("t_nn", C.c_int32), ("merge_iou", C.c_float),
                ("min_neighbors", C.c_int32)]


class _Params(C.Structure):
    _fields_ = [("min_face", C.c_double), ("scale_step", C.c_double), ("thr", C.c_float * 3),
                ("merge_iou", C.c_float), ("min_neighbors", C.c_int32)]


class Region(C.Structure):
    _fields_ = [("index", C.c_int32), ("level", C.c_int32), ("i", C.c_int32), ("j", C.c_int32), ("k2", C.c_int32),
                ("k3", C.c_int32), ("face", C.c_int32), ("response", C.c_float)]

    def as_dict(self):
        return dict(index=self.index, level=self.level, i=self.i, j=self.j, k2=self.k2, k3=self.k3, face=bool(self.face),
                    response=self.response)


class RegionDetection(C.Structure):
    _fields_ = [("x", C.c_int32), ("y", C.c_int32), ("w", C.c_int32), ("h", C.c_int32), ("score", C.c_float),
                ("level", C.c_int32), ("neighbors", C.c_int32), ("index", C.c_int32)]

    def as_dict(self):
        return dict(x=self.x, y=self.y, w=self.w, h=self.h, score=self.score, level=self.level,
                    neighbors=self.neighbors, index=self.index)


class Detection(C.Structure):
    _fields_ = [("x", C.c_int32), ("y", C.c_int32), ("size", C.c_int32), ("score", C.c_float),
                ("level", C.c_int32), ("neighbors", C.c_int32), ("index", C.c_int32), ("reserved", C.c_int32)]

    def as_dict(self):
        return dict(x=self.x, y=self.y, size=self.size, score=self.score, level=self.level,
                    neighbors=self.neighbors, index=self.index)


class Records:
    """The n records a call wrote, kept as the block of host memory the library filled.  len(), indexing and iteration
    give ctypes structures that view that memory (made when asked for, so a caller that only counts pays nothing per
    record); `array` is the same memory as a numpy structured array."""
    __slots__ = ("_raw", "_ctype", "_n")

    def __init__(self, ctype, cap: int):
        self._ctype, self._n = ctype, 0
        self._raw = np.empty(max(int(cap), 1) * C.sizeof(ctype), np.uint8)      # not cleared: the library writes it

    def _pointer(self):
        return self._raw.ctypes.data_as(C.c_void_p)

    def _filled(self, n: int, cap: int):
        self._n = max(0, min(int(n), int(cap)))
        used = self._n * C.sizeof(self._ctype)
        if 2 * used < self._raw.size:
            self._raw = self._raw[:max(used, 1)].copy()
        return self

    def __len__(self):
        return self._n

    def __getitem__(self, i):
        if isinstance(i, slice):
            return [self[k] for k in range(*i.indices(self._n))]
        if i < 0:
            i += self._n
        if not 0 <= i < self._n:
            raise IndexError(i)
        return self._ctype.from_buffer(self._raw, i * C.sizeof(self._ctype))

    def __iter__(self):
        for i in range(self._n):
            yield self[i]

    @property
    def array(self) -> np.ndarray:
        return self._raw[:self._n * C.sizeof(self._ctype)].view(np.dtype(self._ctype))

    def __eq__(self, other):
        """Equal to a sequence of the same length whose elements are the same records (structures or their dicts)."""
        if isinstance(other, Records):
            return self._ctype is other._ctype and self._n == other._n and bool(np.array_equal(self.array, other.array))
        try:
            if len(other) != self._n:
                return False
        except TypeError:
            return NotImplemented
        return all(a.as_dict() == (b.as_dict() if hasattr(b, "as_dict") else b) for a, b in zip(self, other))

    __hash__ = None


_lib = None
_hip = None


def library_path() -> str:
    return _LIB_PATH


def lib():
    """The loaded library.  There is no fallback: a missing build is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("libcnnc.so is not built: run `python -m paper_1508_01292_amd.build` "
                              "(or __graft_entry__.build())")
        L = C.CDLL(_LIB_PATH)
        L.cnnc_last_error.restype = C.c_char_p
        L.cnnc_last_error.argtypes = [C.c_void_p]
        L.cnnc_version.restype = C.c_char_p
        L.cnnc_pipe_last_error.restype = C.c_char_p
        L.cnnc_pipe_last_error.argtypes = [C.c_void_p]
        _lib = L
    return _lib


def _hiprt():
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
    return _hip


class Stream:
    """A HIP stream of default priority that does not synchronise with the null stream, for callers that want to destroy
    their streams again: a process has few hardware queues, streams that stay alive keep their share of them, and the
    streams of a Pipe created later then have to share queues among themselves."""

    def __init__(self):
        h = C.c_void_p(0)
        rc = _hiprt().hipStreamCreateWithFlags(C.byref(h), C.c_uint(1))          # hipStreamNonBlocking
        if rc != 0 or not h.value:
            raise CnncError(-4, "hipStreamCreateWithFlags failed (%d)" % rc)
        self.cuda_stream = h.value

    def synchronize(self):
        if self.cuda_stream and _hiprt().hipStreamSynchronize(C.c_void_p(self.cuda_stream)) != 0:
            raise CnncError(-4, "hipStreamSynchronize failed")

    def close(self):
        if self.cuda_stream:
            _hiprt().hipStreamSynchronize(C.c_void_p(self.cuda_stream))
            _hiprt().hipStreamDestroy(C.c_void_p(self.cuda_stream))
            self.cuda_stream = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _stream(s) -> C.c_void_p:
    if s is None:
        return C.c_void_p(0)
    return C.c_void_p(int(s.cuda_stream))


def _d2h(ptr: int, nbytes: int, dtype) -> np.ndarray:
    out = np.empty(nbytes // np.dtype(dtype).itemsize, dtype)
    if nbytes:
        rc = _hiprt().hipMemcpy(out.ctypes.data_as(C.c_void_p), C.c_void_p(ptr), C.c_size_t(nbytes), C.c_int(2))
        if rc != 0:
            raise RuntimeError("hipMemcpy failed: %d" % rc)
    return out


class Context:
    """One detector context (cnnc_ctx).  Calls on one context must not overlap."""

    def __init__(self, cascade: Sequence, weights: Sequence[np.ndarray], max_w: int, max_h: int,
                 max_survivors: int):
        self._h = C.c_void_p(0)
        self._keep = []
        descs = _stage_descs(cascade, weights, self._keep)
        rc = lib().cnnc_create(C.byref(self._h), descs, C.c_int(max_w), C.c_int(max_h), C.c_int(max_survivors))
        if rc != 0:
            self._h = C.c_void_p(0)
            raise CnncError(rc, "cnnc_create failed")
        self.max_survivors = max_survivors
        self._frame = None

    # -- plumbing ---------------------------------------------------------------------------
    def _check(self, rc: int, allow_overflow: bool = False) -> int:
        if rc != 0 and not (allow_overflow and rc == E_OVERFLOW):
            raise CnncError(rc, (lib().cnnc_last_error(self._h) or b"").decode())
        return rc

    def close(self):
        if self._h:
            lib().cnnc_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _frame_args(self, frame):
        if frame.dtype.__str__() != "torch.uint8" or frame.dim() != 2 or not frame.is_cuda or frame.stride(1) != 1:
            raise ValueError("frame must be a 2-D uint8 device tensor with unit column stride")
        self._frame = frame          # the library reads it again in cnnc_eval_stage
        return (C.c_void_p(frame.data_ptr()), C.c_int(frame.shape[1]), C.c_int(frame.shape[0]),
                C.c_int(frame.stride(0)))

    # -- the C entry points -----------------------------------------------------------------
    def set_params(self, min_face: float, scale_step: float, thr=(0.0, 0.0, 0.0), merge_iou: float = 0.3,
                   min_neighbors: int = 1):
        p = _Params(min_face, scale_step, (C.c_float * 3)(*[float(t) for t in thr]), merge_iou, min_neighbors)
        self._check(lib().cnnc_set_params(self._h, C.byref(p)))

    def pyramid_layout(self, w: int, h: int):
        n = C.c_int(0)
        lw = np.zeros(MAX_LEVELS, np.int32)
        lh = np.zeros(MAX_LEVELS, np.int32)
        sc = np.zeros(MAX_LEVELS, np.float64)
        po = np.zeros(MAX_LEVELS + 1, np.int64)
        so = np.zeros(MAX_LEVELS + 1, np.int64)
        vp = lambda a: a.ctypes.data_as(C.c_void_p)
        self._check(lib().cnnc_pyramid_layout(self._h, C.c_int(w), C.c_int(h), C.byref(n), vp(lw), vp(lh), vp(sc),
                                              vp(po), vp(so)))
        k = n.value
        return dict(n_levels=k, lvl_w=lw[:k].tolist(), lvl_h=lh[:k].tolist(), scale=sc[:k].tolist(),
                    pyr_off=po[:k + 1].tolist(), score_off=so[:k + 1].tolist())

    def build_pyramid(self, frame, stream=None):
        self._check(lib().cnnc_build_pyramid(self._h, *self._frame_args(frame), _stream(stream)))

    def stage1_scoremap(self, stream=None):
        self._check(lib().cnnc_stage1_scoremap(self._h, _stream(stream)))

    def stage1_survivors(self, thr: float, stream=None):
        self._check(lib().cnnc_stage1_survivors(self._h, C.c_float(thr), _stream(stream)))

    def set_async_chunks(self, chunks: int):
        self._check(lib().cnnc_set_async_chunks(self._h, C.c_int(chunks)))

    def set_fused_stage1(self, on: bool):
        self._check(lib().cnnc_set_fused_stage1(self._h, C.c_int(1 if on else 0)))

    def compact_survivors(self, stage: int, thr: float, stream=None):
        self._check(lib().cnnc_compact_survivors(self._h, C.c_int(stage), C.c_float(thr), _stream(stream)))

    def eval_stage(self, k: int, stream=None):
        self._check(lib().cnnc_eval_stage(self._h, C.c_int(k), _stream(stream)))

    def merge_detections(self, cap: int = 4096, stream=None) -> Records:
        out = Records(Detection, cap)
        n = C.c_int(0)
        self._check(lib().cnnc_merge_detections(self._h, out._pointer(), C.c_int(cap), C.byref(n), _stream(stream)))
        return out._filled(n.value, cap)

    def detect(self, frame, cap: int = 4096) -> Records:
        out = Records(Detection, cap)
        n = C.c_int(0)
        self._check(lib().cnnc_detect(self._h, *self._frame_args(frame), out._pointer(), C.c_int(cap), C.byref(n)))
        return out._filled(n.value, cap)

    def detect_async(self, frame, stream=None):
        self._check(lib().cnnc_detect_async(self._h, *self._frame_args(frame), _stream(stream)))

    def fetch_detections(self, cap: int = 4096) -> Records:
        out = Records(Detection, cap)
        n = C.c_int(0)
        self._check(lib().cnnc_fetch_detections(self._h, out._pointer(), C.c_int(cap), C.byref(n)))
        return out._filled(n.value, cap)

    # -- views (copied to the host) -----------------------------------------------------------
    def get_pyramid(self) -> np.ndarray:
        _hiprt().hipDeviceSynchronize()
        p, n = C.c_void_p(0), C.c_int64(0)
        self._check(lib().cnnc_get_pyramid(self._h, C.byref(p), C.byref(n)))
        return _d2h(p.value, n.value, np.uint8)

    def get_scoremap(self) -> np.ndarray:
        _hiprt().hipDeviceSynchronize()
        p, n = C.c_void_p(0), C.c_int64(0)
        self._check(lib().cnnc_get_scoremap(self._h, C.byref(p), C.byref(n)))
        return _d2h(p.value, n.value * 4, np.float32)

    def survivor_count(self, stage: int, stream=None) -> int:
        n = C.c_int(0)
        self._check(lib().cnnc_survivor_count(self._h, C.c_int(stage), C.byref(n), _stream(stream)))
        return n.value

    def get_survivors(self, stage: int, stream=None):
        """(flat window indices, scores of that stage) of the survivors of `stage`."""
        n = self.survivor_count(stage, stream)
        pi, ps = C.c_void_p(0), C.c_void_p(0)
        self._check(lib().cnnc_get_survivors(self._h, C.c_int(stage), C.byref(pi), C.byref(ps)))
        return _d2h(pi.value, n * 4, np.uint32), _d2h(ps.value, n * 4, np.float32)

    def get_stage_scores(self, k: int, stream=None) -> np.ndarray:
        """Scores of stage k (2 or 3) for every survivor of stage k - 1."""
        n = self.survivor_count(k - 1, stream)
        p = C.c_void_p(0)
        self._check(lib().cnnc_get_stage_scores(self._h, C.c_int(k), C.byref(p)))
        return _d2h(p.value, n * 4, np.float32)

    # ---- first stage in the paper's geometry (27 x 31 window, 4 pixel step)
    def scan_set_weights(self, weights: np.ndarray, act: int = 1):
        w = np.ascontiguousarray(weights, np.float32)
        self._check(lib().cnnc_scan_set_weights(self._h, w.ctypes.data_as(C.c_void_p), C.c_int(w.size), C.c_int(act)))

    def scan_layout(self, w: int, h: int):
        n = C.c_int(0)
        ow = np.zeros(MAX_LEVELS, np.int32)
        oh = np.zeros(MAX_LEVELS, np.int32)
        off = np.zeros(MAX_LEVELS + 1, np.int64)
        self._check(lib().cnnc_scan_layout(self._h, C.c_int(w), C.c_int(h), C.byref(n), ow.ctypes.data_as(C.c_void_p),
                                           oh.ctypes.data_as(C.c_void_p), off.ctypes.data_as(C.c_void_p)))
        k = n.value
        return {"n_levels": k, "out_w": ow[:k].copy(), "out_h": oh[:k].copy(), "out_off": off[:k + 1].copy()}

    def scan_scoremap(self, stream=None):
        self._check(lib().cnnc_scan_scoremap(self._h, _stream(stream)))

    def scan_set_tile(self, side: int):
        """Responses per side of a workgroup's tile: 0 (chosen from the frame), 8 or 16."""
        self._check(lib().cnnc_scan_set_tile(self._h, C.c_int(side)))

    def scan_tile(self) -> int:
        return int(lib().cnnc_scan_tile(self._h))

    def get_scan_scoremap(self) -> np.ndarray:
        _hiprt().hipDeviceSynchronize()
        p, n = C.c_void_p(0), C.c_int64(0)
        self._check(lib().cnnc_get_scan_scoremap(self._h, C.byref(p), C.byref(n)))
        return _d2h(p.value, n.value * 4, np.float32)

    # ---- the selective unit in the paper's geometry
    def select_set_weights(self, w2: np.ndarray, w3: np.ndarray, act: int = 1):
        a, b = np.ascontiguousarray(w2, np.float32), np.ascontiguousarray(w3, np.float32)
        self._check(lib().cnnc_select_set_weights(self._h, a.ctypes.data_as(C.c_void_p), C.c_int(a.size),
                                                  b.ctypes.data_as(C.c_void_p), C.c_int(b.size), C.c_int(act)))

    def select_run(self, t1: float, t2: float, t3: float, t_nn: int, stream=None):
        self._check(lib().cnnc_select_run(self._h, C.c_float(t1), C.c_float(t2), C.c_float(t3), C.c_int(t_nn), _stream(stream)))

    def select_fetch(self, cap: int = 65536, maps: bool = False):
        """Records of the positions that passed T_1 (list of Region); with maps=True also the two (n, 5, 5) response maps."""
        out = Records(Region, cap)
        n = C.c_int(0)
        m2 = np.zeros((cap, 5, 5), np.float32) if maps else None
        m3 = np.zeros((cap, 5, 5), np.float32) if maps else None
        self._check(lib().cnnc_select_fetch(self._h, out._pointer(), C.c_int(cap), C.byref(n),
                                            m2.ctypes.data_as(C.c_void_p) if maps else C.c_void_p(0),
                                            m3.ctypes.data_as(C.c_void_p) if maps else C.c_void_p(0)))
        recs = out._filled(n.value, cap)
        return (recs, m2[:n.value], m3[:n.value]) if maps else recs

    def select_set_rule(self, rule: int):
        self._check(lib().cnnc_select_set_rule(self._h, C.c_int(rule)))

    def select_merge(self, iou: float = 0.3, min_neighbors: int = 1, cap: int = 4096, stream=None):
        """Greedy merge of the regions the last select_run accepted (list of RegionDetection, kept order)."""
        out = Records(RegionDetection, cap)
        n = C.c_int(0)
        self._check(lib().cnnc_select_merge(self._h, C.c_float(iou), C.c_int(min_neighbors), out._pointer(), C.c_int(cap),
                                            C.byref(n), _stream(stream)))
        return out._filled(n.value, cap)

    @staticmethod
    def _paper_params(t1, t2, t3, t_nn, iou, min_neighbors):
        return _PaperParams(float(t1), float(t2), float(t3), int(t_nn), float(iou), int(min_neighbors))

    def detect_paper(self, frame, t1: float, t2: float, t3: float, t_nn: int, iou: float = 0.3, min_neighbors: int = 1,
                     cap: int = 4096):
        """The whole path in the paper's geometry on one frame (list of RegionDetection, kept order)."""
        out = Records(RegionDetection, cap)
        n = C.c_int(0)
        p = self._paper_params(t1, t2, t3, t_nn, iou, min_neighbors)
        self._check(lib().cnnc_detect_paper(self._h, *self._frame_args(frame), C.byref(p), out._pointer(), C.c_int(cap), C.byref(n)))
        return out._filled(n.value, cap)

    def detect_paper_async(self, frame, t1: float, t2: float, t3: float, t_nn: int, iou: float = 0.3, min_neighbors: int = 1,
                           stream=None):
        p = self._paper_params(t1, t2, t3, t_nn, iou, min_neighbors)
        self._check(lib().cnnc_detect_paper_async(self._h, *self._frame_args(frame), C.byref(p), _stream(stream)))

    def fetch_paper(self, cap: int = 4096):
        out = Records(RegionDetection, cap)
        n = C.c_int(0)
        self._check(lib().cnnc_fetch_paper(self._h, out._pointer(), C.c_int(cap), C.byref(n)))
        return out._filled(n.value, cap)

    def set_literal_weights(self, on: bool):
        self._check(lib().cnnc_set_literal_weights(self._h, C.c_int(1 if on else 0)))

    def literal_weights(self) -> bool:
        """True when stage 1 runs the build of its kernel that carries this context's weights as instruction literals."""
        return bool(lib().cnnc_literal_weights(self._h))

    def set_eval_impl(self, impl: int):
        self._check(lib().cnnc_set_eval_impl(self._h, C.c_int(impl)))

    def executed_mfma(self, k: int) -> int:
        n = C.c_int64(0)
        self._check(lib().cnnc_executed_mfma(self._h, C.c_int(k), C.byref(n)))
        return n.value

    def set_timing(self, on: bool):
        self._check(lib().cnnc_set_timing(self._h, C.c_int(1 if on else 0)))

    def get_timings(self):
        ms = (C.c_double * len(STEP_NAMES))()
        calls = (C.c_int32 * len(STEP_NAMES))()
        self._check(lib().cnnc_get_timings(self._h, ms, calls))
        return {n: (ms[i], calls[i]) for i, n in enumerate(STEP_NAMES)}


def _stage_descs(cascade, weights, keep):
    descs = (_StageDesc * 3)()
    for s, (st, wt) in enumerate(zip(cascade, weights)):
        layers = (_Layer * len(st.layers))(*[_Layer(l.kind, l.cin, l.cout, l.k, l.act) for l in st.layers])
        w = np.ascontiguousarray(wt, np.float32)
        if w.size != st.n_params:
            raise ValueError("weight blob of stage %d has %d values, expected %d" % (s + 1, w.size, st.n_params))
        keep += [layers, w]
        descs[s] = _StageDesc(st.in_size, len(st.layers), layers, w.ctypes.data_as(C.POINTER(C.c_float)))
    return descs


class Pipe:
    """Frame ingest ring (cnnc_pipe): host frames in, detections out, copies and kernels of several frames overlapped."""

    def __init__(self, cascade, weights, w: int, h: int, max_survivors: int, depth: int = 3, use_graph: bool = True):
        self._h = C.c_void_p(0)
        self._keep = []
        self._frames = {}            # device frames of tickets not fetched yet (kept alive for the library)
        self.w, self.h, self.depth = w, h, depth
        rc = lib().cnnc_pipe_create(C.byref(self._h), _stage_descs(cascade, weights, self._keep), C.c_int(w), C.c_int(h),
                                    C.c_int(max_survivors), C.c_int(depth), C.c_int(1 if use_graph else 0))
        if rc != 0:
            self._h = C.c_void_p(0)
            raise CnncError(rc, "cnnc_pipe_create failed")

    def _check(self, rc: int):
        if rc != 0:
            raise CnncError(rc, (lib().cnnc_pipe_last_error(self._h) or b"").decode())

    def close(self):
        if self._h:
            lib().cnnc_pipe_destroy(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_params(self, min_face: float, scale_step: float, thr=(0.0, 0.0, 0.0), merge_iou: float = 0.3,
                   min_neighbors: int = 1):
        p = _Params(min_face, scale_step, (C.c_float * 3)(*[float(t) for t in thr]), merge_iou, min_neighbors)
        self._check(lib().cnnc_pipe_set_params(self._h, C.byref(p)))

    def frame_buffer(self) -> np.ndarray:
        """The pinned h x w uint8 buffer that the next submit() sends (a view, valid until that frame is fetched)."""
        p = C.c_void_p(0)
        self._check(lib().cnnc_pipe_frame_buffer(self._h, C.byref(p)))
        return np.ctypeslib.as_array(C.cast(p, C.POINTER(C.c_uint8)), shape=(self.h, self.w))

    def submit(self, frame: Optional[np.ndarray] = None) -> int:
        """frame = None: send the buffer last returned by frame_buffer(); else a host uint8 h x w array."""
        t = C.c_int64(0)
        if frame is None:
            self._check(lib().cnnc_pipe_submit(self._h, C.c_void_p(0), C.c_int(self.w), C.byref(t)))
        else:
            if frame.dtype != np.uint8 or frame.ndim != 2 or frame.shape != (self.h, self.w) or frame.strides[1] != 1:
                raise ValueError("frame must be a host uint8 array of the pipe's size with unit column stride")
            self._check(lib().cnnc_pipe_submit(self._h, frame.ctypes.data_as(C.c_void_p), C.c_int(frame.strides[0]), C.byref(t)))
        return t.value

    def submit_device(self, frame) -> int:
        """A frame that is on the device already (2-D uint8 tensor of the pipe's size): nothing is copied.  The caller
        keeps it alive and unchanged until its ticket is fetched."""
        if frame.dtype.__str__() != "torch.uint8" or frame.dim() != 2 or not frame.is_cuda or frame.stride(1) != 1 or \
                tuple(frame.shape) != (self.h, self.w):
            raise ValueError("frame must be a 2-D uint8 device tensor of the pipe's size with unit column stride")
        t = C.c_int64(0)
        self._check(lib().cnnc_pipe_submit_device(self._h, C.c_void_p(frame.data_ptr()), C.c_int(frame.stride(0)), C.byref(t)))
        self._frames[t.value] = frame
        return t.value

    def fetch(self, ticket: int, cap: int = 4096) -> Records:
        self._frames.pop(ticket, None)
        out = Records(Detection, cap)
        n = C.c_int(0)
        self._check(lib().cnnc_pipe_fetch(self._h, C.c_int64(ticket), out._pointer(), C.c_int(cap), C.byref(n)))
        return out._filled(n.value, cap)

    def set_paper(self, scan_weights: np.ndarray, w2: np.ndarray, w3: np.ndarray, t1: float, t2: float, t3: float, t_nn: int,
                  iou: float = 0.3, min_neighbors: int = 1, rule: int = 2, scan_act: int = 1, select_act: int = 1):
        """Switch the pipe to the path in the paper's geometry (scan, selective unit, merge)."""
        a, b, c = (np.ascontiguousarray(x, np.float32) for x in (scan_weights, w2, w3))
        pp = _PaperParams(float(t1), float(t2), float(t3), int(t_nn), float(iou), int(min_neighbors))
        self._check(lib().cnnc_pipe_set_paper(self._h, a.ctypes.data_as(C.c_void_p), C.c_int(a.size), C.c_int(scan_act),
                                              b.ctypes.data_as(C.c_void_p), C.c_int(b.size), c.ctypes.data_as(C.c_void_p),
                                              C.c_int(c.size), C.c_int(select_act), C.c_int(rule), C.byref(pp)))

    def fetch_paper(self, ticket: int, cap: int = 4096) -> Records:
        self._frames.pop(ticket, None)
        out = Records(RegionDetection, cap)
        n = C.c_int(0)
        self._check(lib().cnnc_pipe_fetch_paper(self._h, C.c_int64(ticket), out._pointer(), C.c_int(cap), C.byref(n)))
        return out._filled(n.value, cap)


def cnnc_abi_sizes():
    """(sizeof cnnc_layer, cnnc_stage_desc, cnnc_params, cnnc_det, cnnc_region, CNNC_T_COUNT, sizeof cnnc_rdet) as the
    library was built."""
    out = (C.c_int32 * 7)()
    n = lib().cnnc_abi_sizes(out, C.c_int(7))
    return tuple(out[:n])


def cnnc_compact_noalloc(values, n: int, thr: float, index, score, count, stream=None) -> int:
    """cnnc_compact_noalloc on torch device tensors: values float32, index int32 / uint32 storage and score float32 of
    equal capacity, count a one-element int32 tensor.  Returns the C return code (0, or a negative CNNC_E_*)."""
    cap = min(int(index.numel()), int(score.numel()))
    return lib().cnnc_compact_noalloc(C.c_void_p(values.data_ptr() if values is not None else 0), C.c_int64(n), C.c_float(thr),
                                      C.c_void_p(index.data_ptr()), C.c_void_p(score.data_ptr()), C.c_int32(cap),
                                      C.c_void_p(count.data_ptr()), _stream(stream))


def cnnc_measure_issue_rates():
    """ns per wave instruction and SIMD (four waves per SIMD) of v_fmac_f32 with vector, scalar-register and literal
    operands, and of v_rcp_f32."""
    out = (C.c_double * 4)()
    rc = lib().cnnc_measure_issue_rates(out, C.c_int(4))
    if rc != 0:
        raise CnncError(rc, "cnnc_measure_issue_rates failed")
    return {"v_fmac_vector_operands": out[0], "v_fmac_scalar_register_operand": out[1], "v_fmac_literal_operand": out[2],
            "v_rcp_f32": out[3]}


def cnnc_measure_lds_read(addr, width: int) -> float:
    """ns per wave instruction and compute unit of an LDS read of `width` dwords with lane l at dword address addr[l]."""
    a = (C.c_int32 * 64)(*[int(x) for x in addr])
    ns = C.c_double(0)
    rc = lib().cnnc_measure_lds_read(a, C.c_int(width), C.byref(ns))
    if rc != 0:
        raise CnncError(rc, "cnnc_measure_lds_read failed")
    return ns.value


def cnnc_measure_peaks():
    """(dense fp32 MFMA TFLOP/s, fp32 vector FMA TFLOP/s, HBM copy GB/s) sustained by synthetic probes."""
    a, b, c = C.c_double(0), C.c_double(0), C.c_double(0)
    rc = lib().cnnc_measure_peaks(C.byref(a), C.byref(b), C.byref(c))
    if rc != 0:
        raise CnncError(rc, "cnnc_measure_peaks failed")
    return a.value, b.value, c.value


# The C spelling of every context call: cnnc_<name>(ctx, ...) is Context.<name>(...).
_CTX_CALLS = ("set_params", "pyramid_layout", "build_pyramid", "stage1_scoremap", "stage1_survivors", "set_fused_stage1", "set_async_chunks",
              "compact_survivors", "eval_stage", "merge_detections", "detect", "detect_async", "fetch_detections",
              "get_pyramid", "get_scoremap", "get_survivors", "get_stage_scores", "survivor_count", "set_eval_impl",
              "executed_mfma", "set_timing", "get_timings", "scan_set_weights", "scan_layout", "scan_scoremap",
              "get_scan_scoremap", "scan_set_tile", "scan_tile", "select_set_weights", "select_set_rule", "select_run", "select_fetch", "select_merge", "detect_paper",
              "detect_paper_async", "fetch_paper", "set_literal_weights", "literal_weights")


def _c_spelling(method):
    def call(ctx, *a, **k):
        return getattr(ctx, method)(*a, **k)
    call.__name__ = "cnnc_" + method
    call.__doc__ = "Context.%s" % method
    return call


for _m in _CTX_CALLS:
    globals()["cnnc_" + _m] = _c_spelling(_m)


def cnnc_create(cascade, weights, max_w, max_h, max_survivors) -> Context:
    return Context(cascade, weights, max_w, max_h, max_survivors)


def cnnc_destroy(ctx: Context):
    ctx.close()
