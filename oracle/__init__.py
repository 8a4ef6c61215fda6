"""ctypes front end of the CPU oracle (``nms_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Importers are the tests, the benchmark's
``cpu_baseline`` leg and the smoke check; the product package never imports
this module, and this module never imports the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(_HERE, "nms_oracle.c")
LIBRARY = os.path.join(_HERE, "libnms_oracle.so")
# every float operation rounded on its own, no contraction, no value-changing optimisation
CFLAGS = ["-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
          "-fexcess-precision=standard", "-msse2", "-mfpmath=sse"]


def build(source: str = SOURCE, library: str = LIBRARY, force: bool = True) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared object."""
    if not force and os.path.exists(library) and os.path.getmtime(library) >= os.path.getmtime(source):
        return library
    tmp = library + f".tmp{os.getpid()}"
    subprocess.run(["gcc", *CFLAGS, source, "-o", tmp], check=True)
    os.replace(tmp, library)
    return library


_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_u64p = np.ctypeslib.ndpointer(dtype=np.uint64, flags="C_CONTIGUOUS")


def load(library: str | None = None) -> ctypes.CDLL:
    """Load an oracle shared object and declare its prototypes."""
    if library is None:
        library = build(force=False)
    lib = ctypes.CDLL(library)
    lib.nmso_overlap.restype = ctypes.c_float
    lib.nmso_overlap.argtypes = [_f32p, _f32p]
    lib.nmso_area.restype = ctypes.c_float
    lib.nmso_area.argtypes = [_f32p]
    lib.nmso_outranks.restype = ctypes.c_int
    lib.nmso_outranks.argtypes = [_f32p, ctypes.c_int, ctypes.c_int]
    lib.nmso_map.restype = None
    lib.nmso_map.argtypes = [_f32p, _f32p, ctypes.c_int, ctypes.c_float, _u8p]
    lib.nmso_reduce.restype = None
    lib.nmso_reduce.argtypes = [_u8p, ctypes.c_int, _u8p]
    lib.nmso_keep.restype = None
    lib.nmso_keep.argtypes = [_f32p, _f32p, ctypes.c_int, ctypes.c_float, _u8p]
    lib.nmso_order.restype = None
    lib.nmso_order.argtypes = [_f32p, ctypes.c_int, _i32p]
    lib.nmso_ranked_boxes.restype = None
    lib.nmso_ranked_boxes.argtypes = [_f32p, _i32p, ctypes.c_int, _f32p]
    lib.nmso_ranked_eliminations.restype = None
    lib.nmso_ranked_eliminations.argtypes = [_f32p, _i32p, ctypes.c_int, ctypes.c_float, _u8p]
    lib.nmso_ranked_elimination_words.restype = None
    lib.nmso_ranked_elimination_words.argtypes = [_f32p, _i32p, ctypes.c_int, ctypes.c_float, _u64p]
    lib.nmso_alg12_square.restype = None
    lib.nmso_alg12_square.argtypes = [_f32p, ctypes.c_int, ctypes.c_float, ctypes.c_int, _u8p, _u8p]
    lib.nmso_greedy_keep.restype = None
    lib.nmso_greedy_keep.argtypes = [_f32p, _f32p, ctypes.c_int, ctypes.c_float, _u8p]
    lib.nmso_keep_ex.restype = None
    lib.nmso_keep_ex.argtypes = [_f32p, _f32p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_int,
                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_float, _u8p]
    lib.nmso_eliminates_ex.restype = ctypes.c_int
    lib.nmso_eliminates_ex.argtypes = [_f32p, _f32p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_float,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_float]
    return lib


class Oracle:
    """numpy-in, numpy-out wrapper.  One frame per call."""

    def __init__(self, library: str | None = None):
        self.lib = load(library)

    @staticmethod
    def _frame(boxes, scores):
        boxes = np.ascontiguousarray(boxes, dtype=np.float32).reshape(-1, 4)
        scores = np.ascontiguousarray(scores, dtype=np.float32).reshape(-1)
        if boxes.shape[0] != scores.shape[0]:
            raise ValueError("boxes and scores disagree on n")
        return boxes, scores, int(scores.shape[0])

    def overlap(self, box_i, box_j) -> np.float32:
        bi = np.ascontiguousarray(box_i, dtype=np.float32).reshape(4)
        bj = np.ascontiguousarray(box_j, dtype=np.float32).reshape(4)
        return np.float32(self.lib.nmso_overlap(bi, bj))

    def area(self, box) -> np.float32:
        return np.float32(self.lib.nmso_area(np.ascontiguousarray(box, dtype=np.float32).reshape(4)))

    def outranks(self, scores, j, i) -> bool:
        s = np.ascontiguousarray(scores, dtype=np.float32).reshape(-1)
        return bool(self.lib.nmso_outranks(s, int(j), int(i)))

    def map(self, boxes, scores, theta) -> np.ndarray:
        boxes, scores, n = self._frame(boxes, scores)
        B = np.empty((n, n), dtype=np.uint8)
        self.lib.nmso_map(boxes, scores, n, float(np.float32(theta)), B)
        return B

    def reduce(self, B) -> np.ndarray:
        B = np.ascontiguousarray(B, dtype=np.uint8)
        n = B.shape[0]
        V = np.empty(n, dtype=np.uint8)
        self.lib.nmso_reduce(B, n, V)
        return V

    def keep(self, boxes, scores, theta) -> np.ndarray:
        boxes, scores, n = self._frame(boxes, scores)
        keep = np.empty(n, dtype=np.uint8)
        self.lib.nmso_keep(boxes, scores, n, float(np.float32(theta)), keep)
        return keep

    def greedy_keep(self, boxes, scores, theta) -> np.ndarray:
        boxes, scores, n = self._frame(boxes, scores)
        keep = np.zeros(n, dtype=np.uint8)
        self.lib.nmso_greedy_keep(boxes, scores, n, float(np.float32(theta)), keep)
        return keep

    @staticmethod
    def _classes(classes, n):
        if classes is None:
            return None, None
        c = np.ascontiguousarray(classes, dtype=np.int32).reshape(-1)
        if c.shape[0] != n:
            raise ValueError("classes and scores disagree on n")
        return c, c.ctypes.data_as(ctypes.c_void_p)

    def keep_ex(self, boxes, scores, theta, rule="paper", measure="outranking_area", compare="ge",
                ties="index", pixel_offset=1.0, classes=None) -> np.ndarray:
        """The rule with its selectable variants (see nmso_keep_ex)."""
        boxes, scores, n = self._frame(boxes, scores)
        held, cptr = self._classes(classes, n)
        keep = np.zeros(n, dtype=np.uint8)
        self.lib.nmso_keep_ex(boxes, scores, cptr, n, float(np.float32(theta)),
                              {"paper": 0, "greedy": 1}[rule], {"outranking_area": 0, "iou": 1}[measure],
                              {"ge": 0, "gt": 1}[compare], {"index": 0, "ignore": 1}[ties],
                              float(np.float32(pixel_offset)), keep)
        del held
        return keep

    def eliminates_ex(self, boxes, scores, j, i, theta, measure="outranking_area", compare="ge",
                      ties="index", pixel_offset=1.0, classes=None) -> bool:
        boxes, scores, n = self._frame(boxes, scores)
        held, cptr = self._classes(classes, n)
        r = self.lib.nmso_eliminates_ex(boxes, scores, cptr, int(j), int(i), float(np.float32(theta)),
                                        {"outranking_area": 0, "iou": 1}[measure], {"ge": 0, "gt": 1}[compare],
                                        {"index": 0, "ignore": 1}[ties], float(np.float32(pixel_offset)))
        del held
        return bool(r)

    def order(self, scores) -> np.ndarray:
        scores = np.ascontiguousarray(scores, dtype=np.float32).reshape(-1)
        order = np.empty(scores.shape[0], dtype=np.int32)
        self.lib.nmso_order(scores, int(scores.shape[0]), order)
        return order

    def ranked_boxes(self, boxes, order) -> np.ndarray:
        boxes = np.ascontiguousarray(boxes, dtype=np.float32).reshape(-1, 4)
        order = np.ascontiguousarray(order, dtype=np.int32)
        out = np.empty((order.shape[0], 5), dtype=np.float32)
        self.lib.nmso_ranked_boxes(boxes, order, int(order.shape[0]), out)
        return out

    def ranked_eliminations(self, boxes, order, theta) -> np.ndarray:
        boxes = np.ascontiguousarray(boxes, dtype=np.float32).reshape(-1, 4)
        order = np.ascontiguousarray(order, dtype=np.int32)
        n = int(order.shape[0])
        E = np.empty((n, n), dtype=np.uint8)
        self.lib.nmso_ranked_eliminations(boxes, order, n, float(np.float32(theta)), E)
        return E

    def ranked_elimination_words(self, boxes, order, theta) -> np.ndarray:
        boxes = np.ascontiguousarray(boxes, dtype=np.float32).reshape(-1, 4)
        order = np.ascontiguousarray(order, dtype=np.int32)
        n = int(order.shape[0])
        words = np.empty((n, (n + 63) // 64), dtype=np.uint64)
        self.lib.nmso_ranked_elimination_words(boxes, order, n, float(np.float32(theta)), words)
        return words

    def alg12_square(self, D, theta, k):
        D = np.ascontiguousarray(D, dtype=np.float32).reshape(-1, 4)
        dmax = int(D.shape[0])
        if dmax % k:
            raise ValueError("dmax must be a multiple of k")
        B = np.empty((dmax, dmax), dtype=np.uint8)
        V = np.empty(dmax, dtype=np.uint8)
        self.lib.nmso_alg12_square(D, dmax, float(np.float32(theta)), int(k), B, V)
        return B, V
