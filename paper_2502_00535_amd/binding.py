"""ctypes binding of ``include/nms.h``: argument marshalling only.

Tensor arguments are torch tensors on the GPU (device memory is torch's job);
their ``data_ptr()`` and the current torch HIP stream are handed to the C ABI.
Every function returns nothing and raises :class:`NmsError` on a non-zero status.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libnms_mi355x.so")

NMS_OK = 0
NMS_ERR_INVALID_ARG = -1
NMS_ERR_TOO_LARGE = -2
NMS_ERR_WORKSPACE = -3
NMS_ERR_LAUNCH = -4
NMS_ROUTE_DIRECT, NMS_ROUTE_ALL_PAIRS, NMS_ROUTE_TWO_LAUNCH, NMS_ROUTE_EARLY_EXIT, NMS_ROUTE_SMALL_FRAMES = 0, 1, 2, 3, 4

EXPORTS = (
    "nms_status_string", "nms_version", "nms_last_launch_error", "nms_padded_n", "nms_mask_words",
    "nms_sort_workspace_bytes", "nms_workspace_bytes", "nms_route",
    "nms_sort", "nms_sort_batched", "nms_overlap_mask", "nms_overlap_mask_batched",
    "nms_reduce", "nms_reduce_batched", "nms_run_ws", "nms_run_batched", "nms_run_ranked_batched", "nms_run_direct_batched",
    "nms_run_batched_profiled", "nms_reduce_greedy", "nms_reduce_greedy_batched",
    "nms_greedy_workspace_bytes", "nms_run_greedy_batched", "nms_run_greedy_fused_batched", "nms_run_early_exit_batched", "nms_map_matrix", "nms_reduce_matrix",
    "nms_ex_workspace_bytes", "nms_run_ex_batched",
    "nms_init", "nms_shutdown", "nms_run", "nms_run_static_batched", "nms_host_pair_test",
)


class NmsOptions(ctypes.Structure):
    """struct nms_options of include/nms.h."""
    _fields_ = [("rule", ctypes.c_int32), ("measure", ctypes.c_int32), ("compare", ctypes.c_int32),
                ("ties", ctypes.c_int32), ("pixel_offset", ctypes.c_float), ("reserved", ctypes.c_int32),
                ("classes", ctypes.c_void_p)]


RULES = {"paper": 0, "greedy": 1}
MEASURES = {"outranking_area": 0, "iou": 1}
COMPARES = {"ge": 0, "gt": 1}
TIES = {"index": 0, "ignore": 1}


class NmsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f" [{lib.nms_last_launch_error().decode()}]" if status == NMS_ERR_LAUNCH else ""
        super().__init__(f"{where}: {nms_status_string(status)} ({status}){detail}")


def library_path() -> str:
    return _LIB_PATH


def _load() -> ctypes.CDLL:
    # torch first: its wheel carries its own HIP runtime (soname libamdhip64.so.7).  Once
    # that copy is in the process the loader binds this library to it; loaded the other
    # way round, the system runtime would come in as a second, unusable instance.
    import torch  # noqa: F401

    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2502_00535_amd.build` "
            "(there is no CPU fallback)")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    L.nms_status_string.restype = ctypes.c_char_p
    L.nms_status_string.argtypes = [i32]
    L.nms_version.restype = i32
    L.nms_version.argtypes = []
    L.nms_last_launch_error.restype = ctypes.c_char_p
    L.nms_last_launch_error.argtypes = []
    L.nms_padded_n.restype = i32
    L.nms_padded_n.argtypes = [i32]
    L.nms_mask_words.restype = sz
    L.nms_mask_words.argtypes = [i32]
    L.nms_sort_workspace_bytes.restype = sz
    L.nms_sort_workspace_bytes.argtypes = [i32, i32]
    L.nms_workspace_bytes.restype = sz
    L.nms_workspace_bytes.argtypes = [i32, i32]
    L.nms_route.restype = i32
    L.nms_route.argtypes = [i32, i32]
    L.nms_sort.restype = i32
    L.nms_sort.argtypes = [vp, vp, i32, vp, vp, vp, sz, vp]
    L.nms_sort_batched.restype = i32
    L.nms_sort_batched.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp, sz, vp]
    L.nms_overlap_mask.restype = i32
    L.nms_overlap_mask.argtypes = [vp, i32, f32, vp, vp]
    L.nms_overlap_mask_batched.restype = i32
    L.nms_overlap_mask_batched.argtypes = [vp, vp, i32, i32, f32, vp, vp]
    L.nms_reduce.restype = i32
    L.nms_reduce.argtypes = [vp, vp, i32, vp, vp]
    L.nms_reduce_batched.restype = i32
    L.nms_reduce_batched.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    L.nms_run_ws.restype = i32
    L.nms_run_ws.argtypes = [vp, vp, i32, f32, vp, vp, sz, vp]
    L.nms_run_batched.restype = i32
    L.nms_run_batched.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp, sz, vp]
    L.nms_run_ranked_batched.restype = i32
    L.nms_run_ranked_batched.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp, sz, vp]
    L.nms_run_direct_batched.restype = i32
    L.nms_run_direct_batched.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp]
    L.nms_reduce_greedy.restype = i32
    L.nms_reduce_greedy.argtypes = [vp, vp, i32, vp, vp]
    L.nms_reduce_greedy_batched.restype = i32
    L.nms_reduce_greedy_batched.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    L.nms_greedy_workspace_bytes.restype = sz
    L.nms_greedy_workspace_bytes.argtypes = [i32, i32]
    L.nms_run_greedy_batched.restype = i32
    L.nms_run_greedy_batched.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp, sz, vp]
    L.nms_run_greedy_fused_batched.restype = i32
    L.nms_run_greedy_fused_batched.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp, sz, vp]
    L.nms_run_early_exit_batched.restype = i32
    L.nms_run_early_exit_batched.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp, sz, vp]
    L.nms_run_batched_profiled.restype = i32
    L.nms_run_batched_profiled.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp, sz, vp, ctypes.POINTER(vp)]
    L.nms_map_matrix.restype = i32
    L.nms_map_matrix.argtypes = [vp, vp, i32, i32, f32, vp, vp]
    L.nms_reduce_matrix.restype = i32
    L.nms_reduce_matrix.argtypes = [vp, i32, i32, vp, vp]
    L.nms_ex_workspace_bytes.restype = sz
    L.nms_ex_workspace_bytes.argtypes = [i32, i32]
    L.nms_run_ex_batched.restype = i32
    L.nms_run_ex_batched.argtypes = [vp, vp, vp, i32, i32, f32, ctypes.POINTER(NmsOptions), vp, vp, sz, vp]
    L.nms_init.restype = i32
    L.nms_init.argtypes = [i32, i32, vp, sz]
    L.nms_shutdown.restype = i32
    L.nms_shutdown.argtypes = []
    L.nms_run.restype = i32
    L.nms_run.argtypes = [vp, vp, i32, f32, vp, vp]
    L.nms_run_static_batched.restype = i32
    L.nms_run_static_batched.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp]
    L.nms_host_pair_test.restype = i32
    L.nms_host_pair_test.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_float), f32]
    return L


lib = _load()


# ------------------------------------------------------------------ marshalling helpers

def _on_device(t) -> bool:
    return t.is_cuda


def _ptr(t, dtype_name: str | None, what: str, need: int = 0):
    """Device pointer of a contiguous CUDA/HIP tensor (None -> NULL).  `need` is the number
    of elements the library will read or write there: the C ABI takes bare pointers and
    cannot know a buffer's size, so a tensor that is too small is refused here, before a
    kernel could run past its end."""
    if t is None:
        return None
    import torch

    if not isinstance(t, torch.Tensor):
        raise TypeError(f"{what}: expected a torch tensor")
    if t.numel() < need:
        raise ValueError(f"{what}: {t.numel()} elements, the call needs {need}")
    if not _on_device(t):
        raise ValueError(f"{what}: tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{what}: tensor must be contiguous")
    if dtype_name is not None and str(t.dtype) != f"torch.{dtype_name}":
        raise TypeError(f"{what}: expected dtype {dtype_name}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _sizes(n_max, frames):
    """Element counts of the per-frame buffers for a batch: (frames * n_max, frames * n_pad,
    frames * mask words); zeros when the library will refuse the sizes anyway."""
    n_max, frames = int(n_max), int(frames)
    if n_max < 0 or frames < 0:
        return 0, 0, 0
    return frames * n_max, frames * int(lib.nms_padded_n(n_max)), frames * int(lib.nms_mask_words(n_max))


def _ws(t):
    if t is None:
        return None, 0
    return _ptr(t, None, "workspace"), t.numel() * t.element_size()


def _stream(stream):
    import torch

    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int, where: str):
    if status != NMS_OK:
        raise NmsError(status, where)


# ------------------------------------------------------------------ host-only helpers

def nms_status_string(status: int) -> str:
    return lib.nms_status_string(int(status)).decode()


def nms_version() -> int:
    return int(lib.nms_version())


def nms_padded_n(n: int) -> int:
    return int(lib.nms_padded_n(int(n)))


def nms_mask_words(n: int) -> int:
    return int(lib.nms_mask_words(int(n)))


def nms_sort_workspace_bytes(n_max: int, frames: int) -> int:
    return int(lib.nms_sort_workspace_bytes(int(n_max), int(frames)))


def nms_workspace_bytes(n_max: int, frames: int) -> int:
    return int(lib.nms_workspace_bytes(int(n_max), int(frames)))


def nms_route(n_max: int, frames: int) -> int:
    return int(lib.nms_route(int(n_max), int(frames)))


def nms_host_pair_test(victim, outranking, threshold: float) -> int:
    v = (ctypes.c_float * 4)(*[float(x) for x in victim])
    c = (ctypes.c_float * 4)(*[float(x) for x in outranking])
    return int(lib.nms_host_pair_test(v, c, float(threshold)))


# ------------------------------------------------------------------ device entry points

def nms_sort(boxes, scores, n, order, sorted5, workspace=None, stream=None):
    fn_, fp_, fm_ = _sizes(n, 1)
    w, wb = _ws(workspace)
    _check(lib.nms_sort(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_), int(n),
                        _ptr(order, "int32", "order", fn_), _ptr(sorted5, "float32", "sorted5", 5 * fp_),
                        w, wb, _stream(stream)), "nms_sort")


def nms_sort_batched(boxes, scores, counts, n_max, frames, order, sorted5, workspace=None, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    w, wb = _ws(workspace)
    _check(lib.nms_sort_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames),
                                _ptr(order, "int32", "order", fn_), _ptr(sorted5, "float32", "sorted5", 5 * fp_),
                                w, wb, _stream(stream)), "nms_sort_batched")


def nms_overlap_mask(sorted5, n, threshold, mask, stream=None):
    fn_, fp_, fm_ = _sizes(n, 1)
    _check(lib.nms_overlap_mask(_ptr(sorted5, "float32", "sorted5", 5 * fp_), int(n), float(threshold),
                                _ptr(mask, "int64", "mask", fm_), _stream(stream)), "nms_overlap_mask")


def nms_overlap_mask_batched(sorted5, counts, n_max, frames, threshold, mask, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    _check(lib.nms_overlap_mask_batched(_ptr(sorted5, "float32", "sorted5", 5 * fp_), _ptr(counts, "int32", "counts", int(frames)),
                                        int(n_max), int(frames), float(threshold),
                                        _ptr(mask, "int64", "mask", fm_), _stream(stream)), "nms_overlap_mask_batched")


def nms_reduce(mask, order, n, keep_out, stream=None):
    fn_, fp_, fm_ = _sizes(n, 1)
    _check(lib.nms_reduce(_ptr(mask, "int64", "mask", fm_), _ptr(order, "int32", "order", fn_), int(n),
                          _ptr(keep_out, "uint8", "keep_out", fn_), _stream(stream)), "nms_reduce")


def nms_reduce_batched(mask, order, counts, n_max, frames, keep_out, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    _check(lib.nms_reduce_batched(_ptr(mask, "int64", "mask", fm_), _ptr(order, "int32", "order", fn_),
                                  _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames),
                                  _ptr(keep_out, "uint8", "keep_out", fn_), _stream(stream)), "nms_reduce_batched")


def nms_run_ws(boxes, scores, n, threshold, keep_out, workspace, stream=None):
    fn_, fp_, fm_ = _sizes(n, 1)
    w, wb = _ws(workspace)
    _check(lib.nms_run_ws(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_), int(n),
                          float(threshold), _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream)),
           "nms_run_ws")


def nms_run_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    w, wb = _ws(workspace)
    _check(lib.nms_run_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                               _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                               _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream)), "nms_run_batched")


class RunPlan:
    """nms_run_batched (or another entry point with the same arguments) with its arguments marshalled once.

    For serving loops that call the library many times on the same buffers: the tensors
    are validated and their pointers taken at construction; each call is then a single
    foreign call.  The plan holds references to its tensors, and uses the stream that was
    current when it was built unless one is given.
    """

    SAME_SIGNATURE = ("nms_run_batched", "nms_run_ranked_batched", "nms_run_early_exit_batched",
                      "nms_run_greedy_batched", "nms_run_greedy_fused_batched")

    def __init__(self, boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, stream=None,
                 entry="nms_run_batched"):
        if entry not in self.SAME_SIGNATURE:
            raise ValueError(f"RunPlan: {entry} does not take nms_run_batched's arguments")
        self._entry = entry
        self._keepalive = (boxes, scores, counts, keep_out, workspace)
        w, wb = _ws(workspace)
        fn_, _, _ = _sizes(n_max, frames)
        self._args = (_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                      _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                      _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream))
        self._fn = getattr(lib, entry)

    def __call__(self):
        status = self._fn(*self._args)
        if status != NMS_OK:
            raise NmsError(status, self._entry)


def nms_run_ranked_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    w, wb = _ws(workspace)
    _check(lib.nms_run_ranked_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                      _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                                      _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream)),
           "nms_run_ranked_batched")


def nms_run_direct_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    _check(lib.nms_run_direct_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                      _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                                      _ptr(keep_out, "uint8", "keep_out", fn_), _stream(stream)),
           "nms_run_direct_batched")


def nms_run_batched_profiled(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, events, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    """events: three raw hipEvent_t handles (ints) or None entries."""
    w, wb = _ws(workspace)
    ev = (ctypes.c_void_p * 3)(*[ctypes.c_void_p(e) if e else None for e in events])
    _check(lib.nms_run_batched_profiled(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                        _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                                        _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream), ev),
           "nms_run_batched_profiled")


def nms_reduce_greedy(mask, order, n, keep_out, stream=None):
    fn_, fp_, fm_ = _sizes(n, 1)
    _check(lib.nms_reduce_greedy(_ptr(mask, "int64", "mask", fm_), _ptr(order, "int32", "order", fn_), int(n),
                                 _ptr(keep_out, "uint8", "keep_out", fn_), _stream(stream)), "nms_reduce_greedy")


def nms_reduce_greedy_batched(mask, order, counts, n_max, frames, keep_out, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    _check(lib.nms_reduce_greedy_batched(_ptr(mask, "int64", "mask", fm_), _ptr(order, "int32", "order", fn_),
                                         _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames),
                                         _ptr(keep_out, "uint8", "keep_out", fn_), _stream(stream)),
           "nms_reduce_greedy_batched")


def nms_greedy_workspace_bytes(n_max: int, frames: int) -> int:
    return int(lib.nms_greedy_workspace_bytes(int(n_max), int(frames)))


def nms_run_greedy_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    w, wb = _ws(workspace)
    _check(lib.nms_run_greedy_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                      _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                                      _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream)),
           "nms_run_greedy_batched")


def nms_run_early_exit_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    w, wb = _ws(workspace)
    _check(lib.nms_run_early_exit_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                          _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                                          _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream)),
           "nms_run_early_exit_batched")


def nms_run_greedy_fused_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    w, wb = _ws(workspace)
    _check(lib.nms_run_greedy_fused_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                            _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                                            _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream)),
           "nms_run_greedy_fused_batched")


def nms_map_matrix(boxes, scores, n, capacity, threshold, B, stream=None):
    cap = max(int(capacity), 0)
    _check(lib.nms_map_matrix(_ptr(boxes, "float32", "boxes", 4 * max(int(n), 0)),
                              _ptr(scores, "float32", "scores", max(int(n), 0)), int(n),
                              int(capacity), float(threshold), _ptr(B, "uint8", "B", cap * cap), _stream(stream)),
           "nms_map_matrix")


def nms_reduce_matrix(B, capacity, k, V, stream=None):
    cap = max(int(capacity), 0)
    _check(lib.nms_reduce_matrix(_ptr(B, "uint8", "B", cap * cap), int(capacity), int(k), _ptr(V, "uint8", "V", cap),
                                 _stream(stream)), "nms_reduce_matrix")


def nms_ex_workspace_bytes(n_max: int, frames: int) -> int:
    return int(lib.nms_ex_workspace_bytes(int(n_max), int(frames)))


def nms_run_ex_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, rule="paper",
                       measure="outranking_area", compare="ge", ties="index", pixel_offset=1.0, classes=None,
                       stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    w, wb = _ws(workspace)
    cls = _ptr(classes, "int32", "classes", fn_)
    opt = NmsOptions(RULES[rule], MEASURES[measure], COMPARES[compare], TIES[ties], float(pixel_offset), 0,
                     cls.value if cls is not None else None)
    _check(lib.nms_run_ex_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                  _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                                  ctypes.byref(opt), _ptr(keep_out, "uint8", "keep_out", fn_), w, wb, _stream(stream)),
           "nms_run_ex_batched")


def nms_init(n_max, frames_max, workspace):
    w, wb = _ws(workspace)
    _check(lib.nms_init(int(n_max), int(frames_max), w, wb), "nms_init")


def nms_shutdown():
    _check(lib.nms_shutdown(), "nms_shutdown")


def nms_run(boxes, scores, n, threshold, keep_out, stream=None):
    fn_, fp_, fm_ = _sizes(n, 1)
    _check(lib.nms_run(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_), int(n),
                       float(threshold), _ptr(keep_out, "uint8", "keep_out", fn_), _stream(stream)), "nms_run")


NMS_STATIC_SCRATCH_BYTES = 4194304


def nms_run_static_batched(boxes, scores, counts, n_max, frames, threshold, keep_out, stream=None):
    fn_, fp_, fm_ = _sizes(n_max, frames)
    _check(lib.nms_run_static_batched(_ptr(boxes, "float32", "boxes", 4 * fn_), _ptr(scores, "float32", "scores", fn_),
                                      _ptr(counts, "int32", "counts", int(frames)), int(n_max), int(frames), float(threshold),
                                      _ptr(keep_out, "uint8", "keep_out", fn_), _stream(stream)),
           "nms_run_static_batched")
