"""The C-ABI library without a GPU: it loads, exports every symbol that
include/nms.h declares, its host-only helpers are right, and every argument
error is reported before anything is launched.  No compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nms():
    from paper_2502_00535_amd import build as nms_build

    if nms_build.is_stale():
        nms_build.build_library()
    import paper_2502_00535_amd.binding as binding

    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "nms.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nms_[a-z0-9_]+)\s*\(", text)))


def test_header_and_exports_agree(nms):
    declared = declared_functions()
    assert len(declared) >= 18
    assert sorted(nms.EXPORTS) == declared
    raw = ctypes.CDLL(nms.library_path())
    for name in declared:
        assert hasattr(raw, name), f"{name} declared in nms.h but not exported"


def test_version_and_strings(nms):
    assert nms.nms_version() == 100
    assert nms.nms_status_string(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert nms.nms_status_string(code) not in ("ok", "unknown status")
    assert nms.nms_status_string(-99) == "unknown status"


def test_size_helpers(nms):
    assert [nms.nms_padded_n(n) for n in (0, 1, 63, 64, 65, 1000, 4096, 65536)] == [0, 64, 64, 64, 128, 1024, 4096, 65536]
    assert nms.nms_padded_n(-1) == 0 and nms.nms_padded_n(65537) == 0
    assert nms.nms_mask_words(1024) == 16 * 1024
    assert nms.nms_mask_words(4096) == 64 * 4096
    assert nms.nms_mask_words(65) == 2 * 128
    assert nms.nms_mask_words(0) == 0
    assert nms.nms_sort_workspace_bytes(4096, 256) == 0
    assert nms.nms_sort_workspace_bytes(4097, 1) == 4160 * 8
    assert nms.nms_sort_workspace_bytes(16384, 2) == 2 * 16384 * 8
    # order (int32) + box table (5 floats) + y-scaled boxes (4 floats) + scaled threshold (1 float) per padded
    # box + one flag word per tile, 256-byte aligned parts; beyond 4096 boxes the rank step's keys and the
    # two-launch route's masks (32 words per tile of ranks)
    assert nms.nms_workspace_bytes(1024, 1) == 1024 * 4 + 1024 * 20 + 1024 * 16 + 256 + 1024 * 4
    assert nms.nms_workspace_bytes(16384, 1) == 16384 * 4 + 16384 * 20 + 16384 * 16 + 1024 + 16384 * 4 + 16384 * 8 + 256 * 32 * 8
    assert nms.nms_workspace_bytes(100, 3) == 1280 + 7680 + 6144 + 256 + 1536  # 1200 -> 1280; 3*5*128*4; 3*128*16; 3*2*4 -> 256; 3*128*4
    assert nms.nms_greedy_workspace_bytes(1024, 2) == nms.nms_workspace_bytes(1024, 2) + 2 * 16 * 1024 * 8
    assert nms.nms_workspace_bytes(-1, 1) == 0 and nms.nms_workspace_bytes(1, 70000) == 0


def test_route_by_size():
    """nms_route: which kernels the automatic call launches, for the five benchmark shapes and at
    each border of the size rules."""
    import paper_2502_00535_amd.binding as nms

    D, A, T, E = nms.NMS_ROUTE_DIRECT, nms.NMS_ROUTE_ALL_PAIRS, nms.NMS_ROUTE_TWO_LAUNCH, nms.NMS_ROUTE_EARLY_EXIT
    S = nms.NMS_ROUTE_SMALL_FRAMES
    shapes = {(256, 1): D, (4096, 1): D, (1024, 64): S, (16384, 1): T, (4096, 256): E,
              (4096, 2): S, (4096, 16): S, (4096, 19): S, (4096, 20): E, (2048, 7): D, (2048, 8): S, (2048, 32): S, (2048, 33): A,
              (2048, 64): E, (1536, 14): D, (1536, 15): S, (1536, 42): S, (1536, 43): A, (3000, 3): D, (3000, 4): S, (3000, 25): S, (3000, 26): A,
              (1025, 31): D, (1025, 32): S, (1100, 51): S, (1100, 52): A, (4097, 2): A,
              (1024, 10): D, (1024, 11): S, (1024, 24): S, (1024, 25): S, (576, 75): D, (577, 31): D, (577, 32): S, (768, 17): D, (768, 18): S, 
              (1024, 511): S, (1024, 512): S, (1024, 60000): S, (1025, 255): A, (1025, 256): E, (1023, 513): S,
              (512, 127): D, (512, 128): S, (512, 4000): S, (449, 128): S, (448, 128): D, (448, 500): A, (513, 95): D, (513, 96): S, (640, 25): D, (640, 26): S, (513, 128): S, (513, 129): A, (513, 2040): A,
              (640, 128): S, (640, 256): A, (641, 129): S, (641, 256): S, (641, 257): A, (896, 256): S, (896, 257): A, (896, 511): A,
              (897, 257): S, (897, 511): S, (640, 512): A, (641, 512): S, (704, 5000): S,
              (256, 512): D, (256, 513): A, (257, 508): D, (257, 509): A, (100, 60000): A,
              (4097, 1): A, (11585, 1): A, (11586, 1): T, (16384, 7): T, (16384, 8): E, (46340, 1): T, (46341, 1): E,
              (65536, 1): E, (8192, 2): T, (8192, 1): A}
    for (n, f), want in shapes.items():
        assert nms.nms_route(n, f) == want, (n, f)
    assert nms.nms_route(0, 1) == -1 and nms.nms_route(5, 0) == -1 and nms.nms_route(-1, 1) == -1
    assert nms.nms_route(70000, 1) == -1


def test_argument_errors_before_launch(nms):
    L = nms.lib
    p = ctypes.c_void_p(0x1000)  # never dereferenced: every call below must fail validation first
    null = None
    # negative / too large sizes
    assert L.nms_sort(p, p, -1, p, p, null, 0, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_sort(p, p, 65537, p, p, null, 0, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_sort_batched(p, p, null, 16, 70000, p, p, null, 0, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_overlap_mask(p, -5, 0.5, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_reduce(p, p, 1 << 20, p, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_run_ws(p, p, -1, 0.5, p, p, 1 << 20, null) == nms.NMS_ERR_INVALID_ARG
    # null pointers
    assert L.nms_sort(null, p, 8, p, p, null, 0, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_sort(p, null, 8, p, p, null, 0, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_sort(p, p, 8, null, p, null, 0, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_sort(p, p, 8, p, null, null, 0, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_overlap_mask(null, 8, 0.5, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_overlap_mask(p, 8, 0.5, null, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_reduce(null, p, 8, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_reduce(p, null, 8, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_reduce(p, p, 8, null, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_ws(null, p, 8, 0.5, p, p, 1 << 20, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_ws(p, p, 8, 0.5, null, p, 1 << 20, null) == nms.NMS_ERR_INVALID_ARG
    # NaN threshold
    nan = float("nan")
    assert L.nms_overlap_mask(p, 8, nan, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_ws(p, p, 8, nan, p, p, 1 << 20, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_batched(p, p, null, 8, 2, nan, p, p, 1 << 20, null) == nms.NMS_ERR_INVALID_ARG
    # workspace: missing, too small, misaligned
    assert L.nms_run_ws(p, p, 8, 0.5, p, null, 0, null) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_ws(p, p, 8, 0.5, p, p, 16, null) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_ws(p, p, 8, 0.5, p, ctypes.c_void_p(0x1010), 1 << 20, null) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_ranked_batched(p, p, null, 8, 2, 0.5, p, null, 0, null) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_direct_batched(null, p, null, 8, 2, 0.5, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_direct_batched(p, p, null, 8, 2, 0.5, null, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_direct_batched(p, p, null, 70000, 2, 0.5, p, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_run_direct_batched(p, p, null, 8, 2, float("nan"), p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_direct_batched(null, null, null, 0, 2, 0.5, null, null) == nms.NMS_OK
    assert L.nms_sort(p, p, 5000, p, p, null, 0, null) == nms.NMS_ERR_WORKSPACE
    assert L.nms_sort(p, p, 5000, p, p, p, 100, null) == nms.NMS_ERR_WORKSPACE
    # empty work is fine and launches nothing
    assert L.nms_sort(null, null, 0, null, null, null, 0, null) == nms.NMS_OK
    assert L.nms_overlap_mask(null, 0, 0.5, null, null) == nms.NMS_OK
    assert L.nms_reduce(null, null, 0, null, null) == nms.NMS_OK
    assert L.nms_run_ws(null, null, 0, 0.5, null, null, 0, null) == nms.NMS_OK
    assert L.nms_run_batched(null, null, null, 64, 0, 0.5, null, null, 0, null) == nms.NMS_OK


def test_batches_beyond_one_map_launch_are_refused(nms):
    """The pair-test step of a batch is a single launch of 256-thread workgroups; a batch whose
    launch would not fit the grid is refused up front (before anything is enqueued), and its
    workspace size is reported as 0 like that of any other invalid size."""
    L = nms.lib
    p = ctypes.c_void_p(0x1000)
    null = None
    big = 1 << 62
    assert L.nms_workspace_bytes(16384, 8064) > 0
    assert L.nms_workspace_bytes(16384, 8072) == 0
    assert L.nms_run_batched(p, p, null, 16384, 8072, 0.5, p, p, big, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_overlap_mask_batched(p, null, 16384, 8072, 0.5, p, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_run_greedy_batched(p, p, null, 65536, 512, 0.5, p, p, big, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_workspace_bytes(65536, 504) > 0
    # frames of at most 4096 boxes are never affected
    assert L.nms_workspace_bytes(4096, 65535) > 0


def test_matrix_form_argument_errors(nms):
    L = nms.lib
    p = ctypes.c_void_p(0x1000)
    null = None
    assert L.nms_map_matrix(p, p, -1, 64, 0.5, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_map_matrix(p, p, 65, 64, 0.5, p, null) == nms.NMS_ERR_INVALID_ARG      # n beyond the capacity
    assert L.nms_map_matrix(p, p, 10, 100, 0.5, p, null) == nms.NMS_ERR_INVALID_ARG     # capacity not a multiple of 64
    assert L.nms_map_matrix(p, p, 10, 16448, 0.5, p, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_map_matrix(p, p, 10, 64, float("nan"), p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_map_matrix(null, p, 10, 64, 0.5, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_map_matrix(p, null, 10, 64, 0.5, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_map_matrix(p, p, 10, 64, 0.5, null, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_map_matrix(null, null, 0, 0, 0.5, null, null) == nms.NMS_OK
    assert L.nms_reduce_matrix(p, 64, 0, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_reduce_matrix(p, 64, 3, p, null) == nms.NMS_ERR_INVALID_ARG            # k does not divide the capacity
    assert L.nms_reduce_matrix(p, 4096, 2, p, null) == nms.NMS_ERR_INVALID_ARG          # 2048 threads per row
    assert L.nms_reduce_matrix(p, 100, 4, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_reduce_matrix(p, 16448, 64, p, null) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_reduce_matrix(null, 64, 4, p, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_reduce_matrix(p, 64, 4, null, null) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_reduce_matrix(null, 0, 4, null, null) == nms.NMS_OK


def test_options_argument_errors(nms):
    L = nms.lib
    p = ctypes.c_void_p(0x1000)
    big = 1 << 30

    def call(opt, n=8, frames=1, theta=0.5, ws=p, ws_bytes=big, boxes=p, keep=p):
        ref = ctypes.byref(opt) if opt is not None else None
        return L.nms_run_ex_batched(boxes, p, None, n, frames, theta, ref, keep, ws, ws_bytes, None)

    ok = lambda **kw: nms.NmsOptions(kw.get("rule", 0), kw.get("measure", 0), kw.get("compare", 0), kw.get("ties", 0),
                                     kw.get("pixel_offset", 1.0), kw.get("reserved", 0), None)
    for field in ("rule", "measure", "compare", "ties"):
        assert call(ok(**{field: 2})) == nms.NMS_ERR_INVALID_ARG
        assert call(ok(**{field: -1})) == nms.NMS_ERR_INVALID_ARG
    assert call(ok(pixel_offset=0.5)) == nms.NMS_ERR_INVALID_ARG
    assert call(ok(pixel_offset=float("nan"))) == nms.NMS_ERR_INVALID_ARG
    assert call(ok(reserved=1)) == nms.NMS_ERR_INVALID_ARG
    assert call(ok(), theta=float("nan")) == nms.NMS_ERR_INVALID_ARG
    assert call(ok(), n=-1) == nms.NMS_ERR_INVALID_ARG
    assert call(ok(), n=70000) == nms.NMS_ERR_TOO_LARGE
    assert call(ok(), boxes=None) == nms.NMS_ERR_INVALID_ARG
    assert call(ok(), keep=None) == nms.NMS_ERR_INVALID_ARG
    assert call(ok(), ws=None) == nms.NMS_ERR_WORKSPACE
    assert call(ok(), ws_bytes=1000) == nms.NMS_ERR_WORKSPACE
    assert call(ok(), ws=ctypes.c_void_p(0x1008)) == nms.NMS_ERR_WORKSPACE
    assert call(ok(), n=0) == nms.NMS_OK
    assert call(None, n=0) == nms.NMS_OK
    # mask + ranked scores + ranked labels + ranked areas on top of the fused path's workspace
    assert nms.nms_ex_workspace_bytes(1024, 2) == nms.nms_greedy_workspace_bytes(1024, 2) + 3 * (2 * 1024 * 4)
    assert nms.nms_ex_workspace_bytes(-1, 2) == 0


def test_early_exit_argument_errors(nms):
    L = nms.lib
    p = ctypes.c_void_p(0x1000)
    big = 1 << 30
    assert L.nms_run_early_exit_batched(p, p, None, 65537, 2, 0.5, p, p, big, None) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_run_early_exit_batched(p, p, None, -1, 2, 0.5, p, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_early_exit_batched(p, p, None, 64, 2, float("nan"), p, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_early_exit_batched(None, p, None, 64, 2, 0.5, p, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_early_exit_batched(p, None, None, 64, 2, 0.5, p, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_early_exit_batched(p, p, None, 64, 2, 0.5, None, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_early_exit_batched(p, p, None, 64, 2, 0.5, p, None, 0, None) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_early_exit_batched(p, p, None, 64, 2, 0.5, p, p, 100, None) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_early_exit_batched(p, p, None, 64, 2, 0.5, p, ctypes.c_void_p(0x1010), big, None) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_early_exit_batched(None, None, None, 0, 2, 0.5, None, None, 0, None) == nms.NMS_OK


def test_greedy_fused_argument_errors(nms):
    L = nms.lib
    p = ctypes.c_void_p(0x1000)
    big = 1 << 30
    assert L.nms_run_greedy_fused_batched(p, p, None, 4097, 2, 0.5, p, p, big, None) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_run_greedy_fused_batched(p, p, None, -1, 2, 0.5, p, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_greedy_fused_batched(p, p, None, 64, 2, float("nan"), p, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_greedy_fused_batched(None, p, None, 64, 2, 0.5, p, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_greedy_fused_batched(p, p, None, 64, 2, 0.5, None, p, big, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run_greedy_fused_batched(p, p, None, 64, 2, 0.5, p, None, 0, None) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_greedy_fused_batched(p, p, None, 64, 2, 0.5, p, p, 100, None) == nms.NMS_ERR_WORKSPACE
    assert L.nms_run_greedy_fused_batched(None, None, None, 0, 2, 0.5, None, None, 0, None) == nms.NMS_OK


def test_pool_protocol(nms):
    L = nms.lib
    p = ctypes.c_void_p(0x1000)
    assert L.nms_shutdown() == nms.NMS_OK
    assert L.nms_run(p, p, 8, 0.5, p, None) == nms.NMS_ERR_WORKSPACE       # no pool yet
    assert L.nms_init(0, 1, p, 1 << 20) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_init(1024, 1, None, 1 << 20) == nms.NMS_ERR_WORKSPACE
    assert L.nms_init(1024, 1, p, 100) == nms.NMS_ERR_WORKSPACE
    assert L.nms_init(1024, 1, ctypes.c_void_p(0x1001), 1 << 20) == nms.NMS_ERR_WORKSPACE
    assert L.nms_init(70000, 1, p, 1 << 30) == nms.NMS_ERR_TOO_LARGE
    assert L.nms_init(1024, 1, p, 1 << 20) == nms.NMS_OK
    assert L.nms_run(p, p, 2000, 0.5, p, None) == nms.NMS_ERR_WORKSPACE    # beyond the pool's n_max
    assert L.nms_run(p, p, 8, float("nan"), p, None) == nms.NMS_ERR_INVALID_ARG
    assert L.nms_run(p, p, 0, 0.5, p, None) == nms.NMS_OK
    assert L.nms_shutdown() == nms.NMS_OK
    assert L.nms_run(p, p, 8, 0.5, p, None) == nms.NMS_ERR_WORKSPACE


def test_binding_refuses_cpu_tensors(nms):
    import torch

    t = torch.zeros(8, 4)
    with pytest.raises(ValueError):
        nms.nms_sort(t, torch.zeros(8), 8, torch.zeros(8, dtype=torch.int32), torch.zeros(5 * 64))


class _NoDeviceCalls:
    """Stands in for the loaded library: host-only helpers pass through, anything that would
    enqueue work raises, so a test can never hand a host pointer to a kernel."""

    HOST_ONLY = {"nms_padded_n", "nms_mask_words", "nms_workspace_bytes", "nms_sort_workspace_bytes",
                 "nms_status_string", "nms_last_launch_error"}

    def __init__(self, real):
        self._real = real

    def __getattr__(self, name):
        if name in self.HOST_ONLY:
            return getattr(self._real, name)

        def refuse(*args):
            raise RuntimeError(f"reached the library: {name}")

        return refuse


def test_binding_refuses_undersized_tensors(nms, monkeypatch):
    """The C ABI takes bare pointers; the binding knows the tensors' sizes and refuses a buffer
    that is too small for the call.  Run on host tensors with the device check switched off and
    the library replaced by a stand-in that raises, so every argument's check is reached and
    nothing can be launched."""
    import torch

    monkeypatch.setattr(nms, "_on_device", lambda t: True)
    monkeypatch.setattr(nms, "lib", _NoDeviceCalls(nms.lib))
    monkeypatch.setattr(nms, "_stream", lambda stream: None)

    F, n = 3, 100
    n_pad = nms.nms_padded_n(n)
    ok = dict(boxes=torch.zeros((F, n, 4)), scores=torch.zeros((F, n)), keep=torch.zeros((F, n), dtype=torch.uint8),
              counts=torch.zeros(F, dtype=torch.int32), order=torch.zeros((F, n), dtype=torch.int32),
              sorted5=torch.zeros(F * 5 * n_pad), mask=torch.zeros(F * nms.nms_mask_words(n), dtype=torch.int64),
              classes=torch.zeros((F, n), dtype=torch.int32))
    small = dict(boxes=torch.zeros((F, n, 4))[:, :-1].contiguous(), scores=torch.zeros((F, n - 1)),
                 keep=torch.zeros((F, n - 1), dtype=torch.uint8), counts=torch.zeros(F - 1, dtype=torch.int32),
                 order=torch.zeros((F, n - 1), dtype=torch.int32), sorted5=torch.zeros(F * 5 * n_pad - 1),
                 mask=torch.zeros(F * nms.nms_mask_words(n) - 1, dtype=torch.int64),
                 classes=torch.zeros((F, n - 1), dtype=torch.int32))
    ws = torch.zeros(8, dtype=torch.uint8)
    def args(bad):
        return {k: (small[k] if k == bad else ok[k]) for k in ok}

    def run_batched(a):
        nms.nms_run_batched(a["boxes"], a["scores"], a["counts"], n, F, 0.5, a["keep"], ws)

    def run_static(a):
        nms.nms_run_static_batched(a["boxes"], a["scores"], a["counts"], n, F, 0.5, a["keep"])

    def run_direct(a):
        nms.nms_run_direct_batched(a["boxes"], a["scores"], a["counts"], n, F, 0.5, a["keep"])

    def run_ex(a):
        nms.nms_run_ex_batched(a["boxes"], a["scores"], a["counts"], n, F, 0.5, a["keep"], ws, classes=a["classes"])

    def sort_batched(a):
        nms.nms_sort_batched(a["boxes"], a["scores"], a["counts"], n, F, a["order"], a["sorted5"])

    def mask_batched(a):
        nms.nms_overlap_mask_batched(a["sorted5"], a["counts"], n, F, 0.5, a["mask"])

    def reduce_batched(a):
        nms.nms_reduce_batched(a["mask"], a["order"], a["counts"], n, F, a["keep"])

    def greedy_batched(a):
        nms.nms_reduce_greedy_batched(a["mask"], a["order"], a["counts"], n, F, a["keep"])

    cases = [(run_batched, ("boxes", "scores", "counts", "keep")), (run_static, ("boxes", "scores", "counts", "keep")),
             (run_direct, ("boxes", "scores", "counts", "keep")), (run_ex, ("boxes", "scores", "counts", "keep", "classes")),
             (sort_batched, ("boxes", "scores", "counts", "order", "sorted5")), (mask_batched, ("sorted5", "counts", "mask")),
             (reduce_batched, ("mask", "order", "counts", "keep")), (greedy_batched, ("mask", "order", "counts", "keep"))]
    for call, names in cases:
        for bad in names:
            with pytest.raises(ValueError, match="elements, the call needs"):
                call(args(bad))
        # with every tensor large enough the call goes through to the library
        with pytest.raises(RuntimeError, match="reached the library"):
            call(args(None))
    with pytest.raises(ValueError, match="elements, the call needs"):
        nms.RunPlan(ok["boxes"], ok["scores"], None, n, F + 1, 0.5, ok["keep"], ws)
    with pytest.raises(ValueError, match="elements, the call needs"):
        nms.nms_map_matrix(ok["boxes"], ok["scores"], 100, 128, 0.5, torch.zeros(128 * 127, dtype=torch.uint8))
    with pytest.raises(ValueError, match="elements, the call needs"):
        nms.nms_reduce_matrix(torch.zeros(128 * 128, dtype=torch.uint8), 128, 4, torch.zeros(127, dtype=torch.uint8))
    # the single-frame calls
    with pytest.raises(ValueError, match="elements, the call needs"):
        nms.nms_run_ws(ok["boxes"], ok["scores"], F * n + 1, 0.5, ok["keep"], ws)
    with pytest.raises(ValueError, match="elements, the call needs"):
        nms.nms_run(ok["boxes"], ok["scores"], n, 0.5, torch.zeros(n - 1, dtype=torch.uint8))
