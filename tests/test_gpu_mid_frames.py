"""The sort-free one-launch route on small batches of frames of 1025 to 4096 boxes (two or four input
elements per thread, a frame shared out among up to 64 workgroups) against the oracle's plain double
loop, 0 differing bits: shares of one, two and three to five tiles of victims (the first stage takes
a different form for each), frame lengths around the register and tile sizes, ragged batches, long
lists for the second stage, y coordinates outside the scaled form's range, thresholds that take the
literal division, equal scores and scores of every kind."""
import numpy as np
import pytest

from gpu_util import DeviceFrames, oracle_keep_frames
from workloads import clustered_frame, random_frame, scores_of_every_kind

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nms():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2502_00535_amd.binding as binding

    return binding


def check(nms, oracle, boxes, scores, theta, counts=None):
    F, n = scores.shape
    assert nms.nms_route(n, F) == nms.NMS_ROUTE_SMALL_FRAMES, f"{F} x {n} is not a shape of the one-launch route"
    want = oracle_keep_frames(oracle, boxes, scores, np.float32(theta), counts)
    dev = DeviceFrames(nms, boxes, scores, counts)
    got = dev.fused(float(theta))
    assert np.array_equal(got, want), f"{(got != want).sum()} differing keep bits"
    return want


def clustered(seed, F, n):
    fr = [clustered_frame(seed + f, objects=(n + 15) // 16, width=3840, height=2160, size_lo=24.0, size_hi=384.0) for f in range(F)]
    return np.stack([x[0][:n] for x in fr]), np.stack([x[1][:n] for x in fr])


def uniform(seed, F, n, **kw):
    boxes = np.zeros((F, n, 4), np.float32)
    scores = np.zeros((F, n), np.float32)
    for f in range(F):
        boxes[f], scores[f] = random_frame(seed + f, n, **kw)
    return boxes, scores


# (frames, boxes): tiles of victims per workgroup 1, 1, 2, 4, 5, 1 (47 workgroups per frame), 3, 2, 4 | two elements per thread: 1, 2, 4, 4, 3, 4
SHAPES = [(2, 4096), (4, 4096), (8, 4096), (16, 4096), (19, 4096), (4, 3000), (16, 3000), (9, 2049), (18, 3500),
          (8, 2048), (16, 2048), (32, 2048), (33, 1025), (30, 1100), (40, 1536)]


@pytest.mark.parametrize("frames,n", SHAPES)
def test_clustered_detections(nms, oracle, frames, n):
    print(f"case {frames} x {n}", flush=True)
    boxes, scores = clustered(100 * n + frames, frames, n)
    counts = None
    if frames % 2 == 0:
        counts = np.random.default_rng(n).integers(0, n + 1, frames).astype(np.int32)
        counts[:2] = [n, 65]
    want = check(nms, oracle, boxes, scores, [0.5, 0.45, 0.3][frames % 3], counts)
    assert 0 < want.sum() < want.size // 4


@pytest.mark.parametrize("n", [1025, 1087, 1088, 1089, 1500, 2047, 2048, 2049, 2111, 2112, 2113, 2500, 3071, 3072, 3073, 3999, 4033, 4095, 4096])
def test_frame_lengths(nms, oracle, n):
    F = (1 << 25) // (n * n) + 2
    print(f"case {F} x {n}", flush=True)
    boxes, scores = uniform(40000 + n, F, n, extent=2500, max_side=160, integer=(n % 2 == 1), score_levels=max(3, n // 3))
    want = check(nms, oracle, boxes, scores, [0.5, 0.3, 0.45][n % 3])
    assert 0 < want.sum() < want.size


def test_ragged_batches(nms, oracle):
    """Empty frames, frames shorter than a tile, shorter than a register's 1024 elements, and full ones in one call."""
    for F, n in ((12, 4096), (24, 2048)):
        boxes, scores = uniform(77 + n, F, n, extent=3000, max_side=200, integer=True, score_levels=200)
        counts = np.array(([0, 1, 63, 64, 65, 1023, 1024, 1025, n - 1, n, 2047, 700] * 2)[:F], np.int32)
        counts = np.minimum(counts, n).astype(np.int32)
        check(nms, oracle, boxes, scores, 0.45, counts)


@pytest.mark.parametrize("frames,n", [(18, 3500), (19, 4096), (16, 4096), (32, 2048), (8, 4096), (2, 4096)])
def test_little_eliminated(nms, oracle, frames, n):
    """Boxes spread so far that almost every victim reaches the second stage: lists of up to 320 victims per
    workgroup (the second stage changes its form at 256), and disjoint boxes of which a chosen number repeat
    the best-ranked one."""
    print(f"case {frames} x {n}", flush=True)
    boxes, scores = uniform(500 + n, frames, n, extent=200000, max_side=90, integer=False)
    want = check(nms, oracle, boxes, scores, 0.5)
    assert want.sum() > 0.95 * want.size
    side = int(np.ceil(np.sqrt(n)))
    gx, gy = np.meshgrid(np.arange(side), np.arange(side))
    cells = np.stack([gx.ravel() * 40.0, gy.ravel() * 40.0], 1)[:n]
    base = np.concatenate([cells, cells + 30.0], 1).astype(np.float32)
    scores = np.tile((1.0 - np.arange(n) / n).astype(np.float32), (frames, 1))
    boxes = np.tile(base, (frames, 1, 1))
    for f in range(frames):
        rng = np.random.default_rng(f)
        gone = 1 + rng.permutation(n - 1)[:[0, 1, n // 2, n - 300, n - 257, n - 256, n - 2, n // 5][f % 8]]
        boxes[f, gone] = base[0]
    perm = np.random.default_rng(9).permutation(n)
    check(nms, oracle, boxes, scores, 0.5)
    check(nms, oracle, boxes[:, perm], scores[:, perm], 0.5)


def test_y_ranges_and_literal_division(nms, oracle):
    for F, n in ((6, 4096), (20, 1800)):
        boxes, scores = uniform(770 + n, F, n, extent=3000, max_side=180, integer=False, score_levels=250)
        shifted = boxes.copy()
        for f in range(0, F, 2):
            idx = np.random.default_rng(f).permutation(n)[:1 + 7 * f]
            shifted[f, idx, 1] += 20000.0
            shifted[f, idx, 3] += 20000.0
        check(nms, oracle, shifted, scores, 0.4)
        for theta in (0.0, 2.0 ** -41, 1.5):
            check(nms, oracle, boxes, scores, theta)
        check(nms, oracle, shifted, scores, 0.0)


def test_scores_of_every_kind_and_equal_scores(nms, oracle):
    for F, n in ((5, 4000), (12, 2048)):
        boxes, _ = uniform(5 + n, F, n, extent=2500, max_side=150, integer=True)
        rng = np.random.default_rng(n)
        for f in range(F):
            src, dst = rng.integers(0, n, n // 3), rng.integers(0, n, n // 3)
            boxes[f, dst] = boxes[f, src]
        scores = np.stack([scores_of_every_kind(8 + f, n) for f in range(F)])
        check(nms, oracle, boxes, scores, 0.4)
        check(nms, oracle, boxes, np.full((F, n), 0.25, np.float32), 0.5)
        check(nms, oracle, boxes, np.where(rng.integers(0, 2, (F, n)) == 1, np.float32(0.0), np.float32(-0.0)), 0.5)
