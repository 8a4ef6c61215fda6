"""nms_run_early_exit_batched (the paper's rule with eliminated victims dropped from further tests)
against the oracle's plain double loop, 0 differing bits, on what the route itself can meet: lists
that never shrink, lists that empty at once, eliminators sitting exactly at the stage bounds, ragged
frame lengths around the tile and stage sizes, frames that must leave the y-scaled pair test, and
thresholds that take the literal division."""
import numpy as np
import pytest

from gpu_util import DeviceFrames, oracle_keep_frames
from pins import staircase
from workloads import make_config, random_frame

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nms():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2502_00535_amd.binding as binding

    return binding


def check(nms, oracle, boxes, scores, theta, counts=None):
    want = oracle_keep_frames(oracle, boxes, scores, np.float32(theta), counts)
    dev = DeviceFrames(nms, boxes, scores, counts)
    got = dev.early_exit(float(theta))
    assert np.array_equal(got, want), f"{(got != want).sum()} differing keep bits"
    return want


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 511, 513, 1000, 1025,
                               2047, 2049, 3000, 4095, 4096, 4097, 5000, 8191, 8193, 12345, 16384, 20000])
def test_single_frame_lengths(nms, oracle, n):
    print(f"case n={n}", flush=True)
    boxes, scores = random_frame(9100 + n, n, extent=1500 if n > 600 else 300, max_side=90,
                                 integer=(n % 2 == 0), score_levels=max(3, n // 4))
    want = check(nms, oracle, boxes[None], scores[None], [0.5, 0.3, 0.45][n % 3])
    assert want.sum() >= 1


def test_list_extremes(nms, oracle):
    """Nothing ever eliminated (the list only loses the survivors of each stage), everything
    eliminated by the first box (the list is empty after the first stage), exactly the better half
    surviving, and the staircase (every box eliminated by its predecessor only)."""
    rng = np.random.default_rng(81)
    for n in (4096, 3000, 1100, 200):
        side = 64
        gx, gy = np.meshgrid(np.arange(side), np.arange(side))
        cells = np.stack([gx.ravel() * 40.0, gy.ravel() * 40.0], 1)[rng.permutation(side * side)[:n]]
        disjoint = np.concatenate([cells, cells + 30.0], 1).astype(np.float32)
        scores = rng.permutation(n).astype(np.float32) / n
        assert check(nms, oracle, disjoint[None], scores[None], 0.5).sum() == n
        same = np.tile(np.array([[10, 10, 90, 70]], np.float32), (n, 1))
        assert check(nms, oracle, same[None], scores[None], 0.5).sum() == 1
        half = disjoint.copy()
        half[n // 2:] = half[:n - n // 2]
        scores2 = np.concatenate([1.0 + scores[:n // 2], scores[n // 2:] * 0.5]).astype(np.float32)
        want = check(nms, oracle, half[None], scores2[None], 0.5)
        assert want[0, :n // 2].all() and not want[0, n // 2:].any()
        b, s = staircase(n)
        assert check(nms, oracle, b[None], s[None], 0.5).sum() == 1


def test_single_eliminator_at_every_stage_bound(nms, oracle):
    """Disjoint boxes, except that victim v repeats the box of rank e(v): its one and only
    eliminator.  The eliminators sit on and next to the stage bounds and tile edges (ranks 0, 63,
    64, 127, 128, 129, 255, 256, ... 4094), the victims right behind them and at the far end."""
    n = 4096
    side = 64
    gx, gy = np.meshgrid(np.arange(side), np.arange(side))
    cells = np.stack([gx.ravel() * 40.0, gy.ravel() * 40.0], 1)
    boxes = np.concatenate([cells, cells + 30.0], 1).astype(np.float32)   # rank order: scores descend with the index
    scores = (1.0 - np.arange(n) / n).astype(np.float32)
    elim = [0, 1, 63, 64, 65, 127, 128, 129, 191, 192, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2047, 2048,
            2049, 3071, 3072, 4000, 4094]
    dead = set()
    for k, e in enumerate(elim):
        for v in (e + 1, e + 2 + 37 * k, n - 1 - 2 * k, n - 2 - 2 * k if k % 2 else e + 64):
            if e < v < n and v not in dead and v not in elim:
                boxes[v] = boxes[e]
                dead.add(v)
    rng = np.random.default_rng(5)
    perm = rng.permutation(n)                                              # the input itself is unsorted
    want = check(nms, oracle, boxes[perm][None], scores[perm][None], 0.5)
    assert want.sum() == n - len(dead)
    counts = np.array([n, 2049, 1024, 130], np.int32)                      # and cut short, one frame each
    check(nms, oracle, np.tile(boxes[None], (4, 1, 1)), np.tile(scores[None], (4, 1)), 0.5, counts)


def test_frames_that_leave_the_scaled_form(nms, oracle):
    """A batch in which some frames have y coordinates outside the y-scaled form's range (above
    8190, or tiny): those are staged again unscaled and take the plain form of the pair test."""
    n, F = 2100, 24
    base_b, base_s = random_frame(9300, n, extent=3000, max_side=300, integer=False, score_levels=500)
    boxes = np.tile(base_b[None], (F, 1, 1))
    scores = np.tile(base_s[None], (F, 1))
    for f in range(F):
        if f % 3 == 1:
            boxes[f, f * 7 % n, [1, 3]] += np.float32(9000.0)             # one box far down
        elif f % 3 == 2:
            boxes[f, ::5, [1, 3]] *= np.float32(2.0 ** -70)               # many boxes with tiny y
        rng = np.random.default_rng(f)
        p = rng.permutation(n)
        boxes[f], scores[f] = boxes[f][p], scores[f][p]
    counts = np.full(F, n, np.int32)
    counts[[4, 5, 9]] = [1000, 0, 65]
    for theta in (0.4, 0.7):
        want = check(nms, oracle, boxes, scores, theta, counts)
    assert 0 < want.sum() < want.size


@pytest.mark.parametrize("theta", [0.0, -0.5, 1.0, 1.5, 1e-13, 3e6, float("inf")])
def test_thresholds_of_the_literal_division(nms, oracle, theta):
    print(f"case theta={theta}", flush=True)
    n, F = 700, 6
    boxes = np.zeros((F, n, 4), np.float32)
    scores = np.zeros((F, n), np.float32)
    for f in range(F):
        boxes[f], scores[f] = random_frame(9400 + f, n, extent=600, max_side=150, integer=(f % 2 == 0), score_levels=80)
    counts = np.array([n, n - 1, 64, 129, 0, 513], np.int32)
    check(nms, oracle, boxes, scores, theta, counts)


def test_score_ties(nms, oracle):
    """Equal scores: the lower index outranks; identical boxes with identical scores keep one."""
    n = 1500
    boxes, _ = random_frame(9500, n, extent=500, max_side=120, integer=True, score_levels=5)
    rng = np.random.default_rng(3)
    scores = rng.integers(0, 4, n).astype(np.float32) * np.float32(0.25)
    scores[::97] = np.float32(-0.0)
    boxes[1::2] = boxes[::2]
    check(nms, oracle, boxes[None], scores[None], 0.5)


@pytest.mark.parametrize("frames", [3, 16, 17, 33, 64, 65, 128, 129, 200])
def test_frames_shared_out_among_workgroups(nms, oracle, frames):
    """Batches of fewer frames than the chip has compute units: a frame's victims are shared out
    among 16, 8, 4 or 2 workgroups (ranks part, part + parts, ...), ragged counts included (some
    shares then stay empty)."""
    print(f"case frames={frames}", flush=True)
    n = 1500
    rng = np.random.default_rng(frames)
    boxes = np.zeros((frames, n, 4), np.float32)
    scores = np.zeros((frames, n), np.float32)
    for f in range(min(frames, 12)):
        boxes[f], scores[f] = random_frame(9600 + f, n, extent=900, max_side=140, integer=(f % 2 == 0), score_levels=300)
    for f in range(12, frames):
        p = rng.permutation(n)
        boxes[f], scores[f] = boxes[f % 12][p], scores[f % 12][p]
    counts = rng.integers(0, n + 1, frames).astype(np.int32)
    counts[:3] = [n, 5, 0]
    want = check(nms, oracle, boxes, scores, 0.45, counts)
    assert 0 < want.sum() < want.size
    check(nms, oracle, boxes[:, :700], scores[:, :700], 0.6)


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_configs_full_size(nms, oracle, index):
    print(f"case config={index}", flush=True)
    w = make_config(index)
    want = check(nms, oracle, w.boxes, w.scores, w.theta)
    assert 0 < want.sum() < want.size


def test_wide_frames_batched(nms, oracle):
    """Frames beyond 4096 boxes (only a workgroup's share of the victims is staged, candidates come
    from the ranked table in memory): batches of 1, 3 and 40 frames with ragged counts, both forms
    of the pair test."""
    n = 6000
    base_b, base_s = random_frame(9700, n, extent=2500, max_side=260, integer=False, score_levels=2000)
    for frames, theta in ((1, 0.5), (3, 0.3), (40, 0.45), (3, 0.0), (2, 1.5)):
        rng = np.random.default_rng(frames)
        boxes = np.zeros((frames, n, 4), np.float32)
        scores = np.zeros((frames, n), np.float32)
        for f in range(frames):
            p = rng.permutation(n)
            boxes[f], scores[f] = base_b[p], base_s[p]
        counts = rng.integers(0, n + 1, frames).astype(np.int32)
        counts[0] = n
        if frames > 2:
            counts[1:3] = [4097, 100]
        check(nms, oracle, boxes, scores, theta, counts)
    b, s = staircase(9000)
    assert check(nms, oracle, b[None], s[None], 0.5).sum() == 1
    same = np.tile(np.array([[10, 10, 90, 70]], np.float32), (7000, 1))
    sc = (np.arange(7000)[::-1] / 7000).astype(np.float32)
    assert check(nms, oracle, same[None], sc[None], 0.5).sum() == 1


def test_sizes_beyond_the_limit_are_refused(nms):
    assert nms.lib.nms_run_early_exit_batched(None, None, None, 65537, 1, 0.5, None, None, 0, None) == nms.NMS_ERR_TOO_LARGE
