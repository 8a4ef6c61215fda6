"""The one-launch route that nms_run_batched takes for batches of frames of 257 to 1024 boxes (no
sort: every victim against the two best-ranked of every sixteen input elements, the victims still
alive against the whole frame, rank order as a compare of the two boxes' keys; a frame shared out
among 1 to 16 workgroups) against the oracle's plain double loop, 0 differing bits, on what the
route itself can meet: every number of workgroups per frame, frame lengths around the tile and
stage sizes, ragged batches incl. empty frames and frames shorter than a tile, nothing / everything /
all but a few victims alive after the first stage (short and long lists for the second, at the
length where its form changes), eliminators that the first stage does not hold, equal scores,
y coordinates outside the scaled form's range, thresholds that take the literal division, scores
of every kind."""
import numpy as np
import pytest

from gpu_util import DeviceFrames, oracle_keep_frames
from pins import staircase
from workloads import clustered_frame, random_frame, scores_of_every_kind

pytestmark = pytest.mark.gpu

FIRST = 128  # boxes of the first stage: the two best-ranked of every 16 input elements


@pytest.fixture(scope="module")
def nms():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2502_00535_amd.binding as binding

    return binding


def check(nms, oracle, boxes, scores, theta, counts=None):
    """nms_run_batched (which routes these shapes to the one launch) and the explicit all-pairs route."""
    F, n = scores.shape
    assert nms.nms_route(n, F) == nms.NMS_ROUTE_SMALL_FRAMES, f"{F} x {n} is not a shape of the one-launch route"
    want = oracle_keep_frames(oracle, boxes, scores, np.float32(theta), counts)
    dev = DeviceFrames(nms, boxes, scores, counts)
    got = dev.fused(float(theta))
    assert np.array_equal(got, want), f"{(got != want).sum()} differing keep bits"
    dev.keep.fill_(77)
    nms.nms_run_ranked_batched(dev.boxes, dev.scores, dev.counts, n, F, float(theta), dev.keep, dev.run_ws)
    dev.torch.cuda.synchronize()
    assert np.array_equal(dev.keep.cpu().numpy(), want)
    return want


def lattice(n, rng=None, pitch=40.0, size=30.0):
    """n pairwise disjoint boxes."""
    side = int(np.ceil(np.sqrt(n)))
    gx, gy = np.meshgrid(np.arange(side), np.arange(side))
    cells = np.stack([gx.ravel() * pitch, gy.ravel() * pitch], 1)[:n]
    if rng is not None:
        cells = cells[rng.permutation(n)]
    return np.concatenate([cells, cells + size], 1).astype(np.float32)


def batch(seed, F, n, **kw):
    boxes = np.zeros((F, n, 4), np.float32)
    scores = np.zeros((F, n), np.float32)
    for f in range(F):
        boxes[f], scores[f] = random_frame(seed + f, n, **kw)
    return boxes, scores


@pytest.mark.parametrize("frames", [11, 12, 16, 17, 24, 25, 32, 33, 64, 65, 128, 129, 200, 256, 300, 500])
def test_workgroups_per_frame(nms, oracle, frames):
    """1024-box frames: 16, 8, 4, 2 and 1 workgroups per frame and batches beyond the compute units."""
    print(f"case frames={frames}", flush=True)
    rng = np.random.default_rng(frames)
    boxes, scores = batch(3000 + 7 * frames, frames, 1024, extent=900, max_side=120, integer=(frames % 2 == 0), score_levels=300)
    counts = rng.integers(0, 1025, frames).astype(np.int32) if frames % 3 == 0 else None
    want = check(nms, oracle, boxes, scores, 0.45, counts)
    assert 0 < want.sum() < want.size


@pytest.mark.parametrize("n", [513, 514, 575, 576, 577, 600, 639, 640, 641, 703, 704, 705, 767, 768, 769, 831, 895, 896, 897, 959, 960, 961, 1000, 1023, 1024])
def test_frame_lengths(nms, oracle, n):
    print(f"case n={n}", flush=True)
    F = max(40, (3 << 23) // (n * n) + 2)   # the direct form takes batches up to 3 * 2^23 pair slots
    boxes, scores = batch(5000 + n, F, n, extent=700, max_side=100, integer=(n % 2 == 1), score_levels=max(3, n // 3))
    want = check(nms, oracle, boxes, scores, [0.5, 0.3, 0.45][n % 3])
    assert 0 < want.sum() < want.size


def test_ragged_batches(nms, oracle):
    """Frames that are empty, shorter than a tile, shorter than the first stage, just beyond it, and full, in one call."""
    F, n_max = 80, 1024
    boxes, scores = batch(77, F, n_max, extent=800, max_side=110, integer=True, score_levels=200)
    counts = np.array(([0, 1, 2, 63, 64, 65, 127, 128, 129, 130, 191, 192, 193, 255, 256, 257, 1023, 1024, 700, 5] * 4)[:F], np.int32)
    check(nms, oracle, boxes, scores, 0.45, counts)
    check(nms, oracle, boxes[:, :600], scores[:, :600], 0.3, np.minimum(counts, 600).astype(np.int32)[:F])
    # 300 frames (one workgroup per frame), random counts
    F = 300
    boxes, scores = batch(99, F, 1000, extent=700, max_side=90, integer=False, score_levels=0)
    check(nms, oracle, boxes, scores, 0.4, np.random.default_rng(5).integers(0, 1001, F).astype(np.int32))


def test_live_victim_counts(nms, oracle):
    """Disjoint boxes in rank order, of which a chosen set repeats the box of rank 0 (eliminated in the
    first stage): the rest, `alive` of them behind rank 128, reach the second stage and survive."""
    n, F = 1024, 32
    base = lattice(n)
    scores = np.tile((1.0 - np.arange(n) / n).astype(np.float32), (F, 1))
    behind = n - FIRST
    boxes = np.zeros((F, n, 4), np.float32)
    alive_per_frame = [0, 1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 255, 256, 257, 500, 800, behind - 2,
                       behind - 1, behind, 6, 60]
    for f, alive in enumerate(alive_per_frame):
        rng = np.random.default_rng(alive + 1000 * f)
        boxes[f] = base
        dead = FIRST + rng.permutation(behind)[:behind - alive]
        boxes[f, dead] = base[0]
    want = check(nms, oracle, boxes, scores, 0.5)
    assert want.sum(1).tolist() == [FIRST + a for a in alive_per_frame]
    # the same frames with the input order shuffled (ranks no longer equal indices)
    perm = np.random.default_rng(1).permutation(n)
    check(nms, oracle, boxes[:, perm], scores[:, perm], 0.5)


def test_eliminators_only_behind_the_first_stage(nms, oracle):
    """Victim v repeats the box of rank e(v) >= 128, its one and only eliminator, so v is alive after the
    first stage and must be caught by the second: eliminators directly before their victims, at tile
    borders, at the borders of the second stage's groups of four tiles, and far apart."""
    n, F = 1024, 40
    boxes1 = lattice(n)
    scores = np.tile((1.0 - np.arange(n) / n).astype(np.float32), (F, 1))
    pairs = [(128, 129), (128, 1023), (191, 192), (192, 193), (255, 256), (383, 384), (384, 385), (384, 447), (384, 448), (385, 449),
             (639, 640), (640, 641), (895, 896), (896, 897), (896, 1022), (1020, 1021), (130, 700), (700, 701), (701, 702), (500, 501)]
    victims = set()
    for e, v in pairs:
        assert e < v and v not in victims
        boxes1[v] = boxes1[e]
        victims.add(v)
    boxes = np.tile(boxes1, (F, 1, 1))
    # every frame but the first: a different half of the other boxes eliminated in the first stage
    for f in range(1, F):
        gone = FIRST + np.random.default_rng(f).permutation(n - FIRST)[:(n - FIRST) // 2]
        keep_as_is = np.array(sorted({x for p in pairs for x in p}))
        gone = np.setdiff1d(gone, keep_as_is)
        boxes[f, gone] = boxes1[1]
    want = check(nms, oracle, boxes, scores, 0.5)
    assert sorted(np.flatnonzero(want[0] == 0).tolist()) == sorted(victims)


def test_extremes(nms, oracle):
    n, F = 1000, 48
    rng = np.random.default_rng(3)
    scores = np.stack([rng.permutation(n).astype(np.float32) / n for _ in range(F)])
    disjoint = np.stack([lattice(n, rng) for _ in range(F)])
    assert check(nms, oracle, disjoint, scores, 0.5).sum() == F * n                            # everything alive in both stages
    same = np.tile(np.array([[10, 10, 90, 70]], np.float32), (F, n, 1))
    assert check(nms, oracle, same, scores, 0.5).sum() == F                                    # nothing alive after the first stage
    b, s = staircase(n)
    assert check(nms, oracle, np.tile(b, (F, 1, 1)), np.tile(s, (F, 1)), 0.5).sum() == F       # each box eliminated by its predecessor only
    assert check(nms, oracle, np.tile(b[::-1].copy(), (F, 1, 1)), np.tile(s[::-1].copy(), (F, 1)), np.float32(0.4)).sum() == F


def test_clustered_detections(nms, oracle):
    """The workload the route is for: clusters of candidates around objects, 64 and 200 frames."""
    for F, n in ((64, 1024), (200, 768), (260, 960), (600, 704)):
        fr = [clustered_frame(900 + f, objects=n // 16, width=1920, height=1080, size_lo=32.0, size_hi=256.0) for f in range(F)]
        boxes = np.stack([x[0][:n] for x in fr])
        scores = np.stack([x[1][:n] for x in fr])
        print(f"case {F} x {boxes.shape[1]}", flush=True)
        want = check(nms, oracle, boxes, scores, 0.5)
        assert 0 < want.sum() < want.size // 4


def test_y_ranges_and_literal_division(nms, oracle):
    """Frames with y coordinates that rule out the scaled pair test (every third frame has boxes shifted
    far up), and thresholds that take the literal division, through both stages."""
    F, n = 60, 900
    boxes, scores = batch(770, F, n, extent=800, max_side=100, integer=False, score_levels=250)
    shifted = boxes.copy()
    for f in range(0, F, 3):
        idx = np.random.default_rng(f).permutation(n)[:1 + f]
        shifted[f, idx, 1] += 20000.0
        shifted[f, idx, 3] += 20000.0
    check(nms, oracle, shifted, scores, 0.4)
    for theta in (0.0, 2.0 ** -41, 1.5):
        check(nms, oracle, boxes, scores, theta)
    check(nms, oracle, shifted, scores, 0.0)


def test_scores_of_every_kind(nms, oracle):
    F, n = 50, 1024
    boxes, _ = batch(5, F, n, extent=700, max_side=100, integer=True)
    scores = np.stack([scores_of_every_kind(8 + f, n) for f in range(F)])
    check(nms, oracle, boxes, scores, 0.4)


def test_eliminators_that_the_first_stage_does_not_hold(nms, oracle):
    """Scores fall with the input index, so the first stage holds elements 0 and 1 of every sixteen.  Victims
    repeat the box of an element at position 2 .. 15 of a row (same row, same tile, an earlier tile, the tile
    before a tile-group border): alive after the first stage, caught only by the second; and victims that repeat
    a first-stage box of a later row do not fall (it is ranked behind them)."""
    n, F = 1024, 40
    base = lattice(n)
    scores = np.tile((1.0 - np.arange(n) / n).astype(np.float32), (F, 1))
    pairs = [(2, 3), (2, 15), (14, 31), (4, 16), (5, 63), (62, 79), (61, 64), (18, 200), (255, 256), (254, 257), (300, 1023), (1006, 1007),
             (130, 131), (515, 770), (766, 769)]
    assert all(e < v and e % 16 >= 2 for e, v in pairs)
    spared = [(33, 20), (161, 100), (1009, 500)]  # (first-stage box, a better-ranked element that repeats it)
    boxes1 = base.copy()
    victims = set()
    for e, v in pairs:
        assert v not in victims and all(v != a for a, _ in pairs + spared)
        boxes1[v] = base[e]
        victims.add(v)
    for e, v in spared:
        assert e % 16 < 2 and v < e and v not in victims and all(v not in p for p in pairs)
        boxes1[v] = base[e]
    boxes = np.tile(boxes1, (F, 1, 1))
    for f in range(1, F):  # every frame but the first: a different half of the other boxes falls in the first stage
        free = np.setdiff1d(np.arange(16, n), np.array(sorted({x for p in pairs + spared for x in p})))
        gone = np.random.default_rng(f).permutation(free)[:free.size // 2]
        boxes[f, gone] = base[0]
    want = check(nms, oracle, boxes, scores, 0.5)
    dead = set(np.flatnonzero(want[0] == 0).tolist())
    assert dead == victims | {e for e, _ in spared}
    perm = np.random.default_rng(2).permutation(n)
    check(nms, oracle, boxes[:, perm], scores[:, perm], 0.5)


def test_equal_scores(nms, oracle):
    """One score for the whole frame (and frames of two or three levels, +0.0 next to -0.0): rank order is input
    order, the lower index of a repeated box survives."""
    n, F = 1000, 44
    rng = np.random.default_rng(12)
    boxes = np.stack([lattice(n, rng) for _ in range(F)])
    for f in range(F):
        src = rng.integers(0, n, n // 2)
        dst = rng.integers(0, n, n // 2)
        boxes[f, dst] = boxes[f, src]
    scores = np.full((F, n), 0.25, np.float32)
    scores[1::4] = rng.integers(0, 2, (len(scores[1::4]), n)).astype(np.float32)
    scores[2::4] = rng.integers(0, 3, (len(scores[2::4]), n)).astype(np.float32) * np.float32(0.5) - np.float32(0.5)
    scores[3::4] = np.where(rng.integers(0, 2, (len(scores[3::4]), n)) == 1, np.float32(0.0), np.float32(-0.0))
    want = check(nms, oracle, boxes, scores, 0.5)
    assert 0 < want.sum() < want.size


@pytest.mark.parametrize("frames", [130, 260])
def test_long_lists(nms, oracle, frames):
    """Two workgroups per frame (130 frames) and one (260): disjoint boxes of which a chosen number repeat the
    best-ranked one, so that a workgroup lists 0 .. all of its 512 or 1024 victims for the second stage -- around 256,
    where the second stage changes its form -- and some of the listed fall to boxes that the first stage does not hold."""
    n = 1024
    share = n // (2 if frames <= 256 else 1)
    per_group = [0, 1, 100, 254, 255, 256, 257, 258, 300, 319, 320, 321, 400, 511, 512, 513, 640, 767, 768, 769, 1000, 1022, 1023, 1024]
    scores = np.tile((1.0 - np.arange(n) / n).astype(np.float32), (frames, 1))
    base = lattice(n)
    boxes = np.zeros((frames, n, 4), np.float32)
    for f in range(frames):
        rng = np.random.default_rng(1000 * frames + f)
        alive = min(per_group[f % len(per_group)], share) * (n // share)
        boxes[f] = base
        gone = 1 + rng.permutation(n - 1)[:n - max(alive, 1)]
        boxes[f, gone] = base[0]
        stay = np.setdiff1d(np.arange(2, n), gone)
        late = stay[stay % 16 >= 3]
        for v in rng.permutation(late)[:min(7, late.size)]:  # falls to its unpicked neighbour, in the second stage
            if (v - 1) % 16 >= 2 and boxes[f, v - 1, 0] == base[v - 1, 0]:
                boxes[f, v] = base[v - 1]
    print(f"case frames={frames}", flush=True)
    want = check(nms, oracle, boxes, scores, 0.5)
    assert want.sum(1).min() <= 8 and want.sum(1).max() >= n - 8
    perm = np.random.default_rng(3).permutation(n)
    check(nms, oracle, boxes[:, perm], scores[:, perm], 0.5)


@pytest.mark.parametrize("frames,n", [(22, 700), (12, 960), (16, 900), (28, 641), (40, 600), (11, 1000)])
def test_few_short_frames(nms, oracle, frames, n):
    """More workgroups per frame than the frame has tiles of victims (some workgroups have none), shares of one
    and two tiles, a last tile that is not full."""
    print(f"case {frames} x {n}", flush=True)
    boxes, scores = batch(8000 + n, frames, n, extent=800, max_side=110, integer=(n % 2 == 0), score_levels=n // 2)
    counts = None
    if frames % 2 == 0:
        counts = np.random.default_rng(n).integers(0, n + 1, frames).astype(np.int32)
        counts[:4] = [n, 0, 1, 65]
    want = check(nms, oracle, boxes, scores, 0.45, counts)
    assert 0 < want.sum() < want.size


@pytest.mark.parametrize("frames,n", [(128, 512), (129, 449), (300, 500), (600, 480), (1030, 512)])
def test_frames_of_at_most_512_boxes(nms, oracle, frames, n):
    """The same kernel body in workgroups of eight wavefronts: one, two and four workgroups per frame, batches
    beyond four workgroups per compute unit, ragged counts, sparse frames (long lists), equal scores."""
    print(f"case {frames} x {n}", flush=True)
    boxes, scores = batch(9000 + n, frames, n, extent=600, max_side=100, integer=(n % 2 == 0), score_levels=n // 2)
    counts = None
    if frames % 2 == 0:
        counts = np.random.default_rng(n).integers(0, n + 1, frames).astype(np.int32)
        counts[:4] = [n, 0, 1, 65]
    want = check(nms, oracle, boxes, scores, 0.45, counts)
    assert 0 < want.sum() < want.size
    sparse, _ = batch(9500 + n, frames, n, extent=100000, max_side=60, integer=False)
    assert check(nms, oracle, sparse, scores, 0.5, counts).sum() > 0.4 * frames * n
    check(nms, oracle, boxes, np.full((frames, n), -1.5, np.float32), 0.3)
    check(nms, oracle, boxes, scores, 0.0)


def test_route_can_be_captured_in_a_hip_graph(nms, oracle):
    """The route enqueues one kernel and nothing else, so it may be captured; replays with new inputs in the same
    buffers and eager work in between must give the oracle's keep vectors (frames of 1000, 500 and 3000 boxes: the three
    kernels of the route)."""
    import torch

    dev = torch.device("cuda:0")
    for F, n in ((24, 1000), (130, 500), (5, 3000)):
        assert nms.nms_route(n, F) == nms.NMS_ROUTE_SMALL_FRAMES
        boxes = torch.zeros((F, n, 4), dtype=torch.float32, device=dev)
        scores = torch.zeros((F, n), dtype=torch.float32, device=dev)
        keep = torch.zeros((F, n), dtype=torch.uint8, device=dev)
        ws = torch.zeros(nms.nms_workspace_bytes(n, F), dtype=torch.uint8, device=dev)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            nms.nms_run_batched(boxes, scores, None, n, F, 0.45, keep, ws)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                nms.nms_run_batched(boxes, scores, None, n, F, 0.45, keep, ws)
        torch.cuda.synchronize()
        for rep in range(3):
            b, s = batch(31000 + 1000 * rep + n, F, n, extent=900, max_side=120, integer=(rep % 2 == 0), score_levels=100)
            boxes.copy_(torch.from_numpy(b))
            scores.copy_(torch.from_numpy(s))
            keep.fill_(9)
            (boxes.sum() + scores.sum()).item()
            graph.replay()
            torch.cuda.synchronize()
            want = oracle_keep_frames(oracle, b, s, np.float32(0.45))
            assert np.array_equal(keep.cpu().numpy(), want), f"{F} x {n}, replay {rep}"
