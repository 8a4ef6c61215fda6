"""The two-launch route that nms_run_batched takes for a few frames of more than 4096 boxes
(first launch: every victim against the best 2048 ranks; second launch: the victims still alive,
64 consecutive live ones per wavefront, against the rest) against the oracle's plain double loop,
0 differing bits, on what the route itself can meet: nothing alive after the first launch,
everything alive, exactly one live victim, live counts on and next to multiples of 64, eliminators
that sit only behind rank 2048 (in the tile of their victim's own run, at run and tile borders),
ragged batches whose frames end before, at and behind rank 2048, y coordinates outside the scaled
form's range, thresholds that take the literal division, scores of every kind."""
import numpy as np
import pytest

from gpu_util import DeviceFrames, oracle_keep_frames
from pins import staircase
from workloads import crowd_frame, random_frame, scores_of_every_kind

pytestmark = pytest.mark.gpu

FIRST = 2048  # ranks that the first launch tests every victim against


@pytest.fixture(scope="module")
def nms():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2502_00535_amd.binding as binding

    return binding


def check(nms, oracle, boxes, scores, theta, counts=None):
    """nms_run_batched (which routes these sizes to the two launches) and the explicit all-pairs route."""
    F, n = scores.shape
    assert nms.nms_route(n, F) == nms.NMS_ROUTE_TWO_LAUNCH, "not a size of the two-launch route"
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


@pytest.mark.parametrize("n", [11586, 11587, 12000, 12345, 16384, 20000, 30000])
def test_single_frame_lengths(nms, oracle, n):
    print(f"case n={n}", flush=True)
    boxes, scores = random_frame(4400 + n, n, extent=3000, max_side=110, integer=(n % 2 == 0), score_levels=max(3, n // 4))
    want = check(nms, oracle, boxes[None], scores[None], [0.5, 0.3, 0.45][n % 3])
    assert 1 <= want.sum() < n


def test_live_victim_counts(nms, oracle):
    """Disjoint boxes in rank order, of which a chosen set repeats the box of rank 0 (eliminated in the
    first launch): the rest, `alive` of them behind rank 2048, reach the second launch and survive."""
    n = 12000
    base = lattice(n)
    scores = (1.0 - np.arange(n) / n).astype(np.float32)
    behind = n - FIRST
    for alive in (0, 1, 2, 63, 64, 65, 127, 128, 129, 1000, behind - 1, behind):
        print(f"case alive={alive}", flush=True)
        rng = np.random.default_rng(alive)
        boxes = base.copy()
        dead = FIRST + rng.permutation(behind)[:behind - alive]
        boxes[dead] = boxes[0]
        want = check(nms, oracle, boxes[None], scores[None], 0.5)
        assert want.sum() == FIRST + alive


def test_eliminators_only_behind_the_first_launch(nms, oracle):
    """Victim v repeats the box of rank e(v) >= 2048, its one and only eliminator, so v is alive after
    the first launch and must be caught by the second: eliminators directly before their victims (the
    tile that holds the run's own victims), at tile and run borders, and far apart."""
    n = 14000
    boxes = lattice(n)
    scores = (1.0 - np.arange(n) / n).astype(np.float32)
    pairs = [(2048, 2049), (2048, 13999), (2111, 2112), (2112, 2113), (2175, 2176), (3000, 3001), (3000, 3063),
             (3000, 3064), (3000, 3065), (4095, 4096), (4096, 4160), (8191, 8192), (8192, 13998), (13996, 13997),
             (2050, 9000), (9000, 9001), (9001, 9002), (5000, 5001), (5003, 5004)]   # 9000 -> 9001 -> 9002: a chain of copies
    victims = set()
    for e, v in pairs:
        assert e < v and v not in victims
        boxes[v] = boxes[e]
        victims.add(v)
    want = check(nms, oracle, boxes[None], scores[None], 0.5)
    assert sorted(np.flatnonzero(want[0] == 0).tolist()) == sorted(victims)
    # the same with every second box eliminated in the first launch, so that runs of live victims span many tiles
    boxes2 = boxes.copy()
    boxes2[FIRST + 1:n:2] = boxes2[1]
    for e, v in pairs:
        boxes2[e] = boxes[e]
        boxes2[v] = boxes[e]
    check(nms, oracle, boxes2[None], scores[None], 0.5)


def test_extremes(nms, oracle):
    n = 12000
    rng = np.random.default_rng(3)
    scores = rng.permutation(n).astype(np.float32) / n
    assert check(nms, oracle, lattice(n, rng)[None], scores[None], 0.5).sum() == n          # everything alive
    same = np.tile(np.array([[10, 10, 90, 70]], np.float32), (n, 1))
    assert check(nms, oracle, same[None], scores[None], 0.5).sum() == 1                     # nothing alive
    b, s = staircase(n)
    assert check(nms, oracle, b[None], s[None], 0.5).sum() == 1                            # each box eliminated by its predecessor only
    assert check(nms, oracle, b[::-1].copy()[None], s[::-1].copy()[None], np.float32(0.4)).sum() == 1


def test_ragged_batches(nms, oracle):
    """Frames that end before, at and behind the first launch's ranks, in one call."""
    rng = np.random.default_rng(9)
    n_max, F = 9000, 6
    counts = np.array([9000, 0, 2048, 2049, 1500, 6001], np.int32)
    boxes = np.zeros((F, n_max, 4), np.float32)
    scores = np.zeros((F, n_max), np.float32)
    for f in range(F):
        boxes[f], scores[f] = random_frame(600 + f, n_max, extent=2500, max_side=100, integer=(f % 2 == 0), score_levels=900)
    check(nms, oracle, boxes, scores, 0.45, counts)
    counts2 = rng.integers(0, n_max + 1, F).astype(np.int32)
    check(nms, oracle, boxes, scores, 0.3, counts2)


def test_dense_crowd_batches(nms, oracle):
    """The workload the route is for: dense crowd scenes with exact ties, 1, 2 and 4 frames."""
    for F, grid in ((1, 28), (2, 32), (4, 24)):
        fr = [crowd_frame(70 + f, grid=grid) for f in range(F)]
        boxes = np.stack([x[0] for x in fr])
        scores = np.stack([x[1] for x in fr])
        print(f"case {F} x {boxes.shape[1]}", flush=True)
        check(nms, oracle, boxes, scores, 0.3)


def test_y_ranges_and_literal_division(nms, oracle):
    """Tiles whose y coordinates rule out the scaled pair test (every third box of some rank ranges is
    shifted far up), and thresholds that take the literal division, through both launches."""
    n = 12000
    boxes, scores = random_frame(77, n, extent=2600, max_side=100, integer=False, score_levels=2500)
    shifted = boxes.copy()
    order = np.argsort(-scores, kind="stable")
    for lo, hi in ((0, 200), (2000, 2300), (5000, 5100), (11900, 12000)):   # rank ranges before, across and behind rank 2048
        idx = order[lo:hi:3]
        shifted[idx, 1] += 20000.0
        shifted[idx, 3] += 20000.0
    check(nms, oracle, shifted[None], scores[None], 0.4)
    for theta in (0.0, 2.0 ** -41, 1.5):
        check(nms, oracle, boxes[None], scores[None], theta)
    check(nms, oracle, shifted[None], scores[None], 0.0)


def test_scores_of_every_kind(nms, oracle):
    n = 12000
    boxes, _ = random_frame(5, n, extent=2400, max_side=100, integer=True)
    check(nms, oracle, boxes[None], scores_of_every_kind(8, n)[None], 0.4)
