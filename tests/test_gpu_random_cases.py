"""Seeded random cases across every entry point: random frame counts and lengths (ragged,
including empty frames), thresholds, coordinate styles and options, each compared with the
oracle bit for bit.  The cases are fixed by their seeds; nothing here is time-dependent."""
import numpy as np
import pytest

from gpu_util import DeviceFrames, oracle_keep_frames
from test_gpu_variants import ExFrames, oracle_ex
from workloads import random_frame

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nms():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2502_00535_amd.binding as binding

    return binding


def random_batch(rng, case):
    shape = case % 4
    if shape == 0:      # a few long frames
        F, n_max = int(rng.integers(1, 4)), int(rng.integers(1500, 6000))
    elif shape == 1:    # many short frames
        F, n_max = int(rng.integers(20, 120)), int(rng.integers(1, 400))
    elif shape == 2:    # enough boxes for the greedy rule's mask-free walk (frames * n_max well above its threshold)
        n_max = int(rng.integers(600, 1400))
        F = (128 * 4096) // n_max + int(rng.integers(1, 20))
    else:               # around the tile and chunk borders
        F, n_max = int(rng.integers(1, 6)), int(rng.choice([63, 64, 65, 255, 256, 257, 4095, 4096, 4097]))
    counts = rng.integers(0, n_max + 1, F).astype(np.int32)
    counts[rng.integers(0, F)] = n_max
    if F > 2:
        counts[rng.integers(0, F)] = 0
    boxes = np.zeros((F, n_max, 4), np.float32)
    scores = np.zeros((F, n_max), np.float32)
    extent = float(rng.choice([150, 600, 3000]))
    side = float(rng.choice([30, 120, 400]))
    base = [random_frame(int(rng.integers(1 << 30)), n_max, extent=extent, max_side=side, integer=bool(rng.integers(2)),
                         score_levels=int(rng.choice([0, 7, 200]))) for _ in range(min(F, 6))]
    for f in range(F):
        b, s = base[f % len(base)]
        perm = rng.permutation(n_max) if f >= len(base) else np.arange(n_max)
        boxes[f], scores[f] = b[perm], s[perm]
    theta = float(np.float32(rng.choice([0.3, 0.45, 0.5, 0.7, rng.uniform(0.05, 0.95)])))
    return boxes, scores, counts, theta


@pytest.mark.parametrize("case", range(32))
def test_default_rule_and_greedy_rule(nms, oracle, case):
    rng = np.random.default_rng(9000 + case)
    boxes, scores, counts, theta = random_batch(rng, case)
    print(f"case {case}: frames={scores.shape[0]} n_max={scores.shape[1]} theta={theta}", flush=True)
    use_counts = counts if case % 3 else None
    want = oracle_keep_frames(oracle, boxes, scores, np.float32(theta), use_counts)
    dev = DeviceFrames(nms, boxes, scores, use_counts)
    dev.fused(theta, want=want)                       # automatic, ranked and (where bounded) direct route
    assert np.array_equal(dev.steps(theta), want)     # rank -> mask -> reduce
    want_g = oracle_keep_frames(oracle, boxes, scores, np.float32(theta), use_counts, rule="greedy")
    via_steps, one_call = dev.greedy(theta)           # sweep on the mask, the one call, the mask-free walk
    assert np.array_equal(via_steps, want_g) and np.array_equal(one_call, want_g)


@pytest.mark.parametrize("case", range(24))
def test_variants(nms, oracle, case):
    rng = np.random.default_rng(9500 + case)
    boxes, scores, counts, theta = random_batch(rng, case)
    F, n_max = scores.shape
    if F * n_max > 700_000:  # keep the oracle's share of the test short
        keep_frames = max(1, 700_000 // n_max)
        boxes, scores, counts = boxes[:keep_frames], scores[:keep_frames], counts[:keep_frames]
    classes = rng.integers(0, int(rng.choice([1, 2, 5])), scores.shape).astype(np.int32)
    dev = ExFrames(nms, boxes, scores, classes, counts)
    for _ in range(4):
        opts = dict(rule=str(rng.choice(["paper", "greedy"])), measure=str(rng.choice(["outranking_area", "iou"])),
                    compare=str(rng.choice(["ge", "gt"])), ties=str(rng.choice(["index", "ignore"])),
                    pixel_offset=float(rng.choice([0.0, 1.0])), labelled=bool(rng.integers(2)))
        print(f"case {case}: frames={scores.shape[0]} n_max={n_max} theta={theta} {opts}", flush=True)
        want = oracle_ex(oracle, boxes, scores, classes, theta, opts, counts)
        got = dev.run(theta, opts)
        assert np.array_equal(got, want), f"{opts}: {(got != want).sum()} differing keep bits"


@pytest.mark.parametrize("case", range(36))
def test_batches_of_the_one_launch_route(nms, oracle, case):
    """Random batch shapes among those that nms_run_batched gives to its sort-free one-launch kernels (frames of 449
    to 4096 boxes; see nms_route), with random counts, coordinate styles, score levels (down to a single one) and
    thresholds (including 0 and beyond 1); the all-pairs and early-exit routes are run beside it."""
    rng = np.random.default_rng(9900 + case)
    while True:
        if case % 3 == 0:
            n_max, F = int(rng.integers(449, 1025)), int(rng.choice([11, 16, 24, 33, 64, 100, 128, 129, 200, 256, 300, 520, 900]))
        elif case % 3 == 1:
            n_max = int(rng.integers(1025, 4097))
            F = (1 << 25) // (n_max * n_max) + int(rng.integers(1, 24))
        else:
            n_max, F = int(rng.choice([449, 512, 513, 577, 640, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096])), int(rng.integers(2, 140))
        if nms.nms_route(n_max, F) == nms.NMS_ROUTE_SMALL_FRAMES:
            break
    boxes = np.zeros((F, n_max, 4), np.float32)
    scores = np.zeros((F, n_max), np.float32)
    extent = float(rng.choice([200, 900, 4000, 100000]))
    side = float(rng.choice([30, 120, 400]))
    base = [random_frame(int(rng.integers(1 << 30)), n_max, extent=extent, max_side=side, integer=bool(rng.integers(2)),
                         score_levels=int(rng.choice([0, 1, 2, 9, 300]))) for _ in range(min(F, 5))]
    for f in range(F):
        b, s = base[f % len(base)]
        perm = rng.permutation(n_max) if f >= len(base) else np.arange(n_max)
        boxes[f], scores[f] = b[perm], s[perm]
    counts = rng.integers(0, n_max + 1, F).astype(np.int32)
    counts[rng.integers(0, F)] = n_max
    counts[rng.integers(0, F)] = int(rng.choice([0, 1, 63, 64, 65]))
    use_counts = counts if case % 2 else None
    theta = float(np.float32(rng.choice([0.0, 0.3, 0.45, 0.5, 0.7, 1.0, 1.25, rng.uniform(0.05, 0.95)])))
    print(f"case {case}: frames={F} n_max={n_max} theta={theta}", flush=True)
    want = oracle_keep_frames(oracle, boxes, scores, np.float32(theta), use_counts)
    DeviceFrames(nms, boxes, scores, use_counts).fused(theta, want=want)

