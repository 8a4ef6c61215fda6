"""Scores of every kind through every route: Algorithm 1's guard D[i].s < D[j].s is a
float comparison, valid for negative scores (raw logits), both zeros, denormals and
infinities alike.  Frames mixing all of these with exact ties, through the automatic /
ranked / direct / early-exit routes, the three step calls (order, mask, keep), the greedy
routes, the byte-matrix form and two option sets of the variants call.  Bar: 0 differing bits.
"""
import numpy as np
import pytest

from gpu_util import DeviceFrames, oracle_keep_frames
from test_gpu_matrix_form import expected as matrix_expected
from test_gpu_matrix_form import run_matrix_form
from test_gpu_variants import ExFrames, oracle_ex
from workloads import random_frame, scores_of_every_kind

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nms():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2502_00535_amd.binding as binding

    return binding


def frame(n, seed):
    boxes, _ = random_frame(seed, n, extent=1500 if n > 600 else 300, max_side=90, integer=(seed % 2 == 0))
    return boxes, scores_of_every_kind(seed, n)


@pytest.mark.parametrize("n", [7, 65, 1500, 4097, 6000])
def test_single_frame_every_route(nms, oracle, n):
    print(f"case n={n}", flush=True)
    boxes, scores = frame(n, 300 + n)
    theta = np.float32(0.4)
    dev = DeviceFrames(nms, boxes[None], scores[None])
    want = oracle.keep(boxes, scores, theta)
    dev.fused(float(theta), want=want[None])            # automatic, ranked, direct, early-exit
    assert np.array_equal(dev.steps(float(theta))[0], want)
    order = oracle.order(scores)
    assert np.array_equal(dev.host_order()[0, :n], order), "rank order"
    n_pad = dev.n_pad
    words = oracle.ranked_elimination_words(boxes, order, theta)
    got = dev.host_mask()[0].reshape(n_pad // 64, n_pad)
    for w in range(n_pad // 64):
        assert np.array_equal(got[w, 64 * w:n], words[64 * w:, w]), f"mask word column {w}"
    # classic greedy rule: sweep on the mask, routed call, mask-free walk (n <= 4096)
    want_g = oracle.greedy_keep(boxes, scores, theta)
    via_steps, one_call = dev.greedy(float(theta))
    assert np.array_equal(via_steps[0], want_g) and np.array_equal(one_call[0], want_g)


def test_special_values_only(nms, oracle):
    """Frames whose scores are nothing but special values, so every tile border of the
    rank step and every padding slot meets them: all -inf, all +inf, -inf against the
    padding of a ragged tail, zeros of both signs, denormals of both signs."""
    tiny = np.float32(1e-45)
    pools = {
        "all_minus_inf": [-np.inf],
        "all_plus_inf": [np.inf],
        "infinities": [-np.inf, np.inf],
        "zeros": [0.0, -0.0],
        "denormals": [tiny, -tiny, 2 * tiny, -2 * tiny, 0.0, -0.0],
        "ends": [-np.inf, -3.4028235e38, 3.4028235e38, np.inf, -tiny, tiny],
    }
    for name, pool in pools.items():
        for n in (63, 130, 1030, 4100):
            print(f"case {name} n={n}", flush=True)
            rng = np.random.default_rng(n)
            boxes, _ = random_frame(n, n, extent=200 if n < 2000 else 700, max_side=80, integer=True)
            scores = np.array(pool, np.float32)[rng.integers(0, len(pool), n)]
            theta = np.float32(0.5)
            want = oracle.keep(boxes, scores, theta)
            dev = DeviceFrames(nms, boxes[None], scores[None])
            dev.fused(float(theta), want=want[None])
            assert np.array_equal(dev.steps(float(theta))[0], want)
            assert np.array_equal(dev.host_order()[0, :n], oracle.order(scores))


def test_ragged_batch(nms, oracle):
    rng = np.random.default_rng(77)
    n_max, F = 900, 48
    counts = rng.integers(0, n_max + 1, F).astype(np.int32)
    counts[:5] = [0, 1, 64, 65, n_max]
    boxes = np.zeros((F, n_max, 4), np.float32)
    scores = np.zeros((F, n_max), np.float32)
    for f in range(F):
        boxes[f], scores[f] = frame(n_max, 800 + f)
    theta = np.float32(0.45)
    want = oracle_keep_frames(oracle, boxes, scores, theta, counts)
    dev = DeviceFrames(nms, boxes, scores, counts)
    dev.fused(float(theta), want=want)
    assert np.array_equal(dev.steps(float(theta)), want)
    want_g = oracle_keep_frames(oracle, boxes, scores, theta, counts, rule="greedy")
    via_steps, one_call = dev.greedy(float(theta))
    assert np.array_equal(via_steps, want_g) and np.array_equal(one_call, want_g)


def test_large_batch_early_exit_in_kernel_rank(nms, oracle):
    """Enough frames of more than 2048 boxes that the early-exit route ranks inside its kernel."""
    F, n = 260, 2500
    boxes = np.zeros((F, n, 4), np.float32)
    scores = np.zeros((F, n), np.float32)
    for f in range(F):
        boxes[f], scores[f] = frame(n, 2000 + f)
    theta = np.float32(0.5)
    want = oracle_keep_frames(oracle, boxes, scores, theta)
    dev = DeviceFrames(nms, boxes, scores)
    assert np.array_equal(dev.early_exit(float(theta)), want)
    assert np.array_equal(dev.fused(float(theta)), want)


@pytest.mark.parametrize("n,capacity", [(65, 128), (1500, 1536)])
def test_matrix_form(nms, oracle, n, capacity):
    boxes, scores = frame(n, 900 + n)
    theta = 0.4
    B, V = run_matrix_form(nms, boxes, scores, n, capacity, theta, [4, 32])
    want_B, want_V = matrix_expected(oracle, boxes, scores, n, capacity, theta)
    assert np.array_equal(B, want_B), f"{(B != want_B).sum()} differing matrix bytes"
    assert np.array_equal(V[4], want_V) and np.array_equal(V[32], want_V)


@pytest.mark.parametrize("n", [65, 1500, 4097])
def test_variants(nms, oracle, n):
    """ties ignored (the strict score test as printed) and labelled boxes, both rules."""
    boxes, scores = frame(n, 1300 + n)
    rng = np.random.default_rng(n)
    classes = rng.integers(0, 3, n).astype(np.int32)
    ex = ExFrames(nms, boxes[None], scores[None], classes[None])
    for opts in (dict(rule="paper", measure="outranking_area", compare="ge", ties="ignore", pixel_offset=1.0, labelled=False),
                 dict(rule="paper", measure="iou", compare="gt", ties="index", pixel_offset=0.0, labelled=True),
                 dict(rule="greedy", measure="outranking_area", compare="ge", ties="ignore", pixel_offset=1.0, labelled=True)):
        want = oracle_ex(oracle, boxes[None], scores[None], classes[None], 0.4, opts)
        got = ex.run(0.4, opts)
        assert np.array_equal(got, want), f"{opts}: {(got != want).sum()} differing keep bits"


def test_variants_batch_walk(nms, oracle):
    """A batch large enough that the greedy rule takes the mask-free walk, with ties ignored."""
    F, n = 40, 3300
    boxes = np.zeros((F, n, 4), np.float32)
    scores = np.zeros((F, n), np.float32)
    for f in range(F):
        boxes[f], scores[f] = frame(n, 5000 + f)
    classes = np.random.default_rng(5).integers(0, 2, (F, n)).astype(np.int32)
    ex = ExFrames(nms, boxes, scores, classes)
    opts = dict(rule="greedy", measure="outranking_area", compare="ge", ties="ignore", pixel_offset=1.0, labelled=True)
    want = oracle_ex(oracle, boxes, scores, classes, 0.5, opts, workers=16)
    got = ex.run(0.5, opts)
    assert np.array_equal(got, want), f"{(got != want).sum()} differing keep bits"
