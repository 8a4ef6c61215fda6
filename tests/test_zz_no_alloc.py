"""nms_run_static_batched (scratch in a static device array inside the library, no
allocation) against nms_run_batched, the entry point it is a variant of: same keep bytes,
bit for bit, on two calls in a row of which the second is smaller, so that the array still
holds the first call's tables when the second starts.  The oracle is run beside both.
"""
import numpy as np
import pytest

from gpu_util import oracle_keep_frames
from workloads import make_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nms():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2502_00535_amd.binding as binding

    return binding


def _both(nms, boxes, scores, counts, theta):
    """keep bytes of (existing entry point, static-scratch entry point) for one batch."""
    import torch

    dev = torch.device("cuda:0")
    F, n_max = scores.shape
    d_boxes = torch.from_numpy(np.ascontiguousarray(boxes, np.float32)).to(dev)
    d_scores = torch.from_numpy(np.ascontiguousarray(scores, np.float32)).to(dev)
    d_counts = None if counts is None else torch.from_numpy(np.ascontiguousarray(counts, np.int32)).to(dev)
    ws = torch.empty(nms.nms_workspace_bytes(n_max, F), dtype=torch.uint8, device=dev)
    assert ws.numel() <= nms.NMS_STATIC_SCRATCH_BYTES
    keep_ws = torch.full((F, n_max), 77, dtype=torch.uint8, device=dev)
    keep_static = torch.full((F, n_max), 77, dtype=torch.uint8, device=dev)
    nms.nms_run_batched(d_boxes, d_scores, d_counts, n_max, F, theta, keep_ws, ws)
    before = torch.cuda.memory_allocated()
    nms.nms_run_static_batched(d_boxes, d_scores, d_counts, n_max, F, theta, keep_static)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return keep_ws.cpu().numpy(), keep_static.cpu().numpy()


def _ragged(cfg, frames, n_max, seed):
    w = make_config(cfg, frames=frames)
    rng = np.random.default_rng(seed)
    counts = rng.integers(n_max // 2, n_max + 1, frames).astype(np.int32)
    counts[0] = n_max
    return w.boxes[:, :n_max], w.scores[:, :n_max], counts, w.theta


def test_batch_then_smaller_batch(nms, oracle):
    # 64 x 1024 (ranked route: the rank step's tables go through the array), then 40 ragged
    # frames of at most 1000 boxes on top of what the first call left there
    big = make_config(2)
    first_ws, first_static = _both(nms, big.boxes, big.scores, None, big.theta)
    boxes, scores, counts, theta = _ragged(2, 40, 1000, 5)
    second_ws, second_static = _both(nms, boxes, scores, counts, theta)
    assert np.array_equal(first_static, first_ws), f"{(first_static != first_ws).sum()} differing keep bytes (first call)"
    assert np.array_equal(second_static, second_ws), f"{(second_static != second_ws).sum()} differing keep bytes (second call)"
    assert np.array_equal(first_static, oracle_keep_frames(oracle, big.boxes, big.scores, np.float32(big.theta)))
    assert np.array_equal(second_static, oracle_keep_frames(oracle, boxes, scores, np.float32(theta), counts))


def test_large_frame_then_smaller_frame(nms, oracle):
    # 16,384 boxes (several rank chunks: chunk keys, merge, y-scaled table, tile flags all in the
    # array), then 6000 boxes of the same picture with another threshold
    w = make_config(3)
    first_ws, first_static = _both(nms, w.boxes, w.scores, None, w.theta)
    boxes, scores = w.boxes[:, :6000], w.scores[:, :6000]
    second_ws, second_static = _both(nms, boxes, scores, None, 0.45)
    assert np.array_equal(first_static, first_ws)
    assert np.array_equal(second_static, second_ws)
    assert np.array_equal(second_static, oracle_keep_frames(oracle, boxes, scores, np.float32(0.45)))
    assert np.array_equal(first_static, oracle_keep_frames(oracle, w.boxes, w.scores, np.float32(w.theta)))


def test_limit_and_arguments(nms):
    import torch

    dev = torch.device("cuda:0")
    n_max, F = 4096, 24  # 24 frames of 4096 boxes need more than the array holds
    assert nms.nms_workspace_bytes(n_max, F) > nms.NMS_STATIC_SCRATCH_BYTES
    boxes = torch.zeros((F, n_max, 4), dtype=torch.float32, device=dev)
    scores = torch.zeros((F, n_max), dtype=torch.float32, device=dev)
    keep = torch.full((F, n_max), 77, dtype=torch.uint8, device=dev)
    with pytest.raises(nms.NmsError) as err:
        nms.nms_run_static_batched(boxes, scores, None, n_max, F, 0.5, keep)
    assert err.value.status == nms.NMS_ERR_TOO_LARGE
    with pytest.raises(nms.NmsError) as err:
        nms.nms_run_static_batched(boxes, scores, None, n_max, 1, float("nan"), keep)
    assert err.value.status == nms.NMS_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert int(keep.min()) == 77  # nothing was enqueued
    # an empty batch is fine and touches nothing
    nms.nms_run_static_batched(boxes, scores, None, 0, 1, 0.5, keep)
    nms.nms_run_static_batched(boxes, scores, None, n_max, 23, 0.5, keep)  # the largest 4096-box batch that fits
    torch.cuda.synchronize()
    assert int(keep[:23].max()) <= 1
