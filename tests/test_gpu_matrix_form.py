"""The paper's own data layout on the GPU (byte matrix B over the unsorted input,
Algorithm 2's k-partition reduce) against the oracle's map / reduce, byte for byte."""
import numpy as np
import pytest

from workloads import make_config, random_frame

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nms():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2502_00535_amd.binding as binding

    return binding


def run_matrix_form(nms, boxes, scores, n, capacity, theta, ks):
    import torch

    dev = torch.device("cuda:0")
    d_boxes = torch.from_numpy(np.ascontiguousarray(boxes, np.float32)).to(dev) if n else None
    d_scores = torch.from_numpy(np.ascontiguousarray(scores, np.float32)).to(dev) if n else None
    B = torch.full((capacity, capacity), 7, dtype=torch.uint8, device=dev)
    nms.nms_map_matrix(d_boxes, d_scores, n, capacity, theta, B)
    out = {}
    for k in ks:
        V = torch.full((capacity,), 9, dtype=torch.uint8, device=dev)
        nms.nms_reduce_matrix(B, capacity, k, V)
        out[k] = V
    torch.cuda.synchronize()
    return B.cpu().numpy(), {k: v.cpu().numpy() for k, v in out.items()}


def expected(oracle, boxes, scores, n, capacity, theta):
    B = np.ones((capacity, capacity), np.uint8)
    if n:
        B[:n, :n] = oracle.map(boxes, scores, np.float32(theta))
    return B, oracle.reduce(B)


@pytest.mark.parametrize("n,capacity", [(0, 64), (1, 64), (63, 64), (64, 64), (65, 128), (200, 256), (257, 320),
                                        (1000, 1024), (1027, 4096), (2895, 4096)])
def test_matrix_and_partitioned_reduce(nms, oracle, n, capacity):
    print(f"case n={n} capacity={capacity}", flush=True)
    if n:
        boxes, scores = random_frame(700 + n, n, extent=900, max_side=120, integer=(n % 2 == 0),
                                     score_levels=max(3, n // 4))
    else:
        boxes, scores = np.zeros((0, 4), np.float32), np.zeros(0, np.float32)
    theta = float(np.float32([0.5, 0.3, 0.45][n % 3]))
    ks = [k for k in (1, 2, 4, 8, 16, 32, 64, capacity) if capacity % k == 0 and capacity // k <= 1024]
    B, V = run_matrix_form(nms, boxes, scores, n, capacity, theta, ks)
    want_B, want_V = expected(oracle, boxes, scores, n, capacity, theta)
    assert np.array_equal(B, want_B), f"{(B != want_B).sum()} differing matrix bytes"
    for k in ks:
        assert np.array_equal(V[k], want_V), f"k={k}: {(V[k] != want_V).sum()} differing V bytes"
    # V restricted to the real boxes is the keep vector of the whole path
    if n:
        assert np.array_equal(want_V[:n], oracle.keep(boxes, scores, np.float32(theta)))
        assert np.all(want_V[n:] == 1)


@pytest.mark.parametrize("theta", [0.0, 1.5, 2.0 ** -41])
def test_matrix_form_literal_division_kernel(nms, oracle, theta):
    """Thresholds outside the range of the division-free test."""
    boxes, scores = random_frame(77, 300, extent=300, max_side=90, integer=True, score_levels=40)
    B, V = run_matrix_form(nms, boxes, scores, 300, 320, theta, [5, 64])
    want_B, want_V = expected(oracle, boxes, scores, 300, 320, theta)
    assert np.array_equal(B, want_B)
    assert np.array_equal(V[5], want_V) and np.array_equal(V[64], want_V)


def test_matrix_form_config1_full_size(nms, oracle):
    """Configuration 1 (one 4K frame, 4096 boxes) at the paper's capacity D_max = 4096, k = 32."""
    w = make_config(1)
    boxes, scores = w.boxes[0], w.scores[0]
    B, V = run_matrix_form(nms, boxes, scores, w.n, 4096, w.theta, [4, 32])
    want_B, want_V = expected(oracle, boxes, scores, w.n, 4096, w.theta)
    assert np.array_equal(B, want_B)
    assert np.array_equal(V[4], want_V) and np.array_equal(V[32], want_V)
