"""HIP library against the CPU oracle on the same seeded inputs, through the C ABI.
Bar: 0 differing bits (keep vector, rank order, box table, every mask word)."""
import numpy as np
import pytest

from gpu_util import DeviceFrames, oracle_keep_frames
from workloads import make_config, random_frame

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nms():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2502_00535_amd.binding as binding

    return binding


def frame_for(n, seed, ties=True):
    if n == 0:
        return np.zeros((0, 4), np.float32), np.zeros(0, np.float32)
    return random_frame(seed, n, extent=1500 if n > 600 else 300, max_side=90,
                        integer=(seed % 2 == 0), score_levels=(max(3, n // 4) if ties else 0))


SIZES = [1, 2, 63, 64, 65, 127, 128, 129, 200, 1000, 1024, 1025, 2048, 4095, 4096]


@pytest.mark.parametrize("n", SIZES)
def test_steps_single_frame(nms, oracle, n):
    """rank, map and reduce checked one by one: order, box table, every mask word, keep."""
    print(f"case n={n}", flush=True)
    boxes, scores = frame_for(n, seed=n)
    theta = np.float32([0.5, 0.3, 0.45][n % 3])
    dev = DeviceFrames(nms, boxes[None], scores[None])
    keep = dev.steps(float(theta))[0]

    order = oracle.order(scores)
    assert np.array_equal(dev.host_order()[0, :n], order)
    ranked = oracle.ranked_boxes(boxes, order)
    n_pad = dev.n_pad
    s5 = dev.host_sorted5()[0]
    assert np.array_equal(s5[:4 * n_pad].reshape(n_pad, 4)[:n], ranked[:, :4])
    assert np.array_equal(s5[4 * n_pad:4 * n_pad + n], ranked[:, 4])
    assert np.all(s5[:4 * n_pad].reshape(n_pad, 4)[n:] == 0) and np.all(s5[4 * n_pad + n:] == 1)

    words = oracle.ranked_elimination_words(boxes, order, theta)        # [n, W]
    W = n_pad // 64
    got = dev.host_mask()[0].reshape(W, n_pad)
    for w in range(W):
        lo = 64 * w                                                        # rows r >= 64w own word w
        assert np.array_equal(got[w, lo:n], words[lo:, w]), f"mask word column {w}"
        assert np.all(got[w, n:n_pad] == 0)
    assert np.array_equal(keep[:n], oracle.keep(boxes, scores, theta))


@pytest.mark.parametrize("n", [1, 64, 65, 1000, 4096, 4097, 5000, 8192, 8193, 16384, 20000])
def test_fused_single_frame(nms, oracle, n):
    print(f"case n={n}", flush=True)
    boxes, scores = frame_for(n, seed=1000 + n)
    theta = np.float32(0.4)
    dev = DeviceFrames(nms, boxes[None], scores[None])
    dev.fused(float(theta), want=oracle.keep(boxes, scores, theta)[None])
    if n > 4096:  # several rank chunks: check the merged order as well
        dev.steps(float(theta))
        assert np.array_equal(dev.host_order()[0], oracle.order(scores))


@pytest.mark.parametrize("theta", [0.0, -1.0, 1.0, 1.0000001, 2.0, 1e-30, 2.0 ** -40, 2.0 ** -41, 0.99999994,
                                   0.33333334, 0.1, 1e30, float("inf"), float("-inf")])
def test_threshold_range(nms, oracle, theta):
    """Thresholds outside the fast form's range take the literal division kernel;
    closed forms: theta <= 0 keeps the top rank only, theta > 1 keeps everything."""
    print(f"case theta={theta}", flush=True)
    boxes, scores = frame_for(700, seed=31)
    dev = DeviceFrames(nms, boxes[None], scores[None])
    want = oracle.keep(boxes, scores, np.float32(theta))
    dev.fused(theta, want=want[None])
    assert np.array_equal(dev.steps(theta)[0], want)
    if theta <= 0:
        assert want.sum() == 1
    if theta > 1:
        assert want.sum() == 700


def test_batched_ragged_counts(nms, oracle):
    """Frames of different lengths (including empty and full) in one call; slots
    beyond a frame's count come back 0."""
    rng = np.random.default_rng(12)
    n_max, F = 333, 40
    counts = rng.integers(0, n_max + 1, F).astype(np.int32)
    counts[:6] = [0, 1, 64, 65, n_max, n_max - 1]
    boxes = np.zeros((F, n_max, 4), np.float32)
    scores = np.zeros((F, n_max), np.float32)
    for f in range(F):
        b, s = frame_for(n_max, seed=500 + f)
        boxes[f], scores[f] = b, s
    theta = np.float32(0.45)
    want = oracle_keep_frames(oracle, boxes, scores, theta, counts)
    dev = DeviceFrames(nms, boxes, scores, counts)
    dev.fused(float(theta), want=want)
    assert np.array_equal(dev.steps(float(theta)), want)
    # negative and oversized counts are clamped
    counts2 = counts.copy()
    counts2[0], counts2[1] = -5, n_max + 100
    want2 = oracle_keep_frames(oracle, boxes, scores, theta, np.clip(counts2, 0, n_max))
    dev2 = DeviceFrames(nms, boxes, scores, counts2)
    dev2.fused(float(theta), want=want2)
    assert np.array_equal(dev2.steps(float(theta)), want2)


def test_batched_ragged_counts_many_frames(nms, oracle):
    """Enough frames that the map step packs four tiles into a wavefront: ragged
    counts, a tile-row count (11) that is not a multiple of four, both map kernels."""
    rng = np.random.default_rng(21)
    n_max, F = 700, 720
    counts = rng.integers(0, n_max + 1, F).astype(np.int32)
    counts[:8] = [0, 1, 63, 64, 65, 256, 257, n_max]
    boxes = np.zeros((F, n_max, 4), np.float32)
    scores = np.zeros((F, n_max), np.float32)
    for f in range(F):
        boxes[f], scores[f] = frame_for(n_max, seed=3000 + f)
    theta = np.float32(0.35)
    want = oracle_keep_frames(oracle, boxes, scores, theta, counts)
    dev = DeviceFrames(nms, boxes, scores, counts)
    dev.fused(float(theta), want=want)
    assert np.array_equal(dev.steps(float(theta)), want)
    # every mask word of three frames against the oracle's ranked view
    n_pad, W = dev.n_pad, dev.n_pad // 64
    masks = dev.host_mask()
    orders = dev.host_order()
    for f in (5, 7, 100):
        n = int(counts[f])
        order = oracle.order(scores[f, :n])
        assert np.array_equal(orders[f, :n], order)
        words = oracle.ranked_elimination_words(boxes[f, :n], order, theta)
        got = masks[f].reshape(W, n_pad)
        for w in range((n + 63) // 64):
            assert np.array_equal(got[w, 64 * w:n], words[64 * w:, w]), f"frame {f}, mask word column {w}"


def test_y_ranges_for_the_scaled_form(nms, oracle):
    """The ranked route evaluates tiles whose y coordinates are all 0 or within
    [2^-60, 8190] in magnitude with y scaled by 2^-14, other tiles unscaled.  Frames that
    mix both kinds of tile (decided per 64 ranks), negative coordinates, boxes as tall as
    the range allows, tiny and zero coordinates."""
    rng = np.random.default_rng(8)
    n = 1500
    frames = []
    for kind in range(6):
        x1 = rng.uniform(-300, 300, n)
        w = rng.uniform(1, 250, n)
        if kind == 0:    # all regular, negative and positive y
            y1 = rng.uniform(-8190, 8000, n); h = rng.uniform(1, 180, n)
        elif kind == 1:  # a tenth of the boxes out of range, scattered over the ranks
            y1 = rng.uniform(-3000, 3000, n); h = rng.uniform(1, 400, n)
            far = rng.random(n) < 0.1
            y1[far] += 9000.0
        elif kind == 2:  # tall boxes up to the full range
            y1 = rng.uniform(-8190, -4000, n); h = rng.uniform(4000, 16000, n)
        elif kind == 3:  # tiny and zero y1 (some below 2^-60: irregular)
            y1 = rng.choice([0.0, -0.0, 2.0 ** -60, 2.0 ** -61, 1e-30, 1e-40, 3.0], n); h = rng.uniform(1, 50, n)
        elif kind == 4:  # far out of range everywhere
            y1 = rng.uniform(1e5, 2e5, n); h = rng.uniform(1, 3000, n)
        else:            # exactly at the limits
            y1 = rng.choice([-8190.0, -8191.0, 0.0, 8000.0], n); h = rng.choice([190.0, 191.0, 16380.0], n)
        y2 = np.minimum(y1 + h, np.where(kind in (1, 4), 1e9, 8190.0 if kind != 5 else 8191.0))
        b = np.stack([x1, y1, x1 + w, np.maximum(y2, y1)], axis=1).astype(np.float32)
        b[:, 3] = np.maximum(b[:, 3], b[:, 1])
        s = rng.uniform(0.01, 1.0, n).astype(np.float32)
        frames.append((b, s))
    boxes = np.stack([f[0] for f in frames])
    scores = np.stack([f[1] for f in frames])
    for theta in (0.5, 0.05):
        want = oracle_keep_frames(oracle, boxes, scores, np.float32(theta))
        assert all(0 < want[f].sum() < n for f in range(len(frames)))
        dev = DeviceFrames(nms, boxes, scores)
        dev.fused(theta, want=want)
        assert np.array_equal(dev.steps(theta), want)
    # many frames: the four-tiles-per-wavefront kernel with mixed tiles
    many_b = np.concatenate([boxes[:, :640]] * 134)
    many_s = np.concatenate([scores[:, :640]] * 134)
    want = oracle_keep_frames(oracle, many_b, many_s, np.float32(0.3))
    DeviceFrames(nms, many_b, many_s).fused(0.3, want=want)
    # a large frame (several rank chunks: the merge kernel sets the tile flags)
    big_b = np.concatenate([boxes[0], boxes[1], boxes[3], boxes[5]] * 2)[None]
    big_s = rng.uniform(0.01, 1.0, big_b.shape[1]).astype(np.float32)[None]
    want = oracle_keep_frames(oracle, big_b, big_s, np.float32(0.4))
    DeviceFrames(nms, big_b, big_s).fused(0.4, want=want)


def test_wide_range_of_magnitudes(nms, oracle):
    """Frames whose coordinates are scaled by powers of two between 2^-20 and 2^36 (x and y
    independently; areas up to about 2^80, y both inside and far outside the range of the scaled
    form), negative offsets included: every route against the oracle."""
    rng = np.random.default_rng(19)
    n, F = 900, 12
    boxes = np.zeros((F, n, 4), np.float32)
    scores = np.zeros((F, n), np.float32)
    for f in range(F):
        b, s = random_frame(600 + f, n, extent=400, max_side=120, integer=(f % 3 == 0), score_levels=100)
        sx = np.float32(2.0 ** int(rng.integers(-20, 37)))
        sy = np.float32(2.0 ** int(rng.integers(-20, 37)))
        shift = np.float32(-200.0 if f % 2 else 0.0)
        boxes[f] = ((b + shift) * np.array([sx, sy, sx, sy], np.float32)).astype(np.float32)
        scores[f] = s
    for theta in (0.5, 0.05, 0.9):
        want = oracle_keep_frames(oracle, boxes, scores, np.float32(theta))
        dev = DeviceFrames(nms, boxes, scores)
        dev.fused(theta, want=want)
        assert np.array_equal(dev.steps(theta), want)
    assert 0 < want.sum() < want.size


def steered_pairs(F, theta, seed):
    """F two-box frames whose overlap lands within a few float32 steps of theta: a
    W x H box at the origin and a victim of the same width whose top edge is placed
    so that the shared height is theta * H, up to a perturbation of a few 2^-24."""
    rng = np.random.default_rng(seed)
    boxes = np.zeros((F, 2, 4), np.float32)
    scores = np.tile(np.array([0.9, 0.8], np.float32), (F, 1))
    W = rng.uniform(8, 300, F)
    H = rng.uniform(8, 300, F)
    ih = float(theta) * H * (1.0 + rng.integers(-6, 7, F) * 2.0 ** -24)
    z = np.zeros(F)
    boxes[:, 0] = np.stack([z, z, W - 1, H - 1], axis=1)
    boxes[:, 1] = np.stack([z, H - ih, W - 1, 2 * H], axis=1)
    swap = rng.integers(0, 2, F).astype(bool)  # the outranking box is not always index 0
    boxes[swap] = boxes[swap][:, ::-1]
    scores[swap] = scores[swap][:, ::-1]
    return boxes, np.ascontiguousarray(scores)


@pytest.mark.parametrize("theta", [0.5, 0.3, 0.45, 0.7])
def test_overlap_within_steps_of_threshold(nms, oracle, theta):
    """60000 pairs per threshold whose overlap straddles theta by a few float32
    steps: the division-free device test must decide like the oracle's division."""
    print(f"case theta={theta}", flush=True)
    F = 60000
    boxes, scores = steered_pairs(F, theta, seed=int(theta * 1000))
    want = oracle_keep_frames(oracle, boxes, scores, np.float32(theta))
    assert 0.3 * F < (want.sum() - F) < 0.7 * F  # both outcomes are common
    t32 = float(np.float32(theta))
    sample = range(0, F, 30)
    near = sum(abs(float(oracle.overlap(boxes[f, 1 - int(np.argmax(scores[f]))], boxes[f, int(np.argmax(scores[f]))])) - t32)
               <= 4 * float(np.spacing(np.float32(theta))) for f in sample)
    assert near > 0.6 * len(sample)  # and the overlaps really sit within a few steps of theta
    dev = DeviceFrames(nms, boxes, scores)
    dev.fused(theta, want=want)
    assert np.array_equal(dev.steps(theta), want)


def test_threshold_equal_to_observed_overlaps(nms, oracle):
    """Thresholds set to overlaps that occur in the frame, and their float32
    neighbours: equality must eliminate, one step above must not."""
    w = make_config(0)
    boxes, scores = w.boxes[0], w.scores[0]
    order = oracle.order(scores)
    dev = DeviceFrames(nms, boxes[None], scores[None])
    rng = np.random.default_rng(3)
    tried = 0
    while tried < 12:
        r = int(rng.integers(1, 1024))
        c = int(rng.integers(0, r))
        q = oracle.overlap(boxes[order[r]], boxes[order[c]])
        if not (0.05 < q < 0.95):
            continue
        tried += 1
        for theta in (q, np.nextafter(q, np.float32(2)), np.nextafter(q, np.float32(0))):
            dev.fused(float(theta), want=oracle.keep(boxes, scores, theta)[None])


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_configs_full_size(nms, oracle, index):
    """The five benchmark configurations at full size, fused path (what bench.py
    times) and the three-step path; every keep bit against the oracle."""
    print(f"case config {index}", flush=True)
    w = make_config(index)
    want = oracle_keep_frames(oracle, w.boxes, w.scores, np.float32(w.theta))
    dev = DeviceFrames(nms, w.boxes, w.scores)
    dev.fused(w.theta, want=want)  # automatic, ranked and (where bounded) direct route
    got = dev.steps(w.theta)
    assert np.array_equal(got, want), f"{w.name}: {(got != want).sum()} differing keep bits (steps)"
    assert 0 < want.sum() < want.size


def test_largest_frame(nms, oracle):
    """n = NMS_MAX_N = 65536: sixty-four rank chunks merged in four batches, a 512 MiB mask, sixteen
    blocks of the greedy sweep, sixteen shares of the early-exit route; both rules, every keep bit.  (The two oracle runs take about half a minute; they run
    side by side on two host threads.)"""
    from concurrent.futures import ThreadPoolExecutor

    n = 65536
    boxes, scores = random_frame(65536, n, extent=6000, max_side=100, integer=False, score_levels=20000)
    theta = np.float32(0.4)
    print("case n=65536: oracle running", flush=True)
    with ThreadPoolExecutor(max_workers=2) as pool:
        fut = pool.submit(oracle.keep, boxes, scores, theta)
        fut_g = pool.submit(oracle.greedy_keep, boxes, scores, theta)
        want, want_g = fut.result(), fut_g.result()
    print("case n=65536: GPU running", flush=True)
    dev = DeviceFrames(nms, boxes[None], scores[None])
    dev.fused(float(theta), want=want[None])   # automatic, ranked and early-exit route (the direct one is skipped: 4.3 G pair slots)
    assert np.array_equal(dev.steps(float(theta))[0], want)
    via_steps, one_call = dev.greedy(float(theta))
    assert np.array_equal(via_steps[0], want_g) and np.array_equal(one_call[0], want_g)
    assert 0 < want.sum() < want_g.sum() < n


def test_deterministic_and_inputs_untouched(nms):
    w = make_config(2)
    dev = DeviceFrames(nms, w.boxes, w.scores)
    first = dev.fused(w.theta).copy()
    for _ in range(3):
        assert np.array_equal(dev.fused(w.theta), first)
    assert np.array_equal(dev.boxes.cpu().numpy(), w.boxes)
    assert np.array_equal(dev.scores.cpu().numpy(), w.scores)


def test_pool_entry_point_and_side_stream(nms, oracle):
    import torch

    w = make_config(0)
    boxes, scores = w.boxes[0], w.scores[0]
    want = oracle.keep(boxes, scores, np.float32(w.theta))
    dev = DeviceFrames(nms, boxes[None], scores[None])
    pool = torch.zeros(nms.nms_workspace_bytes(2048, 1), dtype=torch.uint8, device="cuda:0")
    nms.nms_init(2048, 1, pool)
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            dev.keep.fill_(9)
            nms.nms_run(dev.boxes, dev.scores, 1024, w.theta, dev.keep)
        side.synchronize()
        assert np.array_equal(dev.keep.cpu().numpy()[0], want)
        big = DeviceFrames(nms, np.zeros((1, 4096, 4), np.float32), np.zeros((1, 4096), np.float32))
        with pytest.raises(nms.NmsError) as err:  # more boxes than the pool was registered for
            nms.nms_run(big.boxes, big.scores, 4096, w.theta, big.keep)
        assert err.value.status == nms.NMS_ERR_WORKSPACE
        with pytest.raises(ValueError):           # and the binding refuses tensors smaller than n says
            nms.nms_run(dev.boxes, dev.scores, 4096, w.theta, dev.keep)
    finally:
        nms.nms_shutdown()
    with pytest.raises(nms.NmsError):
        nms.nms_run(dev.boxes, dev.scores, 1024, w.theta, dev.keep)
    # single-frame wrappers of the step calls
    order = torch.empty(1024, dtype=torch.int32, device="cuda:0")
    s5 = torch.empty(5 * 1024, dtype=torch.float32, device="cuda:0")
    mask = torch.empty(nms.nms_mask_words(1024), dtype=torch.int64, device="cuda:0")
    keep = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    nms.nms_sort(dev.boxes, dev.scores, 1024, order, s5)
    nms.nms_overlap_mask(s5, 1024, w.theta, mask)
    nms.nms_reduce(mask, order, 1024, keep)
    ws = torch.zeros(nms.nms_workspace_bytes(1024, 1), dtype=torch.uint8, device="cuda:0")
    keep2 = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    nms.nms_run_ws(dev.boxes, dev.scores, 1024, w.theta, keep2, ws)
    torch.cuda.synchronize()
    assert np.array_equal(keep.cpu().numpy(), want) and np.array_equal(keep2.cpu().numpy(), want)
    # arguments marshalled once, called repeatedly
    keep3 = torch.zeros(1024, dtype=torch.uint8, device="cuda:0")
    plan = nms.RunPlan(dev.boxes, dev.scores, None, 1024, 1, w.theta, keep3, ws)
    for _ in range(3):
        keep3.fill_(5)
        plan()
        torch.cuda.synchronize()
        assert np.array_equal(keep3.cpu().numpy(), want)


def test_calls_can_be_captured_in_a_hip_graph(nms, oracle):
    """The entry points only enqueue kernels on the caller's stream (no allocation, no
    synchronisation, no memset), so a caller may capture them in a HIP graph.  The graph is
    replayed several times with new inputs written into the same buffers and eager work in
    between; every replay must give what the oracle gives for the inputs of that replay."""
    import torch

    n, F = 700, 12
    frames = [random_frame(4300 + f, n, extent=300, max_side=90, integer=(f % 2 == 0), score_levels=50) for f in range(3 * F)]
    dev = torch.device("cuda:0")
    boxes = torch.zeros((F, n, 4), dtype=torch.float32, device=dev)
    scores = torch.zeros((F, n), dtype=torch.float32, device=dev)
    keep = torch.zeros((F, n), dtype=torch.uint8, device=dev)
    keep_g = torch.zeros((F, n), dtype=torch.uint8, device=dev)
    keep_x = torch.zeros((F, n), dtype=torch.uint8, device=dev)
    keep_e = torch.zeros((F, n), dtype=torch.uint8, device=dev)
    ws_e = torch.zeros(nms.nms_workspace_bytes(n, F), dtype=torch.uint8, device=dev)
    ws = torch.zeros(nms.nms_workspace_bytes(n, F), dtype=torch.uint8, device=dev)
    ws_g = torch.zeros(nms.nms_greedy_workspace_bytes(n, F), dtype=torch.uint8, device=dev)
    ws_x = torch.zeros(nms.nms_ex_workspace_bytes(n, F), dtype=torch.uint8, device=dev)
    theta = 0.4

    def enqueue():
        nms.nms_run_ranked_batched(boxes, scores, None, n, F, theta, keep, ws)
        nms.nms_run_greedy_batched(boxes, scores, None, n, F, theta, keep_g, ws_g)
        nms.nms_run_ex_batched(boxes, scores, None, n, F, theta, keep_x, ws_x, rule="greedy", measure="iou", pixel_offset=0.0)
        nms.nms_run_early_exit_batched(boxes, scores, None, n, F, theta, keep_e, ws_e)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        enqueue()  # warm-up outside the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    for rep in range(3):
        b = np.stack([frames[rep * F + f][0] for f in range(F)])
        s = np.stack([frames[rep * F + f][1] for f in range(F)])
        boxes.copy_(torch.from_numpy(b))
        scores.copy_(torch.from_numpy(s))
        keep.fill_(9), keep_g.fill_(9), keep_x.fill_(9), keep_e.fill_(9)
        (boxes.sum() + scores.sum()).item()  # eager work and a synchronisation between replays
        graph.replay()
        torch.cuda.synchronize()
        want = oracle_keep_frames(oracle, b, s, np.float32(theta))
        want_g = oracle_keep_frames(oracle, b, s, np.float32(theta), rule="greedy")
        want_x = np.stack([oracle.keep_ex(b[f], s[f], np.float32(theta), rule="greedy", measure="iou", pixel_offset=0.0)
                           for f in range(F)])
        assert np.array_equal(keep.cpu().numpy(), want), f"replay {rep}: paper rule"
        assert np.array_equal(keep_e.cpu().numpy(), want), f"replay {rep}: paper rule, early-exit route"
        assert np.array_equal(keep_g.cpu().numpy(), want_g), f"replay {rep}: greedy rule"
        assert np.array_equal(keep_x.cpu().numpy(), want_x), f"replay {rep}: variants"
