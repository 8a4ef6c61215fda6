"""The device's division-free pair test, run on the host through the library's
test hook, against plain float32 division (numpy) on adversarial inputs: pairs
whose overlap lies within a few float32 steps of the threshold, on both sides.
No GPU, and nothing from oracle/ (this checks the product's own arithmetic)."""
import numpy as np
import pytest


@pytest.fixture(scope="module")
def nms():
    from paper_2502_00535_amd import build as nms_build

    if nms_build.is_stale():
        nms_build.build_library()
    import paper_2502_00535_amd.binding as binding

    return binding


def plain_decision(v, c, theta):
    """not(overlap < theta) with every operation a separate float32 numpy operation."""
    one, zero = np.float32(1), np.float32(0)
    iw = max(zero, (min(v[2], c[2]) - max(v[0], c[0])) + one)
    ih = max(zero, (min(v[3], c[3]) - max(v[1], c[1])) + one)
    area = ((c[2] - c[0]) + one) * ((c[3] - c[1]) + one)
    q = (iw * ih) / area
    assert isinstance(q, np.float32)
    return int(not (q < theta)), q


def random_pair(rng):
    cx1, cy1 = rng.uniform(0, 3000, 2)
    cw, ch = rng.uniform(1, 400, 2)
    c = np.array([cx1, cy1, cx1 + cw, cy1 + ch], np.float32)
    vx1 = cx1 + rng.uniform(-0.9, 0.9) * cw
    vy1 = cy1 + rng.uniform(-0.9, 0.9) * ch
    vw, vh = rng.uniform(1, 400, 2)
    v = np.array([vx1, vy1, vx1 + vw, vy1 + vh], np.float32)
    return v, c


def steps(x, k):
    x = np.float32(x)
    for _ in range(abs(k)):
        x = np.nextafter(x, np.float32(np.inf if k > 0 else -np.inf), dtype=np.float32)
    return x


def test_threshold_within_a_few_steps_of_the_overlap(nms):
    rng = np.random.default_rng(2024)
    checked = flips = 0
    for _ in range(6000):
        v, c = random_pair(rng)
        _, q = plain_decision(v, c, np.float32(0.5))
        if not (q > 1e-6):
            continue
        for k in (-3, -2, -1, 0, 1, 2, 3):
            theta = steps(q, k)
            want, _ = plain_decision(v, c, theta)
            got = nms.nms_host_pair_test(v, c, float(theta))
            assert got == want, f"v={v.tolist()} c={c.tolist()} theta={theta!r} q={q!r}"
            checked += 1
        flips += 1
    assert checked > 30000 and flips > 4000


def test_fixed_thresholds_random_pairs(nms):
    rng = np.random.default_rng(7)
    thetas = [np.float32(t) for t in (0.5, 0.3, 0.45, 0.7, 0.1, 1.0, 0.999999, 1e-3, 0.33333334)]
    hits = 0
    for i in range(20000):
        v, c = random_pair(rng)
        theta = thetas[i % len(thetas)]
        want, _ = plain_decision(v, c, theta)
        assert nms.nms_host_pair_test(v, c, float(theta)) == want
        hits += want
    assert 500 < hits < 19500


def test_overlap_steered_onto_the_threshold(nms):
    """Victims placed so that the overlap with a W x H box lands within a few
    float32 steps of theta, on both sides (the construction the GPU parity test uses)."""
    rng = np.random.default_rng(99)
    near = hits = 0
    N = 20000
    for i in range(N):
        theta = np.float32([0.5, 0.3, 0.45, 0.7][i % 4])
        W, H = rng.uniform(8, 300, 2)
        c = np.array([0, 0, W - 1, H - 1], np.float32)
        ih = float(theta) * H * (1.0 + rng.integers(-6, 7) * 2.0 ** -24)
        v = np.array([0, H - ih, W - 1, 2 * H], np.float32)
        want, q = plain_decision(v, c, theta)
        assert nms.nms_host_pair_test(v, c, float(theta)) == want, f"v={v.tolist()} c={c.tolist()} theta={theta!r}"
        near += abs(float(q) - float(theta)) <= 4 * float(np.spacing(theta))
        hits += want
    assert near > 0.7 * N and 0.3 * N < hits < 0.7 * N


def test_out_of_range_thresholds_take_the_literal_form(nms):
    rng = np.random.default_rng(5)
    for theta in (0.0, -0.0, -1.0, 1e-20, 2.0 ** -41, 2.0 ** 21, 1e30, float("inf"), -float("inf")):
        for _ in range(300):
            v, c = random_pair(rng)
            want, _ = plain_decision(v, c, np.float32(theta))
            assert nms.nms_host_pair_test(v, c, theta) == want
    assert nms.nms_host_pair_test([0, 0, 1, 1], [0, 0, 1, 1], float("nan")) == nms.NMS_ERR_INVALID_ARG


def test_disjoint_on_both_axes_never_eliminates(nms):
    # both extents negative: their product must not be taken for an overlap
    assert nms.nms_host_pair_test([20, 20, 29, 29], [0, 0, 9, 9], 0.5) == 0
    assert nms.nms_host_pair_test([20, 20, 29, 29], [0, 0, 9, 9], 1e-6) == 0
    assert nms.nms_host_pair_test([0, 20, 9, 29], [0, 0, 9, 9], 1e-6) == 0
    assert nms.nms_host_pair_test([20, 0, 29, 9], [0, 0, 9, 9], 1e-6) == 0
    assert nms.nms_host_pair_test([20, 20, 29, 29], [0, 0, 9, 9], 0.0) == 1  # overlap 0 is not below 0


def test_y_scaled_form_and_its_fallback(nms):
    """The fused kernel evaluates y multiplied by 2^-14 with a clamped add when every y of a
    tile is 0 or within [2^-60, 8190] in magnitude, and the unscaled form otherwise; the
    hook makes the same choice per pair.  Both must agree with plain division at the edges
    of that range: largest extents, negative and zero coordinates, tiny coordinates,
    coordinates just inside and just outside the range."""
    rng = np.random.default_rng(41)

    def check(v, c, theta):
        v = np.asarray(v, np.float32)
        c = np.asarray(c, np.float32)
        want, q = plain_decision(v, c, np.float32(theta))
        assert nms.nms_host_pair_test(v, c, float(theta)) == want, f"v={v.tolist()} c={c.tolist()} theta={theta!r} q={q!r}"
        return want

    hits = 0
    for i in range(6000):
        span = [8190.0, 8191.0, 8250.0, 30000.0][i % 4]      # in range, just outside, outside, far outside
        cy1 = rng.uniform(-span, span * 0.2)
        c = [rng.uniform(-500, 500), cy1, rng.uniform(500, 900), rng.uniform(cy1 + 1, span)]
        vy1 = rng.uniform(-span, span * 0.2)
        v = [rng.uniform(-500, 500), vy1, rng.uniform(500, 900), rng.uniform(vy1 + 1, span)]
        _, q = plain_decision(np.asarray(v, np.float32), np.asarray(c, np.float32), np.float32(0.5))
        for theta in (0.5, q if q > 1e-6 else 0.25, np.nextafter(np.float32(max(q, 1e-6)), np.float32(2))):
            hits += check(v, c, theta)
    assert hits > 2000
    # full-height boxes: the largest extent the scaled form may see, 8190 - (-8190) + 1 = 16381
    check([0, -8190, 99, 8190], [0, -8190, 99, 8190], 0.999)
    check([0, -8190, 99, 8190], [0, -8190, 99, 8190], 1.0)
    check([0, -8190, 99, 8190], [10, -8190, 60, 8190], 0.5)
    check([0, -8191, 99, 8191], [0, -8191, 99, 8191], 1.0)       # just outside: unscaled form
    # zeros, signed zeros and tiny coordinates
    tiny = [2.0 ** -60, 2.0 ** -61, 2.0 ** -100, 1e-40, 0.0, -0.0]
    for a in tiny:
        for b in tiny:
            for theta in (0.5, 1.0, 0.25):
                check([0, a, 9, 9], [0, b, 9, 9], theta)
                check([0, -a, 9, 9 + b], [0, 0, 9, 9], theta)
                check([0, 0, 9, a], [0, 0, 9, b], theta)
    # extents that barely exist: (min - max) + 1 just above zero, in y and in x
    e = np.float32(1) - np.float32(2.0 ** -24)
    for theta in (1e-6, 2.0 ** -30, 0.5):
        check([0, 0, 9, 100], [0, float(100 + e), 9, 200], theta)
        check([0, 0, 100, 9], [float(100 + e), 0, 200, 9], theta)


def test_magnitudes_from_tiny_to_two_to_the_forty(nms):
    """Coordinates scaled by powers of two from 2^-30 to 2^38 in x (areas up to about 2^80):
    the per-box threshold must stay exact wherever its product with the area lands."""
    rng = np.random.default_rng(77)
    hits = checked = 0
    for i in range(12000):
        v, c = random_pair(rng)
        k = int(rng.integers(-30, 39))
        sx = np.float32(2.0 ** k)
        sy = np.float32(2.0 ** int(rng.integers(-20, 2)))       # keep |y| <= 8190 half of the time, beyond it otherwise
        if i % 2:
            sy = np.float32(2.0 ** int(rng.integers(2, 30)))
        v = (v * np.array([sx, sy, sx, sy], np.float32)).astype(np.float32)
        c = (c * np.array([sx, sy, sx, sy], np.float32)).astype(np.float32)
        _, q = plain_decision(v, c, np.float32(0.5))
        for theta in (np.float32(0.5), q, steps(q, 1), steps(q, -1)):
            if not (theta > 0):
                continue
            want, _ = plain_decision(v, c, theta)
            assert nms.nms_host_pair_test(v, c, float(theta)) == want, f"v={v.tolist()} c={c.tolist()} theta={theta!r}"
            checked += 1
            hits += want
    assert checked > 30000 and 5000 < hits < checked - 5000


def test_late_scaled_form_at_the_edge_of_its_range(nms):
    """The form that multiplies the y extent by 2^-14 with a clamp instead of flooring it is taken
    when the outranking box is at most 2^14 high (pixel-inclusive); the hook evaluates it next to
    the plain fast form whenever it applies and reports a disagreement.  Heights on both sides of
    the limit, victims taller and shorter than the outranking box, y far outside the y-scaled
    table's range, extents that barely exist, thresholds at the overlap and its neighbours."""
    rng = np.random.default_rng(314)
    checked = hits = 0
    for i in range(8000):
        height = [16382.0, 16383.0, 16384.0, 16385.0, 12000.0, 40000.0, 3.0][i % 7]   # (y2 - y1); the extent is one more
        cy1 = float(np.float32(rng.uniform(-60000, 60000)))
        c = np.array([rng.uniform(-500, 500), cy1, rng.uniform(500, 900), cy1 + height], np.float32)
        vh = rng.uniform(1, 50000)
        vy1 = cy1 + rng.uniform(-1.0, 1.0) * height
        v = np.array([rng.uniform(-500, 500), vy1, rng.uniform(500, 900), vy1 + vh], np.float32)
        _, q = plain_decision(v, c, np.float32(0.5))
        for theta in (np.float32(0.5), q, steps(q, 1), steps(q, -1)):
            if not (theta >= 2.0 ** -40):
                continue
            want, _ = plain_decision(v, c, theta)
            got = nms.nms_host_pair_test(v, c, float(theta))
            assert got == want, f"v={v.tolist()} c={c.tolist()} theta={theta!r} got {got}"
            checked += 1
            hits += want
    assert checked > 20000 and 2000 < hits < checked - 2000
    # the victim spans the whole outranking box, which is exactly 2^14 high: the scaled extent is exactly 1
    assert nms.nms_host_pair_test([0, -100, 99, 30000], [0, 0, 99, 16383], 1.0) == 1
    assert nms.nms_host_pair_test([0, -100, 99, 30000], [0, 0, 99, 16383], float(np.nextafter(np.float32(1), np.float32(2)))) == 0
    # extents that barely exist or do not
    e = np.float32(1) - np.float32(2.0 ** -24)
    for theta in (2.0 ** -30, 1e-6, 0.5):
        assert nms.nms_host_pair_test([0, 0, 9, 100], [0, float(100 + e), 9, 200], theta) == plain_decision(
            np.array([0, 0, 9, 100], np.float32), np.array([0, float(100 + e), 9, 200], np.float32), np.float32(theta))[0]
        assert nms.nms_host_pair_test([0, 0, 9, 100], [0, 101, 9, 200], theta) == 0
