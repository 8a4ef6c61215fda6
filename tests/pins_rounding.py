"""Pins for the float32 operation order of the overlap measure.

Algorithm 1 writes the measure as a sequence of float operations: the nearer far edge
minus the farther near edge, plus one, floored at zero (per axis), the product of the two
extents, divided by the area of the outranking box, itself (extent + 1) * (extent + 1).
Each is a float32 operation rounded to nearest-even on its own.  On small integers only
the division rounds, so the pins of pins.py cannot tell `(a - b) + 1` from `(a + 1) - b`
or a float32 product from an exact one.  The model below applies the float32 rounding
after every operation, in exact rational arithmetic, and is run on coordinates for which
the subtractions, the additions and the products do round; thresholds are taken from the
quotients the model itself produces, so that a change of one float32 step in any quotient
flips a decision.  Nothing here calls the oracle to obtain an expected value.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np



def R(x: Fraction) -> Fraction:
    """Nearest float32 of a rational (pins.f32_round; imported late because pins.py imports
    this module to extend ALL_PINS)."""
    from pins import f32_round

    return f32_round(x)


def _fr(box):
    return [Fraction(float(v)) for v in box]


def rounded_extent(lo: Fraction, hi: Fraction, offset: Fraction) -> Fraction:
    """(hi - lo) + offset: subtract, round, add, round."""
    return R(R(hi - lo) + offset)


def rounded_area(box, offset=1) -> Fraction:
    b = _fr(box)
    off = Fraction(offset)
    return R(rounded_extent(b[0], b[2], off) * rounded_extent(b[1], b[3], off))


def rounded_measure(bi, bj, measure="outranking_area", offset=1) -> Fraction:
    """Overlap of victim bi with the outranking box bj as a float32 (returned as a
    rational), one rounding per operation in the order of Algorithm 1."""
    i, j = _fr(bi), _fr(bj)
    off = Fraction(offset)
    w = max(Fraction(0), rounded_extent(max(i[0], j[0]), min(i[2], j[2]), off))
    h = max(Fraction(0), rounded_extent(max(i[1], j[1]), min(i[3], j[3]), off))
    inter = R(w * h)
    area_j = rounded_area(bj, offset)
    if measure == "outranking_area":
        return R(inter / area_j)
    union = R(R(rounded_area(bi, offset) + area_j) - inter)
    return R(inter / union)


def as_f32(x: Fraction) -> np.float32:
    v = np.float32(float(x))
    assert Fraction(float(v)) == x
    return v


def outranks(scores, j, i) -> bool:
    sj, si = Fraction(float(scores[j])), Fraction(float(scores[i]))
    return sj > si or (sj == si and j < i)


# --------------------------------------------------------------------------- inputs on which the operations round

KINDS = ("pixel_fractions", "sub_pixel", "mixed_magnitude", "next_to_2_24", "around_zero")


def inexact_frame(seed, n=9):
    """Boxes whose float32 coordinates make the measure's operations inexact, by kind:
    pixel_fractions  24-bit mantissas at pixel scale (products round, some sums round)
    sub_pixel        coordinates below 2 and extents below a pixel: the "+1" rounds every time
    mixed_magnitude  x next to 2^20 (spacing 1/8) against y at sub-pixel scale
    next_to_2_24     integers around 2^24, where x + 1 may not be a float32
    around_zero      fractions of either sign (differences of opposite-sign operands round)"""
    rng = np.random.default_rng(7000 + seed)
    kind = KINDS[seed % len(KINDS)]
    if kind == "pixel_fractions":
        x1, y1 = rng.uniform(0, 40, n), rng.uniform(0, 40, n)
        w, h = rng.uniform(6, 40, n), rng.uniform(6, 40, n)
    elif kind == "sub_pixel":
        x1, y1 = rng.uniform(0, 1.2, n), rng.uniform(0, 1.2, n)
        w, h = rng.uniform(0.05, 0.8, n), rng.uniform(0.05, 0.8, n)
    elif kind == "mixed_magnitude":
        x1, y1 = 2.0 ** 20 + rng.uniform(0, 30, n), rng.uniform(0, 1.2, n)
        w, h = rng.uniform(4, 30, n), rng.uniform(0.05, 0.8, n)
    elif kind == "next_to_2_24":
        x1 = 2.0 ** 24 + rng.integers(-12, 12, n)
        y1 = 2.0 ** 24 + rng.integers(-12, 12, n)
        w, h = rng.integers(1, 9, n), rng.integers(1, 9, n)
    else:
        x1, y1 = rng.uniform(-20, 5, n), rng.uniform(-20, 5, n)
        w, h = rng.uniform(3, 25, n), rng.uniform(3, 25, n)
    boxes = np.stack([x1, y1, x1 + w, y1 + h], axis=1).astype(np.float32)
    # the cast may have merged two edges: keep every box at least one float32 step wide
    boxes[:, 2] = np.maximum(boxes[:, 2], np.nextafter(boxes[:, 0], np.float32(np.inf)))
    boxes[:, 3] = np.maximum(boxes[:, 3], np.nextafter(boxes[:, 1], np.float32(np.inf)))
    scores = (rng.integers(1, 7, n) / np.float32(8)).astype(np.float32)  # ties are frequent
    return kind, boxes, scores


def _decisions(boxes, scores, theta, measure, offset, strict):
    n = len(scores)
    t = Fraction(float(theta))
    elim = [[False] * n for _ in range(n)]
    for i in range(n):
        for j in range(n):
            if i != j and outranks(scores, j, i):
                q = rounded_measure(boxes[i], boxes[j], measure, offset)
                elim[i][j] = q > t if strict else q >= t
    return elim


def _keep_from(elim, scores, greedy):
    n = len(scores)
    rank_order = sorted(range(n), key=lambda t: (-Fraction(float(scores[t])), t))
    keep = [0] * n
    for i in rank_order:
        if greedy:
            keep[i] = 0 if any(elim[i][j] and keep[j] for j in range(n)) else 1
        else:
            keep[i] = 0 if any(elim[i]) else 1
    return keep


def chosen_thresholds(boxes, scores, measure, offset):
    """Thresholds equal to quotients that occur between ranked pairs (lower quartile, median,
    upper quartile of the positive ones below 1) and the float32 just above each."""
    n = len(scores)
    qs = sorted({rounded_measure(boxes[i], boxes[j], measure, offset)
                 for i in range(n) for j in range(n) if i != j and outranks(scores, j, i)})
    qs = [q for q in qs if 0 < q < 1]
    if not qs:
        return [np.float32(0.5)]
    picks = {qs[len(qs) // 4], qs[len(qs) // 2], qs[(3 * len(qs)) // 4]}
    out = []
    for q in sorted(picks):
        v = as_f32(q)
        out += [v, np.nextafter(v, np.float32(np.inf))]
    return out


def pin_rounding_order(oracle, seeds=range(15)):
    for seed in seeds:
        kind, boxes, scores = inexact_frame(seed)
        n = len(scores)
        tag = f"seed {seed} ({kind})"
        # every value of the measure and every area, to the bit
        for i in range(n):
            want_a = as_f32(rounded_area(boxes[i]))
            got_a = oracle.area(boxes[i])
            assert got_a == want_a, f"{tag}: area({i}) = {float(got_a).hex()}, model {float(want_a).hex()}"
            for j in range(n):
                if i == j:
                    continue
                want = as_f32(rounded_measure(boxes[i], boxes[j]))
                got = oracle.overlap(boxes[i], boxes[j])
                assert got == want, f"{tag}: overlap({i}|{j}) = {float(got).hex()}, model {float(want).hex()}"
        # decisions at thresholds that sit on quotients
        for theta in chosen_thresholds(boxes, scores, "outranking_area", 1):
            elim = _decisions(boxes, scores, theta, "outranking_area", 1, False)
            B = oracle.map(boxes, scores, theta)
            for i in range(n):
                for j in range(n):
                    assert B[i, j] == (0 if elim[i][j] else 1), f"{tag}, theta {float(theta).hex()}: B[{i},{j}]"
            want = _keep_from(elim, scores, False)
            assert oracle.keep(boxes, scores, theta).tolist() == want, f"{tag}, theta {float(theta).hex()}: keep"
            assert oracle.reduce(B).tolist() == want, f"{tag}, theta {float(theta).hex()}: reduce(map)"
            want_g = _keep_from(elim, scores, True)
            assert oracle.greedy_keep(boxes, scores, theta).tolist() == want_g, f"{tag}, theta {float(theta).hex()}: greedy"
            # ranked views
            order = oracle.order(scores)
            E = oracle.ranked_eliminations(boxes, order, theta)
            ranked = oracle.ranked_boxes(boxes, order)
            for r in range(n):
                assert ranked[r, 4] == as_f32(rounded_area(boxes[order[r]]))
                for c in range(n):
                    assert E[r, c] == (1 if c < r and elim[order[r]][order[c]] else 0), f"{tag}: E[{r},{c}]"


def pin_rounding_order_variants(oracle, seeds=range(10)):
    """The same for the selectable measure and pixel offset (intersection over union adds
    area_i + area_j, then subtracts the intersection: two more rounded operations)."""
    for seed in seeds:
        kind, boxes, scores = inexact_frame(seed)
        n = len(scores)
        for measure in ("outranking_area", "iou"):
            for offset in (1, 0):
                for strict in (False, True):
                    if measure == "outranking_area" and offset == 1 and not strict:
                        continue  # the default rule: pinned above
                    for theta in chosen_thresholds(boxes, scores, measure, offset)[:4]:
                        elim = _decisions(boxes, scores, theta, measure, offset, strict)
                        for greedy in (False, True):
                            want = _keep_from(elim, scores, greedy)
                            got = oracle.keep_ex(boxes, scores, theta, rule="greedy" if greedy else "paper",
                                                 measure=measure, compare="gt" if strict else "ge",
                                                 pixel_offset=float(offset)).tolist()
                            assert got == want, (f"seed {seed} ({kind}), {measure}, offset {offset}, strict {strict}, "
                                                 f"greedy {greedy}, theta {float(theta).hex()}: {got} != {want}")
                        for i in range(n):
                            for j in range(n):
                                one = oracle.eliminates_ex(boxes, scores, j, i, theta, measure=measure,
                                                           compare="gt" if strict else "ge", pixel_offset=float(offset))
                                assert one == elim[i][j], f"seed {seed} ({kind}): pair ({j} eliminates {i})"


ROUNDING_PINS = [
    ("rounding_order", pin_rounding_order),
    ("rounding_order_variants", pin_rounding_order_variants),
]
