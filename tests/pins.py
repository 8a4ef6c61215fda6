"""Pins for the CPU oracle: checks whose expected values come from the paper's
definitions and from mathematics, never from the oracle itself.

Each pin is a function ``pin(oracle)`` that raises AssertionError when the
oracle disagrees.  ``ALL_PINS`` is run against the real oracle (all must pass)
and against deliberately broken copies of it (each must fail at least one pin),
see test_oracle_pins.py and test_oracle_mutants.py.

Contents
  * hand-worked examples (tests/golden/*.txt)
  * an independent exact evaluation in rational arithmetic of the rule on tiny
    frames, with exhaustive search over all survivor sets (n <= 8)
  * closed forms: empty frame, one box, disjoint boxes, theta <= 0, theta > 1,
    staircase chain of any length, disjoint clusters of identical boxes
  * the paper's own square-box statement (strict guard, fixed capacity, k partitions) against the per-axis form
"""
from __future__ import annotations

import glob
import itertools
import os
from fractions import Fraction

import numpy as np

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# --------------------------------------------------------------------------- golden files

def parse_golden(path):
    case = {"boxes": [], "scores": [], "overlaps": [], "overlaps_f32": [], "areas_f32": [], "keep": None,
            "greedy": None, "literal_keep": None, "theta": None, "path": path}
    with open(path) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            tok = line.split()
            if tok[0] == "theta":
                t = np.float32(tok[1])
                if len(tok) > 2:
                    assert tok[2] == "next_up"
                    t = np.nextafter(t, np.float32(np.inf), dtype=np.float32)
                case["theta"] = t
            elif tok[0] == "box":
                case["boxes"].append([float(v) for v in tok[1:5]])
                case["scores"].append(float(tok[5]))
                assert np.float32(case["boxes"][-1]).astype(np.float64).tolist() == case["boxes"][-1], \
                    f"{path}: a coordinate is not a float32"
            elif tok[0] == "overlap":
                p, q = tok[3].split("/")
                case["overlaps"].append((int(tok[1]), int(tok[2]), int(p), int(q)))
            elif tok[0] == "overlap_f32":
                # the float32 the measure must come out as, written as a C99 hexadecimal literal
                value = float.fromhex(tok[3])
                assert float(np.float32(value)) == value, f"{path}: {tok[3]} is not a float32"
                case["overlaps_f32"].append((int(tok[1]), int(tok[2]), np.float32(value)))
            elif tok[0] == "area_f32":
                value = float.fromhex(tok[2])
                assert float(np.float32(value)) == value, f"{path}: {tok[2]} is not a float32"
                case["areas_f32"].append((int(tok[1]), np.float32(value)))
            elif tok[0] in ("keep", "greedy", "literal_keep"):
                case[tok[0]] = np.array([int(v) for v in tok[1:]], dtype=np.uint8)
            else:
                raise ValueError(f"{path}: unknown directive {tok[0]}")
    case["boxes"] = np.array(case["boxes"], dtype=np.float32).reshape(-1, 4)
    case["scores"] = np.array(case["scores"], dtype=np.float32)
    return case


def golden_cases():
    paths = sorted(glob.glob(os.path.join(GOLDEN_DIR, "*.txt")))
    assert len(paths) >= 12, "golden fixtures missing"
    return [parse_golden(p) for p in paths]


def pin_golden(oracle):
    for case in golden_cases():
        name = os.path.basename(case["path"])
        b, s, th = case["boxes"], case["scores"], case["theta"]
        for (i, j, p, q) in case["overlaps"]:
            got = oracle.overlap(b[i], b[j])
            want = np.float32(p) / np.float32(q)  # p, q small integers: one correctly rounded division
            assert got == want, f"{name}: overlap({i}|{j}) = {got}, hand value {p}/{q}"
            assert oracle.outranks(s, j, i), f"{name}: {j} should outrank {i}"
            assert not oracle.outranks(s, i, j), f"{name}: {i} should not outrank {j}"
        for (i, j, want) in case["overlaps_f32"]:
            got = oracle.overlap(b[i], b[j])
            assert got == want, f"{name}: overlap({i}|{j}) = {float(got).hex()}, hand value {float(want).hex()}"
        for (i, want) in case["areas_f32"]:
            got = oracle.area(b[i])
            assert got == want, f"{name}: area({i}) = {float(got).hex()}, hand value {float(want).hex()}"
        keep = oracle.keep(b, s, th)
        assert keep.tolist() == case["keep"].tolist(), f"{name}: keep {keep.tolist()}"
        via_matrix = oracle.reduce(oracle.map(b, s, th))
        assert via_matrix.tolist() == case["keep"].tolist(), f"{name}: reduce(map) {via_matrix.tolist()}"
        greedy = oracle.greedy_keep(b, s, th)
        assert greedy.tolist() == case["greedy"].tolist(), f"{name}: greedy {greedy.tolist()}"
        # the paper's square-box statement on the same case, when its boxes are squares
        # with positive scores
        side = b[:, 2] - b[:, 0]
        if np.all(side == b[:, 3] - b[:, 1]) and np.all(s > 0):
            D = np.stack([b[:, 0], b[:, 1], side, s], axis=1).astype(np.float32)
            want = case["literal_keep"] if case["literal_keep"] is not None else case["keep"]
            for k in (1, len(s)):
                _, V = oracle.alg12_square(D, th, k)
                assert V.tolist() == want.tolist(), f"{name}: square-box form, k={k}: {V.tolist()}"


# --------------------------------------------------------------------------- exact rational model

def f32_round(x: Fraction) -> Fraction:
    """Round a rational to the nearest float32 (ties to even), returned as a
    rational.  Either sign; below the normal range the spacing stays 2^-149."""
    if x == 0:
        return Fraction(0)
    if x < 0:
        return -f32_round(-x)
    e = 0
    while x >= Fraction(2) ** (e + 1):
        e += 1
    while x < Fraction(2) ** e:
        e -= 1
    e = max(e, -126)
    ulp = Fraction(2) ** (e - 23)
    k, rem = divmod(x, ulp)
    k = int(k)
    if rem > ulp / 2 or (rem == ulp / 2 and (k & 1)):
        k += 1
    out = k * ulp
    assert out < Fraction(2) ** 128, "beyond the float32 range"
    return out


def exact_overlap(bi, bj) -> Fraction:
    """Overlap of victim bi with outranking bj for coordinates on which every
    float32 add, subtract and multiply is exact (small integers): only the final
    division rounds."""
    bi = [Fraction(float(v)) for v in bi]
    bj = [Fraction(float(v)) for v in bj]
    w = max(Fraction(0), min(bi[2], bj[2]) - max(bi[0], bj[0]) + 1)
    h = max(Fraction(0), min(bi[3], bj[3]) - max(bi[1], bj[1]) + 1)
    a = (bj[2] - bj[0] + 1) * (bj[3] - bj[1] + 1)
    return f32_round(w * h / a)


def exact_eliminates(boxes, scores, theta, j, i) -> bool:
    """Does j outrank i and overlap it with overlap >= theta?  Pure rationals."""
    sj, si = Fraction(float(scores[j])), Fraction(float(scores[i]))
    if not (sj > si or (sj == si and j < i)):
        return False
    return exact_overlap(boxes[i], boxes[j]) >= Fraction(float(theta))


def survivor_sets(boxes, scores, theta, rule):
    """All subsets K of {0..n-1} consistent with the rule, by exhaustive search.
    rule 'paper' : i in K  <=>  no j eliminates i
    rule 'greedy': i in K  <=>  no j IN K eliminates i"""
    n = len(scores)
    elim = [[exact_eliminates(boxes, scores, theta, j, i) for j in range(n)] for i in range(n)]
    found = []
    for bits in itertools.product((0, 1), repeat=n):
        ok = True
        for i in range(n):
            if rule == "paper":
                hit = any(elim[i][j] for j in range(n))
            else:
                hit = any(elim[i][j] and bits[j] for j in range(n))
            if bool(bits[i]) != (not hit):
                ok = False
                break
        if ok:
            found.append(list(bits))
    return found


def small_integer_frame(seed, n):
    rng = np.random.default_rng(seed)
    x1 = rng.integers(0, 24, n)
    y1 = rng.integers(0, 24, n)
    w = rng.integers(1, 17, n)
    h = rng.integers(1, 17, n)
    boxes = np.stack([x1, y1, x1 + w - 1, y1 + h - 1], axis=1).astype(np.float32)
    # few score levels so exact ties are frequent
    scores = (rng.integers(1, 6, n) / np.float32(8)).astype(np.float32)
    return boxes, scores


def pin_bruteforce(oracle, seeds=range(24)):
    thetas = [np.float32(0.5), np.float32(0.3), np.float32(0.125), np.float32(0.7)]
    for seed in seeds:
        n = 2 + seed % 7  # 2..8
        boxes, scores = small_integer_frame(seed, n)
        theta = thetas[seed % len(thetas)]
        paper = survivor_sets(boxes, scores, theta, "paper")
        assert len(paper) == 1
        got = oracle.keep(boxes, scores, theta).tolist()
        assert got == paper[0], f"seed {seed}: oracle {got}, exhaustive {paper[0]}"
        greedy = survivor_sets(boxes, scores, theta, "greedy")
        assert len(greedy) == 1, f"seed {seed}: greedy fixed point not unique"
        got_g = oracle.greedy_keep(boxes, scores, theta).tolist()
        assert got_g == greedy[0], f"seed {seed}: greedy oracle {got_g}, exhaustive {greedy[0]}"
        # the matrix and the ranked views, entry by entry
        B = oracle.map(boxes, scores, theta)
        for i in range(n):
            for j in range(n):
                want = 0 if exact_eliminates(boxes, scores, theta, j, i) else 1
                assert B[i, j] == want, f"seed {seed}: B[{i},{j}]"
        order = oracle.order(scores)
        rank_key = sorted(range(n), key=lambda t: (-Fraction(float(scores[t])), t))
        assert order.tolist() == rank_key, f"seed {seed}: order"
        E = oracle.ranked_eliminations(boxes, order, theta)
        words = oracle.ranked_elimination_words(boxes, order, theta)
        for r in range(n):
            for c in range(n):
                want = 1 if (c < r and exact_eliminates(boxes, scores, theta, order[c], order[r])) else 0
                assert E[r, c] == want, f"seed {seed}: E[{r},{c}]"
                assert ((int(words[r, c >> 6]) >> (c & 63)) & 1) == want
        ranked = oracle.ranked_boxes(boxes, order)
        for r in range(n):
            b = boxes[order[r]]
            area = (int(b[2]) - int(b[0]) + 1) * (int(b[3]) - int(b[1]) + 1)
            assert ranked[r].tolist() == [b[0], b[1], b[2], b[3], float(area)]


# --------------------------------------------------------------------------- closed forms

def pin_trivial(oracle):
    empty = oracle.keep(np.zeros((0, 4), np.float32), np.zeros(0, np.float32), 0.5)
    assert empty.shape == (0,)
    one = oracle.keep(np.array([[3, 4, 10, 12]], np.float32), np.array([0.2], np.float32), 0.5)
    assert one.tolist() == [1]
    # a 7x5 lattice of 10x10 boxes with one empty pixel between neighbours, including diagonal ones
    boxes = np.array([[11 * gx, 11 * gy, 11 * gx + 9, 11 * gy + 9] for gy in range(5) for gx in range(7)], np.float32)
    scores = np.linspace(0.9, 0.1, boxes.shape[0]).astype(np.float32)[::-1].copy()
    assert oracle.keep(boxes, scores, 0.01).tolist() == [1] * boxes.shape[0]
    assert oracle.greedy_keep(boxes, scores, 0.01).tolist() == [1] * boxes.shape[0]


def pin_theta_extremes(oracle):
    rng = np.random.default_rng(5)
    n = 40
    x1 = rng.integers(0, 200, n)
    y1 = rng.integers(0, 200, n)
    boxes = np.stack([x1, y1, x1 + rng.integers(1, 60, n), y1 + rng.integers(1, 60, n)], axis=1).astype(np.float32)
    scores = rng.permutation(n).astype(np.float32) / np.float32(n)
    top = int(np.argmax(scores))
    only_top = [1 if i == top else 0 for i in range(n)]
    # overlap is never negative, so with theta <= 0 every outranking box eliminates
    assert oracle.keep(boxes, scores, 0.0).tolist() == only_top
    assert oracle.keep(boxes, scores, -1.0).tolist() == only_top
    # the intersection lies inside the outranking box, so overlap <= 1 < theta: nothing is eliminated
    assert oracle.keep(boxes, scores, 1.0000001).tolist() == [1] * n
    assert oracle.keep(boxes, scores, 2.0).tolist() == [1] * n
    # theta = 1: eliminated exactly when the outranking box lies inside the victim
    keep = oracle.keep(boxes, scores, 1.0)
    for i in range(n):
        inside = any(scores[j] > scores[i] and boxes[j, 0] >= boxes[i, 0] and boxes[j, 1] >= boxes[i, 1]
                     and boxes[j, 2] <= boxes[i, 2] and boxes[j, 3] <= boxes[i, 3] for j in range(n))
        assert keep[i] == (0 if inside else 1)


def staircase(N, step=3):
    """N 10x10 boxes, each `step` rows below the previous one, scores strictly
    descending.  Overlap with the box s steps up is (10-3s)/10 for s <= 3: 0.7, 0.4, 0.1."""
    boxes = np.array([[0, step * k, 9, step * k + 9] for k in range(N)], np.float32)
    scores = (np.float32(1.0) - np.arange(N, dtype=np.float32) / np.float32(2 * N)).astype(np.float32)
    assert np.all(np.diff(scores) < 0)
    return boxes, scores


def pin_staircase(oracle, sizes=(1, 2, 3, 7, 64, 65, 200)):
    for N in sizes:
        boxes, scores = staircase(N)
        # theta 0.5: only the neighbour one step up eliminates -> paper rule keeps box 0 only,
        # the sequential procedure keeps every second box
        assert oracle.keep(boxes, scores, 0.5).tolist() == [1] + [0] * (N - 1)
        assert oracle.greedy_keep(boxes, scores, 0.5).tolist() == [1 - (k & 1) for k in range(N)]
        # theta 0.75: nothing reaches it
        assert oracle.keep(boxes, scores, 0.75).tolist() == [1] * N
        # theta 0.4 exactly: float32(40/100) vs float32(0.4) are the same number -> two steps up eliminates too;
        # sequential procedure then keeps every third box
        assert oracle.greedy_keep(boxes, scores, np.float32(0.4)).tolist() == [1 if k % 3 == 0 else 0 for k in range(N)]
        # reversed input order must give the reversed answer (distinct scores)
        assert oracle.keep(boxes[::-1].copy(), scores[::-1].copy(), 0.5).tolist() == [0] * (N - 1) + [1]
        # ranked views of the reversed input: rank r is input index N-1-r, and at theta 0.5
        # the only eliminator of rank r is rank r-1
        rb, rs = boxes[::-1].copy(), scores[::-1].copy()
        order = oracle.order(rs)
        assert order.tolist() == list(range(N - 1, -1, -1))
        E = oracle.ranked_eliminations(rb, order, 0.5)
        words = oracle.ranked_elimination_words(rb, order, 0.5)
        assert words.shape == (N, (N + 63) // 64)
        for r in range(N):
            want_row = [1 if c == r - 1 else 0 for c in range(N)]
            assert E[r].tolist() == want_row
            want_words = [0] * words.shape[1]
            if r > 0:
                want_words[(r - 1) >> 6] = 1 << ((r - 1) & 63)
            assert [int(v) for v in words[r]] == want_words


def pin_clusters(oracle):
    """m groups of c identical boxes, groups at least one empty pixel apart: one
    survivor per group, the group's best score; with equal scores inside a group,
    its lowest index."""
    rng = np.random.default_rng(11)
    m, c = 9, 5
    boxes, scores, group = [], [], []
    for g in range(m):
        x = 40 * (g % 3)
        y = 40 * (g // 3)
        for _ in range(c):
            boxes.append([x, y, x + 29, y + 19])
            group.append(g)
    boxes = np.array(boxes, np.float32)
    group = np.array(group)
    scores = (rng.permutation(m * c) + 1).astype(np.float32) / np.float32(64)
    perm = rng.permutation(m * c)
    boxes, group, scores = boxes[perm], group[perm], scores[perm]
    want = np.zeros(m * c, np.uint8)
    for g in range(m):
        idx = np.flatnonzero(group == g)
        want[idx[np.argmax(scores[idx])]] = 1
    assert oracle.keep(boxes, scores, 0.5).tolist() == want.tolist()
    assert oracle.greedy_keep(boxes, scores, 0.5).tolist() == want.tolist()
    # all scores equal: the first box of each group in input order survives
    flat = np.full(m * c, 0.5, np.float32)
    want = np.zeros(m * c, np.uint8)
    for g in range(m):
        want[np.flatnonzero(group == g)[0]] = 1
    assert oracle.keep(boxes, flat, 0.5).tolist() == want.tolist()


# --------------------------------------------------------------------------- the paper's square-box statement vs per-axis form

def pin_square_form(oracle):
    """On square boxes with distinct positive scores the per-axis oracle must equal
    the paper's Algorithm 1 + Algorithm 2 stated on {x, y, z, s} tuples in a
    zero-filled vector of capacity D_max > n, for every partition count k.
    Integer coordinates, so x + z and (x2 - x1) + 1 = z + 1 are exact and both
    forms see the same numbers."""
    for seed in range(6):
        rng = np.random.default_rng(100 + seed)
        n, dmax = 37 + seed, 64
        x = rng.integers(0, 120, n).astype(np.float32)
        y = rng.integers(0, 120, n).astype(np.float32)
        z = rng.integers(3, 40, n).astype(np.float32)
        s = ((rng.permutation(n) + 1) / np.float32(n + 1)).astype(np.float32)
        D = np.zeros((dmax, 4), np.float32)
        D[:n] = np.stack([x, y, z, s], axis=1)
        boxes = np.stack([x, y, x + z, y + z], axis=1).astype(np.float32)
        theta = np.float32([0.5, 0.3, 0.45][seed % 3])
        keep = oracle.keep(boxes, s, theta)
        B_general = oracle.map(boxes, s, theta)
        for k in (1, 2, 4, 8, 32, 64):
            B, V = oracle.alg12_square(D, theta, k)
            assert V[:n].tolist() == keep.tolist(), f"seed {seed}, k={k}"
            assert np.array_equal(B[:n, :n], B_general), f"seed {seed}, k={k}: matrix"
            # columns of empty slots (score 0) never pass the score guard: still the preset ones
            assert np.all(B[:, n:] == 1)
    # The listing's second term, "AND D[j].z != 0", as it stands: where the guard does fire against
    # an empty slot j (score 0, side 0) -- that takes a NEGATIVE score s_i -- the term is false, so
    # B_ij = 0 and V_i = 0 whatever the overlap.  Two squares far from the origin and from each
    # other, capacity 4 (two empty slots): the positive-score one survives, the negative-score one
    # does not; its row has zeros exactly in the empty slots' columns.
    D = np.zeros((4, 4), np.float32)
    D[0] = [100, 100, 10, 0.5]
    D[1] = [300, 300, 10, -0.5]
    for k in (1, 2, 4):
        B, V = oracle.alg12_square(D, np.float32(0.5), k)
        assert V.tolist() == [1, 0, 1, 1], f"k={k}: {V.tolist()}"
        assert B.tolist() == [[1, 1, 1, 1], [1, 1, 0, 0], [1, 1, 1, 1], [1, 1, 1, 1]], f"k={k}"


ALL_PINS = [
    ("golden", pin_golden),
    ("bruteforce", pin_bruteforce),
    ("trivial", pin_trivial),
    ("theta_extremes", pin_theta_extremes),
    ("staircase", pin_staircase),
    ("clusters", pin_clusters),
    ("square_form", pin_square_form),
]


def _with_variants():
    from pins_rounding import ROUNDING_PINS  # both import f32_round from this module: resolved lazily
    from pins_variants import VARIANT_PINS

    return VARIANT_PINS + ROUNDING_PINS


ALL_PINS = ALL_PINS + _with_variants()
