"""Pins for the oracle's selectable variants (``Oracle.keep_ex``): intersection over
union, strict compare, ignored ties, pixel offset 0, class labels, greedy rule.

As in pins.py, no expected value comes from the oracle: hand-worked fixtures
(tests/golden/variants), an exact rational model with exhaustive search over all
survivor sets on tiny frames, closed forms and containments that hold for every input.
"""
from __future__ import annotations

import glob
import itertools
import os
from fractions import Fraction

import numpy as np

VARIANT_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "variants")
DEFAULTS = {"rule": "paper", "measure": "outranking_area", "compare": "ge", "ties": "index", "offset": "1",
            "classes": "off"}


def parse_variant_file(path):
    case = {"boxes": [], "scores": [], "classes": None, "theta": None, "expect": [], "path": path}
    with open(path) as fh:
        for raw in fh:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            tok = line.split()
            if tok[0] == "theta":
                case["theta"] = np.float32(tok[1])
            elif tok[0] == "box":
                case["boxes"].append([float(v) for v in tok[1:5]])
                case["scores"].append(float(tok[5]))
            elif tok[0] == "classes":
                case["classes"] = np.array([int(v) for v in tok[1:]], np.int32)
            elif tok[0] == "expect":
                opts = dict(DEFAULTS)
                keep = None
                for kv in tok[1:]:
                    k, v = kv.split("=")
                    if k == "keep":
                        keep = [int(b) for b in v.split(",")]
                    else:
                        assert k in opts, f"{path}: unknown option {k}"
                        opts[k] = v
                assert keep is not None
                case["expect"].append((opts, keep))
            else:
                raise ValueError(f"{path}: unknown directive {tok[0]}")
    case["boxes"] = np.array(case["boxes"], np.float32).reshape(-1, 4)
    case["scores"] = np.array(case["scores"], np.float32)
    return case


def call_keep_ex(oracle, boxes, scores, theta, opts, classes):
    return oracle.keep_ex(boxes, scores, theta, rule=opts["rule"], measure=opts["measure"], compare=opts["compare"],
                          ties=opts["ties"], pixel_offset=float(opts["offset"]),
                          classes=classes if opts["classes"] == "on" else None)


def pin_variant_golden(oracle):
    paths = sorted(glob.glob(os.path.join(VARIANT_DIR, "*.txt")))
    assert len(paths) >= 12, "variant fixtures missing"
    seen = set()
    for path in paths:
        case = parse_variant_file(path)
        name = os.path.basename(path)
        assert case["expect"], name
        for opts, keep in case["expect"]:
            if opts["classes"] == "on":
                assert case["classes"] is not None, name
            got = call_keep_ex(oracle, case["boxes"], case["scores"], case["theta"], opts, case["classes"]).tolist()
            assert got == keep, f"{name}: {opts}: keep {got}, hand value {keep}"
            seen.update((k, v) for k, v in opts.items() if v != DEFAULTS[k])
    # every switch is exercised by some fixture
    assert seen >= {("rule", "greedy"), ("measure", "iou"), ("compare", "gt"), ("ties", "ignore"), ("offset", "0"),
                    ("classes", "on")}


# --------------------------------------------------------------------------- exact rational model

def exact_eliminates_ex(boxes, scores, classes, theta, j, i, measure, compare, ties, offset):
    """Does j eliminate i under the options?  Integer coordinates: every add, subtract
    and multiply is exact in float32, only the final division rounds."""
    from pins import f32_round  # here, not at the top: pins imports this module to extend ALL_PINS

    sj, si = Fraction(float(scores[j])), Fraction(float(scores[i]))
    if ties == "ignore":
        if not sj > si:
            return False
    elif not (sj > si or (sj == si and j < i)):
        return False
    if classes is not None and int(classes[j]) != int(classes[i]):
        return False
    bi = [Fraction(float(v)) for v in boxes[i]]
    bj = [Fraction(float(v)) for v in boxes[j]]
    off = Fraction(offset)
    w = max(Fraction(0), min(bi[2], bj[2]) - max(bi[0], bj[0]) + off)
    h = max(Fraction(0), min(bi[3], bj[3]) - max(bi[1], bj[1]) + off)
    inter = w * h
    area_i = (bi[2] - bi[0] + off) * (bi[3] - bi[1] + off)
    area_j = (bj[2] - bj[0] + off) * (bj[3] - bj[1] + off)
    denom = area_j if measure == "outranking_area" else area_i + area_j - inter
    assert denom > 0
    q = f32_round(inter / denom)
    t = Fraction(float(theta))
    return q > t if compare == "gt" else q >= t


def survivor_sets_ex(n, elim, rule):
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


def small_frame(seed, n):
    """Integer boxes with at least one pixel between the corners (so that offset 0 still
    gives positive areas), few score levels, few labels."""
    rng = np.random.default_rng(seed)
    x1 = rng.integers(0, 20, n)
    y1 = rng.integers(0, 20, n)
    w = rng.integers(1, 15, n)
    h = rng.integers(1, 15, n)
    boxes = np.stack([x1, y1, x1 + w, y1 + h], axis=1).astype(np.float32)
    scores = (rng.integers(1, 5, n) / np.float32(8)).astype(np.float32)
    classes = rng.integers(0, 3, n).astype(np.int32)
    return boxes, scores, classes


OPTION_GRID = [dict(rule=r, measure=m, compare=c, ties=t, offset=o, classes=k)
               for r in ("paper", "greedy") for m in ("outranking_area", "iou") for c in ("ge", "gt")
               for t in ("index", "ignore") for o in ("1", "0") for k in ("off", "on")]


def pin_variant_bruteforce(oracle, seeds=range(16)):
    thetas = [np.float32(0.5), np.float32(0.25), np.float32(1.0 / 3.0), np.float32(0.125)]
    for seed in seeds:
        n = 2 + seed % 6  # 2..7
        boxes, scores, classes = small_frame(seed, n)
        theta = thetas[seed % len(thetas)]
        # all 64 option combinations on the first seeds, a rotating quarter afterwards
        grid = OPTION_GRID if seed < 4 else OPTION_GRID[seed % 4::4]
        for opts in grid:
            cls = classes if opts["classes"] == "on" else None
            elim = [[exact_eliminates_ex(boxes, scores, cls, theta, j, i, opts["measure"], opts["compare"],
                                         opts["ties"], int(opts["offset"])) for j in range(n)] for i in range(n)]
            want = survivor_sets_ex(n, elim, opts["rule"])
            assert len(want) == 1, f"seed {seed} {opts}: survivor set not unique"
            got = call_keep_ex(oracle, boxes, scores, theta, opts, classes).tolist()
            assert got == want[0], f"seed {seed} {opts}: oracle {got}, exhaustive {want[0]}"
            for i in range(n):
                for j in range(n):
                    one = oracle.eliminates_ex(boxes, scores, j, i, theta, measure=opts["measure"],
                                               compare=opts["compare"], ties=opts["ties"],
                                               pixel_offset=float(opts["offset"]), classes=cls)
                    assert one == elim[i][j], f"seed {seed} {opts}: pair ({j} eliminates {i})"


# --------------------------------------------------------------------------- closed forms and containments

def pin_variant_closed_forms(oracle):
    rng = np.random.default_rng(17)
    n = 60
    x1 = rng.integers(0, 150, n)
    y1 = rng.integers(0, 150, n)
    boxes = np.stack([x1, y1, x1 + rng.integers(1, 50, n), y1 + rng.integers(1, 50, n)], axis=1).astype(np.float32)
    scores = (rng.integers(1, 30, n) / np.float32(32)).astype(np.float32)  # ties are common
    theta = np.float32(0.3)
    base = oracle.keep_ex(boxes, scores, theta)

    # all switches off: the functions pinned in pins.py
    assert base.tolist() == oracle.keep(boxes, scores, theta).tolist()
    assert oracle.keep_ex(boxes, scores, theta, rule="greedy").tolist() == oracle.greedy_keep(boxes, scores, theta).tolist()

    # labels: all different -> nothing interacts; all equal -> as without labels
    for rule in ("paper", "greedy"):
        assert oracle.keep_ex(boxes, scores, theta, rule=rule, classes=np.arange(n)).tolist() == [1] * n
        assert oracle.keep_ex(boxes, scores, theta, rule=rule, classes=np.full(n, 4)).tolist() == \
            oracle.keep_ex(boxes, scores, theta, rule=rule).tolist()
    # two labels: each class behaves as a frame of its own
    labels = rng.integers(0, 2, n).astype(np.int32)
    for rule in ("paper", "greedy"):
        got = oracle.keep_ex(boxes, scores, theta, rule=rule, classes=labels)
        for c in (0, 1):
            idx = np.flatnonzero(labels == c)
            alone = oracle.keep_ex(boxes[idx], scores[idx], theta, rule=rule)
            assert got[idx].tolist() == alone.tolist()

    # fewer eliminations -> more survivors (paper rule): union >= outranking area (exact on integer
    # boxes), ">" is implied by ">=", ignoring ties removes eliminators
    def subset(a, b):
        return bool(np.all(a <= b))
    iou = oracle.keep_ex(boxes, scores, theta, measure="iou")
    assert subset(base, iou) and base.sum() < iou.sum()
    assert subset(base, oracle.keep_ex(boxes, scores, theta, compare="gt"))
    ign = oracle.keep_ex(boxes, scores, theta, ties="ignore")
    assert subset(base, ign) and base.sum() < ign.sum()
    # paper rule keeps a subset of the greedy rule, whatever the options
    for kw in (dict(measure="iou"), dict(compare="gt"), dict(ties="ignore"), dict(pixel_offset=0.0),
               dict(measure="iou", pixel_offset=0.0, classes=labels)):
        assert subset(oracle.keep_ex(boxes, scores, theta, **kw), oracle.keep_ex(boxes, scores, theta, rule="greedy", **kw))

    # one score for everybody, ties ignored: nothing outranks anything
    flat = np.full(n, 0.5, np.float32)
    for rule in ("paper", "greedy"):
        assert oracle.keep_ex(boxes, flat, theta, rule=rule, ties="ignore").tolist() == [1] * n
    # ... by index: box 0 survives, and so does exactly one box per group of mutually overlapping copies
    copies = np.repeat(boxes[:5], 4, axis=0)
    far = copies + np.repeat(np.arange(5, dtype=np.float32) * 1000, 4)[:, None]
    want = [1, 0, 0, 0] * 5
    assert oracle.keep_ex(far, np.full(20, 0.5, np.float32), 0.9, measure="iou").tolist() == want
    assert oracle.keep_ex(far, np.full(20, 0.5, np.float32), 0.9, measure="iou", rule="greedy").tolist() == want
    # identical boxes have IoU exactly 1: ">" at theta = 1 keeps them all, ">=" does not
    assert oracle.keep_ex(far, np.full(20, 0.5, np.float32), 1.0, measure="iou", compare="gt").tolist() == [1] * 20
    assert oracle.keep_ex(far, np.full(20, 0.5, np.float32), 1.0, measure="iou").tolist() == want

    # IoU extremes: theta <= 0 leaves the top rank only, theta > 1 everything
    distinct = (rng.permutation(n) + 1).astype(np.float32) / np.float32(n + 1)
    top = int(np.argmax(distinct))
    assert oracle.keep_ex(boxes, distinct, 0.0, measure="iou").tolist() == [1 if i == top else 0 for i in range(n)]
    assert oracle.keep_ex(boxes, distinct, 1.0000001, measure="iou").tolist() == [1] * n
    # IoU = 1 only for identical boxes: at theta = 1 a box dies iff an identical box outranks it
    keep1 = oracle.keep_ex(boxes, distinct, 1.0, measure="iou")
    for i in range(n):
        twin = any(distinct[j] > distinct[i] and np.array_equal(boxes[j], boxes[i]) for j in range(n))
        assert keep1[i] == (0 if twin else 1)

    # offset 0 on a lattice of boxes that share edges: zero-width intersections, nobody dies;
    # with offset 1 the shared pixel row/column has positive overlap
    lattice = np.array([[10 * gx, 10 * gy, 10 * gx + 10, 10 * gy + 10] for gy in range(4) for gx in range(5)], np.float32)
    ls = np.linspace(0.9, 0.1, 20).astype(np.float32)
    assert oracle.keep_ex(lattice, ls, 0.01, pixel_offset=0.0).tolist() == [1] * 20
    assert oracle.keep_ex(lattice, ls, 0.01, pixel_offset=0.0, measure="iou").tolist() == [1] * 20
    # offset 1: neighbours share an 11-pixel edge strip, 11/121 = 0.0909 >= 0.01 -> only box 0 (top score,
    # no outranking neighbour) and boxes whose better-scored neighbours are all diagonal... every box but
    # the first has its left or upper neighbour outranking it
    assert oracle.keep_ex(lattice, ls, 0.01, pixel_offset=1.0).tolist() == [1] + [0] * 19


VARIANT_PINS = [
    ("variant_golden", pin_variant_golden),
    ("variant_bruteforce", pin_variant_bruteforce),
    ("variant_closed_forms", pin_variant_closed_forms),
]
