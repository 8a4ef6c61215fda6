"""Properties of the paper's rule that hold for every input (no GPU).

Each property is checked on the oracle's output with the pair tests recomputed
here in float32 numpy.  That recomputation repeats the formula, so it says nothing
about the formula itself or its rounding order (tests/pins.py and
tests/pins_rounding.py pin those against hand-worked values and an exact model);
what this file adds are the properties: witnesses, containments, invariances.
"""
import numpy as np
import pytest

from workloads import make_config, random_frame


def np_overlap_matrix(boxes):
    """Q[i, j] = overlap of victim i with box j (Algorithm 1's measure, per axis),
    float32 throughout: numpy evaluates every elementwise operation separately."""
    b = boxes.astype(np.float32)
    one = np.float32(1.0)
    zero = np.float32(0.0)
    far_x = np.minimum(b[:, None, 2], b[None, :, 2])
    near_x = np.maximum(b[:, None, 0], b[None, :, 0])
    w = np.maximum(zero, (far_x - near_x) + one)
    far_y = np.minimum(b[:, None, 3], b[None, :, 3])
    near_y = np.maximum(b[:, None, 1], b[None, :, 1])
    h = np.maximum(zero, (far_y - near_y) + one)
    area = ((b[:, 2] - b[:, 0]) + one) * ((b[:, 3] - b[:, 1]) + one)
    q = (w * h) / area[None, :]
    assert q.dtype == np.float32
    return q


def np_outranks_matrix(scores):
    """R[i, j] = j outranks i."""
    s = scores.astype(np.float32)
    idx = np.arange(s.shape[0])
    return (s[None, :] > s[:, None]) | ((s[None, :] == s[:, None]) & (idx[None, :] < idx[:, None]))


FRAMES = [
    ("int_ties", lambda: random_frame(1, 300, integer=True, score_levels=7), 0.5),
    ("int", lambda: random_frame(2, 257, integer=True), 0.3),
    ("float", lambda: random_frame(3, 320, integer=False), 0.45),
    ("float_ties", lambda: random_frame(4, 191, integer=False, score_levels=5), 0.5),
    ("cfg0", lambda: (make_config(0).boxes[0], make_config(0).scores[0]), 0.5),
    ("cfg4_frame", lambda: (make_config(4, frames=1).boxes[0][:1500], make_config(4, frames=1).scores[0][:1500]), 0.45),
]


@pytest.mark.parametrize("name,make,theta", FRAMES, ids=[f[0] for f in FRAMES])
def test_rule_properties(oracle, name, make, theta):
    boxes, scores = make()
    theta = np.float32(theta)
    n = scores.shape[0]
    keep = oracle.keep(boxes, scores, theta).astype(bool)
    greedy = oracle.greedy_keep(boxes, scores, theta).astype(bool)
    Q = np_overlap_matrix(boxes)
    R = np_outranks_matrix(scores)
    elim = R & ~(Q < theta)  # elim[i, j]: j eliminates i

    # the top-ranked box survives
    top = int(np.lexsort((np.arange(n), -scores.astype(np.float64)))[0])
    assert keep[top] and greedy[top]
    # every eliminated box has a witness, every survivor has none (ReduceKernel postcondition)
    assert np.array_equal(keep, ~elim.any(axis=1))
    # survivors do not eliminate each other
    assert not elim[np.ix_(keep, keep)].any()
    # whatever the paper's rule keeps, the sequential procedure keeps too
    assert not (keep & ~greedy).any()
    # sequential procedure: a box is out iff a KEPT box eliminates it
    assert np.array_equal(greedy, ~(elim & greedy[None, :]).any(axis=1))
    # MapKernel postcondition, entry by entry
    B = oracle.map(boxes, scores, theta).astype(bool)
    assert np.array_equal(B, ~elim)
    assert np.array_equal(oracle.reduce(B.astype(np.uint8)).astype(bool), keep)


@pytest.mark.parametrize("name,make,theta", FRAMES, ids=[f[0] for f in FRAMES])
def test_ranked_views(oracle, name, make, theta):
    boxes, scores = make()
    theta = np.float32(theta)
    n = scores.shape[0]
    order = oracle.order(scores)
    # a permutation, scores non-increasing, equal scores in index order
    assert sorted(order.tolist()) == list(range(n))
    so = scores[order]
    assert np.all(so[:-1] >= so[1:])
    same = so[:-1] == so[1:]
    assert np.all(order[:-1][same] < order[1:][same])
    assert order.tolist() == np.lexsort((np.arange(n), -scores.astype(np.float64))).tolist()
    # ranked boxes: a gather plus the area of Algorithm 1's first line
    ranked = oracle.ranked_boxes(boxes, order)
    assert np.array_equal(ranked[:, :4], boxes[order])
    one = np.float32(1)
    assert np.array_equal(ranked[:, 4], ((boxes[order, 2] - boxes[order, 0]) + one) * ((boxes[order, 3] - boxes[order, 1]) + one))
    # ranked elimination bits = complement of B, permuted, strictly lower triangle
    B = oracle.map(boxes, scores, theta)
    E = oracle.ranked_eliminations(boxes, order, theta)
    assert np.array_equal(E, (1 - B[np.ix_(order, order)]))
    assert not np.triu(E).any()
    words = oracle.ranked_elimination_words(boxes, order, theta)
    bits = np.unpackbits(words.view(np.uint8), bitorder="little").reshape(n, -1)[:, :n]
    assert np.array_equal(bits, E)
    # keep from the ranked view, scattered back to input order
    keep = oracle.keep(boxes, scores, theta)
    ranked_keep = np.zeros(n, np.uint8)
    ranked_keep[order] = (~E.any(axis=1)).astype(np.uint8)
    assert np.array_equal(ranked_keep, keep)


def test_permutation_invariance(oracle):
    """Distinct scores: the result does not depend on the order of D (the paper's
    claim that the input need not be sorted)."""
    boxes, scores = random_frame(7, 400, integer=False)
    assert np.unique(scores).size == scores.size
    keep = oracle.keep(boxes, scores, 0.4)
    for seed in range(3):
        perm = np.random.default_rng(seed).permutation(scores.size)
        assert np.array_equal(oracle.keep(boxes[perm], scores[perm], 0.4), keep[perm])


def test_monotone_in_theta(oracle):
    boxes, scores = random_frame(8, 300, integer=False, score_levels=9)
    prev = None
    for theta in (0.0, 0.1, 0.25, 0.5, 0.5000001, 0.75, 1.0, 1.5):
        keep = oracle.keep(boxes, scores, theta).astype(bool)
        if prev is not None:
            assert not (prev & ~keep).any()
        prev = keep


def test_integer_translation(oracle):
    """Integer coordinates far below 2^24: all sums exact, so shifting every box by
    an integer vector cannot change a single decision."""
    boxes, scores = random_frame(9, 256, integer=True, score_levels=11)
    keep = oracle.keep(boxes, scores, 0.37)
    shifted = boxes + np.array([1000, 513, 1000, 513], np.float32)
    assert np.array_equal(oracle.keep(shifted, scores, 0.37), keep)


def test_rules_differ_on_crowd(oracle):
    """The dense-crowd configuration has suppression chains: the paper's rule keeps
    a strict subset of what the sequential procedure keeps."""
    w = make_config(3)
    b, s = w.boxes[0][:3000], w.scores[0][:3000]
    keep = oracle.keep(b, s, w.theta).astype(bool)
    greedy = oracle.greedy_keep(b, s, w.theta).astype(bool)
    assert not (keep & ~greedy).any()
    assert greedy.sum() > keep.sum()
