"""The oracle's rank order on scores of every kind (no GPU): Algorithm 1's guard
D[i].s < D[j].s is a float comparison and holds for any non-NaN float, so negative
scores, both zeros, denormals and infinities must order as the real numbers they stand
for (with -inf and +inf at the ends), ties going to the lower index."""
from fractions import Fraction

import numpy as np
import pytest

from workloads import random_frame, scores_of_every_kind


def real_key(score, index):
    """Sort key of the total order, worked in exact arithmetic: better first."""
    s = float(score)
    if s == float("inf"):
        return (0, Fraction(0), index)
    if s == float("-inf"):
        return (2, Fraction(0), index)
    return (1, -Fraction(s), index)  # Fraction(-0.0) == Fraction(0.0): the two zeros tie


@pytest.mark.parametrize("n,seed", [(7, 0), (65, 1), (300, 2), (1500, 3)])
def test_order_on_every_kind_of_score(oracle, n, seed):
    scores = scores_of_every_kind(seed, n)
    want = sorted(range(n), key=lambda t: real_key(scores[t], t))
    assert oracle.order(scores).tolist() == want
    # the pair predicate itself, on a sample of pairs
    rng = np.random.default_rng(seed)
    for j, i in rng.integers(0, n, (400, 2)):
        assert oracle.outranks(scores, j, i) == (real_key(scores[j], j) < real_key(scores[i], i))


def test_special_scores_hand_case(oracle):
    """Seven copies of one box: only the best-ranked copy survives (every pair overlaps
    fully), whatever kind of number the scores are."""
    box = np.array([[3, 4, 20, 30]] * 7, np.float32)
    tiny = np.float32(1e-45)
    scores = np.array([-np.inf, -1.0, -0.0, 0.0, tiny, 1.0, np.inf], np.float32)
    assert oracle.order(scores).tolist() == [6, 5, 4, 2, 3, 1, 0]  # -0.0 and +0.0 tie: index 2 before 3
    assert oracle.keep(box, scores, 0.5).tolist() == [0, 0, 0, 0, 0, 0, 1]
    assert oracle.greedy_keep(box, scores, 0.5).tolist() == [0, 0, 0, 0, 0, 0, 1]
    two_inf = np.array([np.inf, -tiny, np.inf, -np.inf, -np.inf, tiny, -tiny], np.float32)
    assert oracle.order(two_inf).tolist() == [0, 2, 5, 1, 6, 3, 4]
    assert oracle.keep(box, two_inf, 0.5).tolist() == [1, 0, 0, 0, 0, 0, 0]
    # ties ignored (Algorithm 1's strict test as printed): the two +inf copies do not touch each other
    assert oracle.keep_ex(box, two_inf, 0.5, ties="ignore").tolist() == [1, 0, 1, 0, 0, 0, 0]
    # disjoint boxes: nobody is eliminated, the scores do not matter
    far = box + (np.arange(7, dtype=np.float32) * 100)[:, None]
    assert oracle.keep(far, two_inf, 0.5).tolist() == [1] * 7


def test_keep_matches_rank_transformed_scores(oracle):
    """The rule depends on the scores only through their order: replacing every score by
    minus its rank position (distinct small integers) must not change the result."""
    for seed, n in [(11, 200), (12, 513)]:
        boxes, _ = random_frame(seed, n, extent=400, max_side=90, integer=(seed % 2 == 0))
        scores = scores_of_every_kind(seed, n)
        order = sorted(range(n), key=lambda t: real_key(scores[t], t))
        plain = np.empty(n, np.float32)
        plain[order] = -np.arange(n, dtype=np.float32)
        for theta in (0.3, 0.5):
            assert oracle.keep(boxes, scores, theta).tolist() == oracle.keep(boxes, plain, theta).tolist()
            assert oracle.greedy_keep(boxes, scores, theta).tolist() == oracle.greedy_keep(boxes, plain, theta).tolist()
