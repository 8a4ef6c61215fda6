"""Synthetic stand-ins for the paper's detector outputs (Evaluation Methodology
section: hundreds of face detections per 1080p frame, four times that on the 4K
mosaic, about 3000 on the large still picture; capacity D_max = 4096).

Every frame is produced from ``numpy.random.default_rng(seed)`` and cast to
float32 exactly once, so the identical arrays reach the oracle and the GPU.
Boxes are ``(x1, y1, x2, y2)`` with ``x2 >= x1 + 1`` and ``y2 >= y1 + 1``;
scores lie in (0, 1).  Nothing here evaluates overlaps or ranks boxes.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

CONFIG_NAMES = (
    "cfg0_1x1024_1080p",
    "cfg1_1x4096_4k",
    "cfg2_64x1024_1080p",
    "cfg3_1x16384_crowd_ties",
    "cfg4_256x4096_anchors",
)


@dataclass
class Workload:
    """A batch of frames: boxes [F, n, 4] f32, scores [F, n] f32, threshold."""

    name: str
    boxes: np.ndarray
    scores: np.ndarray
    theta: float

    @property
    def frames(self) -> int:
        return int(self.boxes.shape[0])

    @property
    def n(self) -> int:
        return int(self.boxes.shape[1])

    @property
    def pair_tests(self) -> int:
        """Evaluated pairs: F * n(n-1)/2 (the ranked half of the n x n grid)."""
        n = self.n
        return self.frames * (n * (n - 1) // 2)


def _finish_boxes(cx, cy, w, h, width, height):
    """Corner form, clipped to the frame, at least one pixel wide and high."""
    x1 = np.clip(cx - 0.5 * w, 0.0, width - 1.0)
    y1 = np.clip(cy - 0.5 * h, 0.0, height - 1.0)
    x2 = np.clip(cx + 0.5 * w, 0.0, width - 1.0)
    y2 = np.clip(cy + 0.5 * h, 0.0, height - 1.0)
    boxes = np.stack([x1, y1, x2, y2], axis=1).astype(np.float32)
    # clipping (or the float32 cast) may leave a sliver: widen it to one pixel,
    # moving whichever edge still has room inside the frame
    for lo, hi, lim in ((0, 2, width), (1, 3, height)):
        thin = boxes[:, hi] < boxes[:, lo] + np.float32(1.0)
        grow_hi = thin & (boxes[:, lo] + np.float32(1.0) <= np.float32(lim - 1.0))
        grow_lo = thin & ~grow_hi
        boxes[grow_hi, hi] = boxes[grow_hi, lo] + np.float32(1.0)
        boxes[grow_lo, lo] = boxes[grow_lo, hi] - np.float32(1.0)
    return boxes


def _jittered_candidates(rng, cx, cy, w, h, per_object):
    """per_object candidates around every object: centre noise 8 % of the side,
    side lengths scaled by exp(N(0, 0.1)) independently."""
    m = cx.shape[0]
    cxs = np.repeat(cx, per_object) + rng.normal(0.0, 1.0, m * per_object) * 0.08 * np.repeat(w, per_object)
    cys = np.repeat(cy, per_object) + rng.normal(0.0, 1.0, m * per_object) * 0.08 * np.repeat(h, per_object)
    ws = np.repeat(w, per_object) * np.exp(rng.normal(0.0, 0.1, m * per_object))
    hs = np.repeat(h, per_object) * np.exp(rng.normal(0.0, 0.1, m * per_object))
    return cxs, cys, ws, hs


def clustered_frame(seed, objects, width, height, size_lo, size_hi, per_object=16):
    """Objects uniform in the frame, each with a cluster of jittered candidates
    (configs 0, 1, 2).  Aspect ratio 2^U[-1,1]; scores Beta(5,2); shuffled."""
    rng = np.random.default_rng(seed)
    cx = rng.uniform(0.0, width, objects)
    cy = rng.uniform(0.0, height, objects)
    size = rng.uniform(size_lo, size_hi, objects)
    rho = np.exp2(rng.uniform(-1.0, 1.0, objects))
    w = size * np.sqrt(rho)
    h = size / np.sqrt(rho)
    cxs, cys, ws, hs = _jittered_candidates(rng, cx, cy, w, h, per_object)
    boxes = _finish_boxes(cxs, cys, ws, hs, width, height)
    scores = rng.beta(5.0, 2.0, boxes.shape[0]).astype(np.float32)
    perm = rng.permutation(boxes.shape[0])
    return boxes[perm], scores[perm]


def crowd_frame(seed, grid=32, width=3840, height=2160, size_lo=24.0, size_hi=96.0,
                per_object=16, tie_fraction=0.01):
    """Dense crowd (config 3): grid x grid near-square objects on a jittered
    lattice so neighbouring clusters overlap; 1 % of the scores are overwritten
    with another box's score to create exact ties."""
    rng = np.random.default_rng(seed)
    objects = grid * grid
    pitch_x = width / grid
    pitch_y = height / grid
    gx, gy = np.meshgrid(np.arange(grid), np.arange(grid), indexing="xy")
    cx = (gx.ravel() + 0.5 + rng.uniform(-0.5, 0.5, objects)) * pitch_x
    cy = (gy.ravel() + 0.5 + rng.uniform(-0.5, 0.5, objects)) * pitch_y
    size = rng.uniform(size_lo, size_hi, objects)
    rho = np.exp2(rng.uniform(-0.1, 0.1, objects))
    w = size * np.sqrt(rho)
    h = size / np.sqrt(rho)
    cxs, cys, ws, hs = _jittered_candidates(rng, cx, cy, w, h, per_object)
    boxes = _finish_boxes(cxs, cys, ws, hs, width, height)
    n = boxes.shape[0]
    scores = rng.beta(5.0, 2.0, n).astype(np.float32)
    perm = rng.permutation(n)
    boxes, scores = boxes[perm], scores[perm]
    ties = int(round(tie_fraction * n))
    dst = rng.choice(n, size=ties, replace=False)
    src = rng.integers(0, n, size=ties)
    scores[dst] = scores[src]
    return boxes, scores


def _anchor_table(image=512, strides=(8, 16, 32, 64, 128, 256), aspects=(0.5, 1.0, 2.0)):
    rows = []
    for stride in strides:
        cells = image // stride
        centre = (np.arange(cells) + 0.5) * stride
        gx, gy = np.meshgrid(centre, centre, indexing="xy")
        for a in aspects:
            size = 4.0 * stride
            w = size * np.sqrt(a)
            h = size / np.sqrt(a)
            rows.append(np.stack([gx.ravel(), gy.ravel(),
                                  np.full(gx.size, w), np.full(gx.size, h)], axis=1))
    return np.concatenate(rows, axis=0)


_ANCHORS = None


def anchor_frame(seed, n=4096, image=512, hot_fraction=0.02):
    """SSD-style frame (config 4): n anchors drawn without replacement from a
    six-level pyramid, regressed by N(0, 0.1) offsets; 2 % of the boxes score
    Beta(8,2), the rest Beta(1,8)."""
    global _ANCHORS
    if _ANCHORS is None:
        _ANCHORS = _anchor_table(image)
    rng = np.random.default_rng(seed)
    pick = rng.choice(_ANCHORS.shape[0], size=n, replace=False)
    a = _ANCHORS[pick]
    cx = a[:, 0] + rng.normal(0.0, 0.1, n) * a[:, 2]
    cy = a[:, 1] + rng.normal(0.0, 0.1, n) * a[:, 3]
    w = a[:, 2] * np.exp(rng.normal(0.0, 0.1, n))
    h = a[:, 3] * np.exp(rng.normal(0.0, 0.1, n))
    boxes = _finish_boxes(cx, cy, w, h, image, image)
    hot = int(round(hot_fraction * n))
    scores = rng.beta(1.0, 8.0, n)
    hot_idx = rng.choice(n, size=hot, replace=False)
    scores[hot_idx] = rng.beta(8.0, 2.0, hot)
    return boxes, scores.astype(np.float32)


def random_frame(seed, n, extent=256, max_side=64, integer=True, score_levels=0):
    """Small unstructured frame for unit tests: uniform corners, optional integer
    coordinates (all arithmetic on them is exact in float32) and optionally only
    ``score_levels`` distinct scores so that exact ties are common."""
    rng = np.random.default_rng(seed)
    if integer:
        x1 = rng.integers(0, extent, n).astype(np.float64)
        y1 = rng.integers(0, extent, n).astype(np.float64)
        w = rng.integers(1, max_side + 1, n).astype(np.float64)
        h = rng.integers(1, max_side + 1, n).astype(np.float64)
    else:
        x1 = rng.uniform(0, extent, n)
        y1 = rng.uniform(0, extent, n)
        w = rng.uniform(1, max_side, n)
        h = rng.uniform(1, max_side, n)
    boxes = np.stack([x1, y1, x1 + w, y1 + h], axis=1).astype(np.float32)
    if not integer:
        boxes[:, 2] = np.maximum(boxes[:, 2], boxes[:, 0] + np.float32(1.0))
        boxes[:, 3] = np.maximum(boxes[:, 3], boxes[:, 1] + np.float32(1.0))
    if score_levels:
        scores = (rng.integers(1, score_levels + 1, n) / np.float32(score_levels + 1)).astype(np.float32)
    else:
        scores = rng.uniform(0.01, 1.0, n).astype(np.float32)
    return boxes, scores


def scores_of_every_kind(seed, n):
    """Scores as a detector may emit them before any squashing (raw logits): negative and
    positive values over many magnitudes, both zeros, denormals of both signs, both
    infinities, and exact ties among all of these.  No NaN."""
    rng = np.random.default_rng(seed)
    tiny = np.float32(1e-45)  # the smallest positive denormal
    palette = np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, tiny, -tiny, 3 * tiny, -3 * tiny, 1e-39, -1e-39,
                        1.1754944e-38, -1.1754944e-38, 3.4028235e38, -3.4028235e38, 0.5, -0.5], np.float32)
    kind = rng.integers(0, 4, n)
    scores = np.empty(n, np.float32)
    scores[:] = rng.normal(0.0, 4.0, n).astype(np.float32)                      # logits
    wide = (rng.normal(0.0, 1.0, n) * np.exp2(rng.integers(-140, 120, n).astype(np.float64))).astype(np.float32)
    scores[kind == 1] = wide[kind == 1]                                        # every magnitude incl. denormals
    scores[kind == 2] = palette[rng.integers(0, palette.shape[0], n)][kind == 2]  # special values, many ties
    tie = kind == 3                                                            # exact copies of other boxes' scores
    scores[tie] = scores[rng.integers(0, n, n)][tie]
    assert not np.any(np.isnan(scores))
    return scores


def make_config(index: int, frames: int | None = None) -> Workload:
    """Build configuration ``index`` (0..4).  ``frames`` truncates the batched
    configurations (2 and 4) to their first frames; it is ignored elsewhere."""
    if index == 0:
        b, s = clustered_frame(0, 64, 1920, 1080, 32.0, 256.0)
        return Workload(CONFIG_NAMES[0], b[None], s[None], 0.5)
    if index == 1:
        b, s = clustered_frame(1, 256, 3840, 2160, 24.0, 384.0)
        return Workload(CONFIG_NAMES[1], b[None], s[None], 0.5)
    if index == 2:
        f = 64 if frames is None else frames
        fr = [clustered_frame(1000 + k, 64, 1920, 1080, 32.0, 256.0) for k in range(f)]
        return Workload(CONFIG_NAMES[2], np.stack([x[0] for x in fr]), np.stack([x[1] for x in fr]), 0.5)
    if index == 3:
        b, s = crowd_frame(3)
        return Workload(CONFIG_NAMES[3], b[None], s[None], 0.3)
    if index == 4:
        f = 256 if frames is None else frames
        fr = [anchor_frame(4000 + k) for k in range(f)]
        return Workload(CONFIG_NAMES[4], np.stack([x[0] for x in fr]), np.stack([x[1] for x in fr]), 0.45)
    raise ValueError(f"no configuration {index}")
