"""Helpers shared by the GPU parity tests: device buffers for the C ABI and the
oracle run frame by frame on host threads."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np


def oracle_keep_frames(oracle, boxes, scores, theta, counts=None, workers=16, rule="paper"):
    """oracle.keep (or oracle.greedy_keep) per frame (the C call releases the GIL)
    -> [F, n_max] uint8, zero beyond each frame's count."""
    F, n_max = scores.shape
    out = np.zeros((F, n_max), np.uint8)
    fn = oracle.keep if rule == "paper" else oracle.greedy_keep

    def one(f):
        n = n_max if counts is None else int(counts[f])
        if n > 0:
            out[f, :n] = fn(boxes[f, :n], scores[f, :n], theta)

    with ThreadPoolExecutor(max_workers=workers) as pool:
        list(pool.map(one, range(F)))
    return out


class DeviceFrames:
    """Uploads a batch and owns the output / scratch tensors of every entry point."""

    def __init__(self, nms, boxes, scores, counts=None):
        import torch

        self.torch = torch
        self.nms = nms
        dev = torch.device("cuda:0")
        self.F, self.n_max = scores.shape
        self.n_pad = nms.nms_padded_n(self.n_max)
        self.boxes = torch.from_numpy(np.ascontiguousarray(boxes, np.float32)).to(dev)
        self.scores = torch.from_numpy(np.ascontiguousarray(scores, np.float32)).to(dev)
        self.counts = None if counts is None else torch.from_numpy(np.ascontiguousarray(counts, np.int32)).to(dev)
        F, n_max, n_pad = self.F, self.n_max, self.n_pad
        self.order = torch.full((F, max(n_max, 1)), -7, dtype=torch.int32, device=dev)
        self.sorted5 = torch.full((F, 5 * max(n_pad, 1)), float("nan"), dtype=torch.float32, device=dev)
        self.mask = torch.full((F, max(nms.nms_mask_words(n_max), 1)), -1, dtype=torch.int64, device=dev)
        self.keep = torch.full((F, max(n_max, 1)), 77, dtype=torch.uint8, device=dev)
        self.sort_ws = torch.zeros(max(nms.nms_sort_workspace_bytes(n_max, F), 256), dtype=torch.uint8, device=dev)
        self.run_ws = torch.zeros(max(nms.nms_workspace_bytes(n_max, F), 256), dtype=torch.uint8, device=dev)

    def steps(self, theta):
        """rank -> map -> reduce through the three batched step calls."""
        nms = self.nms
        nms.nms_sort_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, self.order, self.sorted5, self.sort_ws)
        nms.nms_overlap_mask_batched(self.sorted5, self.counts, self.n_max, self.F, theta, self.mask)
        self.keep.fill_(77)
        nms.nms_reduce_batched(self.mask, self.order, self.counts, self.n_max, self.F, self.keep)
        self.torch.cuda.synchronize()
        return self.keep.cpu().numpy()

    def fused(self, theta, want=None):
        """nms_run_batched (automatic route).  With `want`, the ranked, the direct and the
        early-exit route are run as well and all must equal it bit for bit."""
        self.keep.fill_(77)
        self.nms.nms_run_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, theta, self.keep, self.run_ws)
        self.torch.cuda.synchronize()
        got = self.keep.cpu().numpy()
        if want is not None:
            assert np.array_equal(got, want), f"automatic route: {(got != want).sum()} differing keep bits"
            self.keep.fill_(77)
            self.nms.nms_run_ranked_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, theta, self.keep, self.run_ws)
            self.torch.cuda.synchronize()
            ranked = self.keep.cpu().numpy()
            assert np.array_equal(ranked, want), f"ranked route: {(ranked != want).sum()} differing keep bits"
            if self.F * self.n_max * self.n_max <= (1 << 31):  # the direct route is quadratic in full: keep it bounded
                self.keep.fill_(77)
                self.nms.nms_run_direct_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, theta, self.keep)
                self.torch.cuda.synchronize()
                direct = self.keep.cpu().numpy()
                assert np.array_equal(direct, want), f"direct route: {(direct != want).sum()} differing keep bits"
            if 0 < self.n_max:
                # the same rule with eliminated victims dropped from further tests
                self.keep.fill_(77)
                self.nms.nms_run_early_exit_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, theta, self.keep,
                                                    self.run_ws)
                self.torch.cuda.synchronize()
                early = self.keep.cpu().numpy()
                assert np.array_equal(early, want), f"early-exit route: {(early != want).sum()} differing keep bits"
        return got

    def early_exit(self, theta):
        """nms_run_early_exit_batched alone."""
        self.keep.fill_(77)
        self.nms.nms_run_early_exit_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, theta, self.keep, self.run_ws)
        self.torch.cuda.synchronize()
        return self.keep.cpu().numpy()

    def greedy(self, theta):
        """Greedy rule two ways: nms_reduce_greedy_batched on the mask of the step calls, and
        the one-call nms_run_greedy_batched.  Returns both keep arrays."""
        nms = self.nms
        nms.nms_sort_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, self.order, self.sorted5, self.sort_ws)
        nms.nms_overlap_mask_batched(self.sorted5, self.counts, self.n_max, self.F, theta, self.mask)
        self.keep.fill_(77)
        nms.nms_reduce_greedy_batched(self.mask, self.order, self.counts, self.n_max, self.F, self.keep)
        self.torch.cuda.synchronize()
        via_steps = self.keep.cpu().numpy()
        ws = self.torch.zeros(max(nms.nms_greedy_workspace_bytes(self.n_max, self.F), 256), dtype=self.torch.uint8,
                              device=self.boxes.device)
        self.keep.fill_(77)
        nms.nms_run_greedy_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, theta, self.keep, ws)
        self.torch.cuda.synchronize()
        one_call = self.keep.cpu().numpy()
        if 0 < self.n_max <= 4096:
            # the mask-free route (one workgroup per frame), whatever the batch size
            self.keep.fill_(77)
            nms.nms_run_greedy_fused_batched(self.boxes, self.scores, self.counts, self.n_max, self.F, theta, self.keep,
                                             self.run_ws)
            self.torch.cuda.synchronize()
            fused = self.keep.cpu().numpy()
            assert np.array_equal(fused, via_steps), f"mask-free greedy route: {(fused != via_steps).sum()} bits differ from the sweep"
        return via_steps, one_call

    def host_order(self):
        return self.order.cpu().numpy()

    def host_sorted5(self):
        return self.sorted5.cpu().numpy()

    def host_mask(self):
        return self.mask.cpu().numpy().view(np.uint64)
