#!/usr/bin/env python3
"""Benchmark of the NMS hot path on one MI355X.

A step = one pass of the whole path (rank -> pair tests with the row reduction
folded in) over one batch of synthetic frames already resident in HBM.  The
headline workload is configuration 4 (256 frames x 4096 SSD-style anchors, theta
0.45); `value` is evaluated pair tests per second, F * n(n-1)/2 per step.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel (the pair-test kernel) against the FP32 vector peak
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload
  extra         per-kernel split, the three-step (mask) pipeline, and the single-frame
                latencies of the other configurations (us/frame at 1024 boxes etc.)
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FLOPS_PER_PAIR = 13            # ALGORITHMIC: min,max,sub,add,max0 per axis (10) + mul + div + compare
VALU_PER_PAIR = 10             # EXECUTED by the fused kernel per pair: min,max,sub,add (x), min,max,sub,add+clamp (y), mul, cmp
PEAK_FP32_VECTOR_TFLOPS = 157.3  # MI355X datasheet: 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz x 2 (every instruction an FMA)
PEAK_HBM_GBS = 8000.0

VALU_SOURCE = os.path.join(ROOT, "bench_valu.hip")
VALU_LIBRARY = os.path.join(ROOT, "libbench_valu.so")
# probes 0..6 of bench_valu.hip are the pair test's own instructions: which issue class each belongs to
PAIR_TEST_PROBES = {"full_rate": (0, 1, 2, 3), "half_rate": (4, 5, 6)}
PAIR_TEST_MIX_PROBE = 7   # the ten instructions together, as the fused kernel issues them
# how many of the ten instructions per pair fall in each class (sub, add, sub, add+clamp, mul | 2 min, 2 max, cmp)
PAIR_TEST_MIX = {"full_rate": 5, "half_rate": 5}


class HipEvents:
    """Raw HIP events through ctypes (events that the library records itself)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.made = []

    def create(self) -> int:
        ev = ctypes.c_void_p()
        assert self.hip.hipEventCreate(ctypes.byref(ev)) == 0
        self.made.append(ev.value)
        return ev.value

    def sync(self, ev):
        assert self.hip.hipEventSynchronize(ctypes.c_void_p(ev)) == 0

    def ms(self, a, b) -> float:
        out = ctypes.c_float()
        assert self.hip.hipEventElapsedTime(ctypes.byref(out), ctypes.c_void_p(a), ctypes.c_void_p(b)) == 0
        return float(out.value)

    def close(self):
        for ev in self.made:
            self.hip.hipEventDestroy(ctypes.c_void_p(ev))
        self.made = []


def build_valu_probes() -> str:
    """Compile the measurement kernels of the calibration leg (gfx950; always compiles)."""
    import subprocess

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = VALU_LIBRARY + f".tmp{os.getpid()}"
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           VALU_SOURCE, "-o", tmp]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + proc.stdout + proc.stderr)
    os.replace(tmp, VALU_LIBRARY)
    return VALU_LIBRARY


class ValuProbes:
    """The probes of bench_valu.hip: issue rate of single VALU instructions over the whole chip."""

    def __init__(self, torch):
        if not os.path.exists(VALU_LIBRARY):
            build_valu_probes()
        self.torch = torch
        L = ctypes.CDLL(VALU_LIBRARY)
        L.valu_probe_count.restype = ctypes.c_int
        L.valu_probe_name.restype = ctypes.c_char_p
        L.valu_probe_name.argtypes = [ctypes.c_int]
        L.valu_probe_lane_ops.restype = ctypes.c_double
        L.valu_probe_lane_ops.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.valu_probe_run.restype = ctypes.c_int
        L.valu_probe_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        self.L = L
        props = torch.cuda.get_device_properties(0)
        self.cus = int(props.multi_processor_count)
        self.blocks = self.cus * 8          # 256 threads each: 8 wavefronts per SIMD
        self.out = torch.empty(self.blocks * 256, dtype=torch.float32, device="cuda:0")
        self.clocks = torch.zeros(2, dtype=torch.int64, device="cuda:0")
        hip = ctypes.CDLL("libamdhip64.so")
        rate = ctypes.c_int(0)
        # hipDeviceAttributeWallClockRate: the constant rate (kHz) of the counter behind wall_clock64()
        attr = 10017
        self.wall_khz = None
        try:
            if hip.hipDeviceGetAttribute(ctypes.byref(rate), ctypes.c_int(attr), ctypes.c_int(0)) == 0 and rate.value > 0:
                self.wall_khz = int(rate.value)
        except Exception:
            pass

    def names(self):
        return [self.L.valu_probe_name(i).decode() for i in range(self.L.valu_probe_count())]

    def measure(self, i, iters=1000, reps=3):
        """Best of `reps` launches: (lane-ops/s, shader-clock ticks, wall-clock ticks of one wavefront)."""
        torch = self.torch
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        run = lambda n: self.L.valu_probe_run(i, self.blocks, n, ctypes.c_void_p(self.out.data_ptr()),
                                              ctypes.c_void_p(self.clocks.data_ptr()), stream)
        assert run(10) == 0
        best = None
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            assert run(iters) == 0
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b)
            ticks = self.clocks.cpu().tolist()
            if best is None or ms < best[0]:
                best = (ms, ticks)
        rate = self.L.valu_probe_lane_ops(i, self.blocks, iters) / (best[0] * 1e-3)
        return rate, best[1][0], best[1][1]

    def calibrate(self):
        """Issue rates of the pair test's own instructions, by class, and the shader clock under that load."""
        names = self.names()
        per_probe, classes, clock_hz = {}, {}, []
        for cls, idxs in PAIR_TEST_PROBES.items():
            rates = []
            for i in idxs:
                rate, shader_ticks, wall_ticks = self.measure(i)
                per_probe[names[i]] = round(rate / 1e12, 3)
                rates.append(rate)
                if self.wall_khz and wall_ticks > 0:
                    clock_hz.append(shader_ticks / wall_ticks * self.wall_khz * 1e3)
            classes[cls] = sum(rates) / len(rates)
        mix_rate, shader_ticks, wall_ticks = self.measure(PAIR_TEST_MIX_PROBE)
        mix_clock = shader_ticks / wall_ticks * self.wall_khz * 1e3 if self.wall_khz and wall_ticks > 0 else None
        return {"per_probe_T_lane_ops_per_s": per_probe, "class_lane_ops_per_s": classes,
                "shader_clock_hz_by_probe": [round(c) for c in clock_hz], "wall_clock_khz": self.wall_khz,
                "compute_units": self.cus, "mix_lane_ops_per_s": mix_rate, "mix_shader_clock_hz": mix_clock}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload configuration of the headline number (0..4)")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-early-exit", action="store_true", help="skip the timing of the automatic / early-exit route")
    ap.add_argument("--cpu-sample-frames", type=int, default=256)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies (a known-size kernel to scale HBM counters by)")
    ap.add_argument("--valu-table", action="store_true",
                    help="print the issue rate of every probed VALU instruction as text and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2502_00535_amd.binding as nms   # raises if the HIP library is missing: no fallback
    from workloads import make_config

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    K, W = args.steps, args.warmup
    events = HipEvents()
    probes = ValuProbes(torch)

    if args.valu_table:
        print(f"{probes.cus} compute units, {probes.blocks} workgroups x 256 threads, 2000 loop trips x 64 instructions per lane")
        for i, name in enumerate(probes.names()):
            rate, shader_ticks, wall_ticks = probes.measure(i, iters=2000)
            clock = shader_ticks / wall_ticks * probes.wall_khz * 1e3 if probes.wall_khz and wall_ticks else float("nan")
            simd_cycles = probes.cus * 4 * clock / (rate / 64) if clock == clock else float("nan")
            print(f"{name:24s} {rate / 1e12:7.2f} T lane-ops/s   shader clock {clock / 1e9:5.3f} GHz   "
                  f"{simd_cycles:4.2f} cycles per wave64 instruction per SIMD")
        return

    def upload(w):
        d = {
            "w": w, "F": w.frames, "n": w.n,
            "boxes": torch.from_numpy(w.boxes).to(dev), "scores": torch.from_numpy(w.scores).to(dev),
            "keep": torch.empty((w.frames, w.n), dtype=torch.uint8, device=dev),
            "ws": torch.empty(nms.nms_workspace_bytes(w.n, w.frames), dtype=torch.uint8, device=dev),
        }
        return d

    def run_fused(d):
        # arguments marshalled once (binding.RunPlan); every call is one nms_run_batched
        if "plan" not in d:
            d["plan"] = nms.RunPlan(d["boxes"], d["scores"], None, d["n"], d["F"], d["w"].theta, d["keep"], d["ws"])
        d["plan"]()

    def mask_set_bits(mask, frames, n):
        """Pairs (victim, outranking box) that eliminate = bits set in the defined words of the mask
        (word (w, r) at w * n_pad + r is written only for w <= r / 64)."""
        n_pad_ = nms.nms_padded_n(n)
        W_ = n_pad_ // 64
        defined = (torch.arange(W_, device=dev)[:, None] <= (torch.arange(n_pad_, device=dev) // 64)[None, :])
        total = 0
        per = max(1, (64 << 20) // (W_ * n_pad_ * 8))  # frames per pass: 64 MiB of mask at a time
        m3 = mask.view(frames, W_, n_pad_)
        for f0 in range(0, frames, per):
            x = torch.where(defined[None], m3[f0:f0 + per], torch.zeros((), dtype=torch.int64, device=dev)).contiguous().view(torch.int32)
            x = x - ((x >> 1) & 0x55555555)
            x = (x & 0x33333333) + ((x >> 2) & 0x33333333)
            x = (x + (x >> 4)) & 0x0F0F0F0F
            x = ((x * 0x01010101) >> 24) & 0xFF
            total += int(x.sum(dtype=torch.int64).item())
        return total

    def time_steps(fn, steps, warmup):
        """`steps` calls between two HIP events on the stream the kernels run on, bracketed by device
        synchronisation on both sides; ms per step (GPU time from the first kernel's start to the last one's end)"""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    def step_percentiles(fn, steps):
        """start-to-start times of consecutive calls (an event before every call and one after the last)"""
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        for k in range(steps):
            evs[k].record()
            fn()
        evs[steps].record()
        torch.cuda.synchronize()
        v = sorted(evs[k].elapsed_time(evs[k + 1]) for k in range(steps))
        return [pct(v, 0.1), pct(v, 0.5), pct(v, 0.9)]

    def pct(v, q):
        return round(v[min(len(v) - 1, int(q * len(v)))], 4)

    # ------------------------------------------------------------------ calibration leg: VALU issue rates, shader clock
    # (first, so that the roofline below is priced in rates measured in this run; about 25 ms of GPU work)
    w = make_config(args.config)
    d = upload(w)
    calib = probes.calibrate()

    # ------------------------------------------------------------------ headline workload
    # Every pair of the ranked triangle is evaluated: the explicit all-pairs route.  (nms_run_batched
    # itself routes a batch of this size to the early-exit kernels, which return the same keep vector
    # from a fraction of the pair tests; that is reported in frames/s under extra.automatic_route.)
    all_pairs_entry = "nms_run_ranked_batched" if w.frames * w.n * w.n > (3 << 24) or w.n > 4096 else "nms_run_batched"
    headline = nms.RunPlan(d["boxes"], d["scores"], None, w.n, w.frames, w.theta, d["keep"], d["ws"], entry=all_pairs_entry)
    pairs = w.pair_tests

    # Order of the legs.  After a few milliseconds of idle time this GPU runs the pair-test kernel at
    # 0.50 ms and comes down to its steady 0.44 ms over the next thirty launches or so (clock
    # management; other kinds of load do not count).  The per-step percentiles (at least 60 steps)
    # therefore run first; the W warm-up steps and the K timed steps follow them directly, and the
    # per-kernel leg comes last, when the clocks have long settled.
    step_p = step_percentiles(headline, max(K, 60))
    ms_per_step = time_steps(headline, K, W)
    value = pairs / (ms_per_step * 1e-3)
    t0 = time.perf_counter()
    for _ in range(K):
        headline()
    torch.cuda.synchronize()
    host_ms_per_step = (time.perf_counter() - t0) * 1e3 / K
    keep_gpu = d["keep"].cpu().numpy()

    # per-kernel durations, live, with HIP events recorded by the library between its launches
    # (at most 100 steps: the event records themselves cost a few microseconds between kernels, which
    # adds up in the queue of a longer run)
    KP = min(max(K, 20), 100)
    ev = [[events.create() for _ in range(3)] for _ in range(KP)]
    for k in range(KP):
        nms.nms_run_batched_profiled(d["boxes"], d["scores"], None, d["n"], d["F"], w.theta, d["keep"], d["ws"], ev[k])
    torch.cuda.synchronize()
    rank_ms = sum(events.ms(e[0], e[1]) for e in ev) / KP
    map_all = sorted(events.ms(e[1], e[2]) for e in ev)
    map_ms = sum(map_all) / KP
    events.close()

    achieved_tflops = FLOPS_PER_PAIR * pairs / (map_ms * 1e-3) / 1e12
    rates = calib["class_lane_ops_per_s"]
    # the ceiling of the instruction mix: the ten instructions of a pair issued back to back from registers
    # (measured together), and the same summed from the single-instruction rates of the two classes
    issue_bound_ms = pairs * VALU_PER_PAIR / calib["mix_lane_ops_per_s"] * 1e3
    issue_bound_classes_ms = pairs * sum(PAIR_TEST_MIX[c] / rates[c] for c in PAIR_TEST_MIX) * 1e3
    roofline = {
        "kernel": "map_fused_kernel<fast, 4 victim tiles per unit> (pair tests + row reduction)",
        "bound": "alu",
        "achieved": round(achieved_tflops, 3),
        "peak": PEAK_FP32_VECTOR_TFLOPS,
        "unit": "TFLOP/s",
        "frac": round(achieved_tflops / PEAK_FP32_VECTOR_TFLOPS, 4),
        "traffic": None,
        "traffic_source": None,
        "kernel_ms": round(map_ms, 4),
        "kernel_ms_p10_p50_p90": [pct(map_all, 0.1), pct(map_all, 0.5), pct(map_all, 0.9)],
        "flops_per_pair_algorithmic": FLOPS_PER_PAIR,
        "valu_instructions_per_pair_executed": VALU_PER_PAIR,
        "pairs_per_launch": pairs,
        "measured_valu_lane_ops_per_s": {k: round(v, 1) for k, v in rates.items()},
        "measured_valu_T_lane_ops_per_s_by_instruction": calib["per_probe_T_lane_ops_per_s"],
        "measured_pair_test_mix_lane_ops_per_s": round(calib["mix_lane_ops_per_s"], 1),
        "shader_clock_hz_measured": {"pair_test_mix_probe": calib["mix_shader_clock_hz"],
                                     "single_instruction_probes": calib["shader_clock_hz_by_probe"]},
        "compute_units": calib["compute_units"],
        "valu_issue_bound_ms": round(issue_bound_ms, 4),           # the ten-instruction mix at its measured issue rate
        "frac_of_valu_issue_bound": round(issue_bound_ms / map_ms, 4),
        "valu_issue_bound_ms_from_single_instruction_rates": round(issue_bound_classes_ms, 4),
    }
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):
        try:
            t = json.load(open(traffic_file))
            roofline["traffic"] = t.get(w.name, {}).get("map_fused_kernel_bytes")
            if roofline["traffic"] is not None:
                roofline["traffic_source"] = "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not this run)"
        except Exception:
            pass

    extra = {
        "headline_entry_point": all_pairs_entry,
        "ms_per_step_start_to_start_p10_p50_p90": step_p,
        "ms_per_step_host_clock": round(host_ms_per_step, 4),
        "rank_kernel_ms": round(rank_ms, 4),
        "map_kernel_ms": round(map_ms, 4),
        "frames_per_s": round(w.frames / (ms_per_step * 1e-3), 1),
        "us_per_frame": round(ms_per_step * 1e3 / w.frames, 3),
        "survivors": int(keep_gpu.sum()),
    }

    # ------------------------------------------------------------------ three-step (mask) pipeline on the same workload
    if not args.no_extra:
        n_pad = nms.nms_padded_n(w.n)
        order = torch.empty((w.frames, w.n), dtype=torch.int32, device=dev)
        sorted5 = torch.empty((w.frames, 5 * n_pad), dtype=torch.float32, device=dev)
        mask = torch.empty((w.frames, nms.nms_mask_words(w.n)), dtype=torch.int64, device=dev)
        keep3 = torch.empty((w.frames, w.n), dtype=torch.uint8, device=dev)
        sws = torch.empty(max(nms.nms_sort_workspace_bytes(w.n, w.frames), 256), dtype=torch.uint8, device=dev)

        def run_steps():
            nms.nms_sort_batched(d["boxes"], d["scores"], None, w.n, w.frames, order, sorted5, sws)
            nms.nms_overlap_mask_batched(sorted5, None, w.n, w.frames, w.theta, mask)
            nms.nms_reduce_batched(mask, order, None, w.n, w.frames, keep3)

        steps3 = min(100, max(5, K // 5))
        ms3 = time_steps(run_steps, steps3, 2)
        te = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        split = [0.0, 0.0, 0.0]
        for _ in range(steps3):
            te[0].record()
            nms.nms_sort_batched(d["boxes"], d["scores"], None, w.n, w.frames, order, sorted5, sws)
            te[1].record()
            nms.nms_overlap_mask_batched(sorted5, None, w.n, w.frames, w.theta, mask)
            te[2].record()
            nms.nms_reduce_batched(mask, order, None, w.n, w.frames, keep3)
            te[3].record()
            torch.cuda.synchronize()
            for i in range(3):
                split[i] += te[i].elapsed_time(te[i + 1]) / steps3
        tri_bytes = w.frames * (n_pad // 64) * (n_pad // 64 + 1) // 2 * 512
        extra["three_step"] = {
            "ms_per_step": round(ms3, 4),
            "pair_tests_per_s": round(pairs / (ms3 * 1e-3), 1),
            "sort_ms": round(split[0], 4), "overlap_mask_ms": round(split[1], 4), "reduce_ms": round(split[2], 4),
            "mask_write_GBs": round(tri_bytes / (split[1] * 1e-3) / 1e9, 1),
            "mask_read_GBs": round(tri_bytes / (split[2] * 1e-3) / 1e9, 1),
            "frac_hbm_peak_reduce": round(tri_bytes / (split[2] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "keep_equals_fused": bool(torch.equal(keep3, d["keep"])),
            "eliminating_pairs_per_frame": round(mask_set_bits(mask, w.frames, w.n) / w.frames, 1),
        }
        # the selectable classic greedy rule on the same mask (sequential sweep, one workgroup per frame)
        keep_g = torch.empty((w.frames, w.n), dtype=torch.uint8, device=dev)
        tg = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        sweep_ms = 0.0
        for _ in range(steps3):
            tg[0].record()
            nms.nms_reduce_greedy_batched(mask, order, None, w.n, w.frames, keep_g)
            tg[1].record()
            torch.cuda.synchronize()
            sweep_ms += tg[0].elapsed_time(tg[1]) / steps3
        ws_g = torch.empty(nms.nms_greedy_workspace_bytes(w.n, w.frames), dtype=torch.uint8, device=dev)
        keep_g1 = torch.empty((w.frames, w.n), dtype=torch.uint8, device=dev)
        ms_g = time_steps(lambda: nms.nms_run_greedy_batched(d["boxes"], d["scores"], None, w.n, w.frames, w.theta,
                                                             keep_g1, ws_g), steps3, 2)
        greedy_same = bool(torch.equal(keep_g1, keep_g))
        del ws_g, keep_g1
        extra["greedy_rule"] = {
            # the one call takes the mask-free route on this batch (one workgroup per frame, only
            # survivors are used as outranking boxes): most of the pair grid is never evaluated, so
            # it is quoted in frames/s, not pair tests/s
            "nms_run_greedy_batched_ms_per_step": round(ms_g, 4),
            "frames_per_s": round(w.frames / (ms_g * 1e-3), 1),
            "one_call_equals_steps": greedy_same,
            "sweep_ms": round(sweep_ms, 4),
            "ms_per_step_rank_mask_sweep": round(split[0] + split[1] + sweep_ms, 4),
            "survivors": int(keep_g.sum().item()),
            "survivors_paper_rule": int(d["keep"].sum().item()),
        }
        del order, sorted5, mask, keep3, keep_g

        # -------------------------------------------------------------- selectable variants on the same workload
        # (literal division form, one tile per wavefront, mask in memory: a coverage path, not the tuned one)
        ws_ex = torch.empty(nms.nms_ex_workspace_bytes(w.n, w.frames), dtype=torch.uint8, device=dev)
        keep_ex = torch.empty((w.frames, w.n), dtype=torch.uint8, device=dev)
        variants = {}
        # "defaults" is routed to nms_run_batched; "strict_compare" is the variants' kernel in its plainest form
        for label, kw in (("defaults", {}), ("strict_compare", dict(compare="gt")),
                          ("iou_greedy_offset0", dict(rule="greedy", measure="iou", pixel_offset=0.0)),
                          ("iou_paper_rule", dict(measure="iou"))):
            fn = lambda: nms.nms_run_ex_batched(d["boxes"], d["scores"], None, w.n, w.frames, w.theta, keep_ex, ws_ex, **kw)
            ms_v = time_steps(fn, steps3, 2)
            variants[label] = {"ms_per_step": round(ms_v, 4), "pair_tests_per_s": round(pairs / (ms_v * 1e-3), 1),
                               "survivors": int(keep_ex.sum().item())}
        variants["defaults_equal_fused"] = None
        nms.nms_run_ex_batched(d["boxes"], d["scores"], None, w.n, w.frames, w.theta, keep_ex, ws_ex)
        variants["defaults_equal_fused"] = bool(torch.equal(keep_ex, d["keep"]))
        extra["variants_nms_run_ex_batched"] = variants
        del ws_ex, keep_ex

        # -------------------------------------------------------------- the other configurations (latency view)
        others = {}
        for idx in (0, 1, 2, 3):
            if idx == args.config:
                continue
            wo = make_config(idx)
            do = upload(wo)
            steps_o = 200 if wo.n <= 4096 else 50
            ms_o = time_steps(lambda: run_fused(do), steps_o, 10)
            # what one caller sees for one call: enqueue -> synchronise
            lat = []
            for _ in range(30):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                run_fused(do)
                torch.cuda.synchronize()
                lat.append((time.perf_counter() - t0) * 1e6)
            lat.sort()
            keep_o = do["keep"].cpu().numpy()
            # the classic greedy rule on the same frames, for the structure of the workload
            ws_go = torch.empty(nms.nms_greedy_workspace_bytes(wo.n, wo.frames), dtype=torch.uint8, device=dev)
            keep_go = torch.empty((wo.frames, wo.n), dtype=torch.uint8, device=dev)
            nms.nms_run_greedy_batched(do["boxes"], do["scores"], None, wo.n, wo.frames, wo.theta, keep_go, ws_go)
            torch.cuda.synchronize()
            # bits set in the mask of the three step calls: how many pairs eliminate
            order_o = torch.empty((wo.frames, wo.n), dtype=torch.int32, device=dev)
            sorted5_o = torch.empty((wo.frames, 5 * nms.nms_padded_n(wo.n)), dtype=torch.float32, device=dev)
            sws_o = torch.empty(max(nms.nms_sort_workspace_bytes(wo.n, wo.frames), 256), dtype=torch.uint8, device=dev)
            mask_o = torch.empty((wo.frames, nms.nms_mask_words(wo.n)), dtype=torch.int64, device=dev)
            nms.nms_sort_batched(do["boxes"], do["scores"], None, wo.n, wo.frames, order_o, sorted5_o, sws_o)
            nms.nms_overlap_mask_batched(sorted5_o, None, wo.n, wo.frames, wo.theta, mask_o)
            torch.cuda.synchronize()
            structure = {"survivors_per_frame": round(float(keep_o.sum()) / wo.frames, 1),
                         "survivors_per_frame_greedy_rule": round(float(keep_go.sum().item()) / wo.frames, 1),
                         "eliminating_pairs_per_frame": round(mask_set_bits(mask_o, wo.frames, wo.n) / wo.frames, 1)}
            del order_o, sorted5_o, sws_o, mask_o
            if not args.no_cpu_baseline:
                from oracle import Oracle

                orc_o = Oracle()
                t0 = time.perf_counter()
                differing = sum(int((orc_o.keep(wo.boxes[f], wo.scores[f], np.float32(wo.theta)) != keep_o[f]).sum())
                                for f in range(wo.frames))
                structure["differing_keep_bits_vs_oracle"] = differing
                structure["oracle_1_core_us_per_frame"] = round((time.perf_counter() - t0) * 1e6 / wo.frames, 1)
            del ws_go, keep_go
            route = {0: "direct (one launch)", 1: "all pairs (rank + fused pair-test kernel)",
                     2: "two launches (best 2048 ranks, then the victims still alive)", 3: "early exit",
                     4: "small frames (one launch, no sort: picked boxes, then the victims still alive against the frame)"}[nms.nms_route(wo.n, wo.frames)]
            skips = nms.nms_route(wo.n, wo.frames) >= 2
            ms_pairs = ms_o  # the time in which every pair of the ranked triangle is evaluated
            if skips:
                # the automatic route skips tests of decided victims here: time the all-pairs route beside it
                ms_all = time_steps(lambda: nms.nms_run_ranked_batched(do["boxes"], do["scores"], None, wo.n, wo.frames, wo.theta,
                                                                       do["keep"], do["ws"]), steps_o, 10)
                structure["all_pairs_route_us_per_frame"] = round(ms_all * 1e3 / wo.frames, 3)
                structure["all_pairs_route_equals_automatic"] = bool(np.array_equal(do["keep"].cpu().numpy(), keep_o))
                ms_pairs = ms_all
            others[wo.name] = {
                "route_of_nms_run_batched": route,
                **structure,
                "us_per_frame": round(ms_o * 1e3 / wo.frames, 3),
                "frames_per_s": round(wo.frames / (ms_o * 1e-3), 1),
                # pair tests that are evaluated: through the all-pairs route where the automatic one skips some
                "pair_tests_per_s": round(wo.pair_tests / (ms_pairs * 1e-3), 1),
                "pair_tests_per_s_is_of": "the all-pairs route" if skips else "this route (it evaluates every pair)",
                "frac_fp32_vector_peak": round(FLOPS_PER_PAIR * wo.pair_tests / (ms_pairs * 1e-3) / 1e12 / PEAK_FP32_VECTOR_TFLOPS, 5),
                "sync_call_us_median": round(lat[len(lat) // 2], 2),
            }
        extra["other_configs"] = others
        extra["us_per_frame_at_1024_boxes"] = others.get("cfg0_1x1024_1080p", {}).get("us_per_frame")

        # -------------------------------------------------------------- the paper's own layout (byte matrix, k-partition reduce)
        # capacity D_max = 4096 as in the paper's experiments; n = the detection counts of its
        # discrete-GPU table (1027, 2895) and the full capacity; k swept as in its k experiment
        w1 = make_config(1)
        cap = 4096
        Bm = torch.empty((cap, cap), dtype=torch.uint8, device=dev)
        Vm = torch.empty(cap, dtype=torch.uint8, device=dev)
        b1 = torch.from_numpy(w1.boxes[0]).to(dev)
        s1 = torch.from_numpy(w1.scores[0]).to(dev)

        def event_ms(fn, reps=50):
            for _ in range(5):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        mform = {"capacity": cap, "map_ms": {}, "reduce_ms_by_k": {}}
        for n_m in (1027, 2895, 4096):
            mform["map_ms"][str(n_m)] = round(event_ms(lambda: nms.nms_map_matrix(b1, s1, n_m, cap, w1.theta, Bm)), 4)
        for k_m in (4, 8, 16, 32, 64):
            mform["reduce_ms_by_k"][str(k_m)] = round(event_ms(lambda: nms.nms_reduce_matrix(Bm, cap, k_m, Vm)), 4)
        mform["matrix_bytes"] = cap * cap
        extra["paper_matrix_form"] = mform
        del Bm, Vm

        # -------------------------------------------------------------- the detection counts of the paper's discrete-GPU table
        # (its latencies there: 0.107 / 0.324 / 1.313 ms on a GTX 1060 and 0.024 / 0.088 / 0.430 ms on a Tesla T4)
        sizes = {}
        for n_t in (200, 1027, 2895):
            bt = b1[:n_t].contiguous()
            st_ = s1[:n_t].contiguous()
            kt = torch.empty(n_t, dtype=torch.uint8, device=dev)
            wt = torch.empty(nms.nms_workspace_bytes(n_t, 1), dtype=torch.uint8, device=dev)
            plan_t = nms.RunPlan(bt, st_, None, n_t, 1, w1.theta, kt, wt)
            lat_t = []
            for _ in range(30):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                plan_t()
                torch.cuda.synchronize()
                lat_t.append((time.perf_counter() - t0) * 1e6)
            lat_t.sort()
            sizes[str(n_t)] = {"kernel_us_back_to_back": round(event_ms(plan_t, 200) * 1e3, 2),
                               "sync_call_us_median": round(lat_t[len(lat_t) // 2], 2)}
        extra["single_frame_at_the_papers_detection_counts"] = sizes

        # -------------------------------------------------------------- single frames replayed from a HIP graph
        # (the calls only enqueue kernels, so a caller can take the per-call launch cost out: 100 calls
        # of nms_run_batched on one frame captured once, then replayed)
        graphed = {}
        for idx in (0, 1):
            wg = make_config(idx)
            dg = upload(wg)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            calls = 100
            with torch.cuda.stream(side):
                plan_g = nms.RunPlan(dg["boxes"], dg["scores"], None, wg.n, wg.frames, wg.theta, dg["keep"], dg["ws"])
                plan_g()
                side.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    for _ in range(calls):
                        plan_g()
            torch.cuda.synchronize()
            us = time_steps(graph.replay, 20, 3) * 1e3 / calls
            graphed[wg.name] = {"us_per_frame": round(us, 3), "calls_per_graph": calls}
            del dg
        extra["single_frame_calls_replayed_from_a_hip_graph"] = graphed

    # -------------------------------------------------------------- what a caller of nms_run_batched gets
    # (the automatic route: on a batch of this size the early-exit kernels, same keep vector from a
    # fraction of the pair tests -- quoted in frames/s, never in pair tests/s: the headline counts pairs
    # that are evaluated, all of them.  Timed after everything else: a tensor allocated before the
    # three-step pipeline shifts where its 512 MiB mask lands, and the mask-writing kernel's time with it)
    if not args.no_early_exit:
        keep_e = torch.empty((w.frames, w.n), dtype=torch.uint8, device=dev)
        steps_e = min(200, max(20, K))
        auto = nms.RunPlan(d["boxes"], d["scores"], None, w.n, w.frames, w.theta, keep_e, d["ws"])
        ms_a = time_steps(auto, steps_e, 5)
        same_auto = bool(torch.equal(keep_e, d["keep"]))
        keep_e.fill_(9)
        early = nms.RunPlan(d["boxes"], d["scores"], None, w.n, w.frames, w.theta, keep_e, d["ws"],
                            entry="nms_run_early_exit_batched")
        ms_e = time_steps(early, steps_e, 5)
        extra["automatic_route"] = {
            "nms_run_batched_ms_per_step": round(ms_a, 4),
            "frames_per_s": round(w.frames / (ms_a * 1e-3), 1),
            "us_per_frame": round(ms_a * 1e3 / w.frames, 3),
            "equals_all_pairs_route": same_auto,
            "speedup_over_all_pairs": round(ms_per_step / ms_a, 3),
            "nms_run_early_exit_batched_ms_per_step": round(ms_e, 4),
            "early_exit_equals_all_pairs_route": bool(torch.equal(keep_e, d["keep"])),
        }
        del keep_e

    if args.calibrate_copy:
        src = torch.empty(64 << 20, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        extra["calibration_copy_bytes_read_and_written_each"] = src.numel() * 4
        del src, dst

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    cpu_baseline = None
    if not args.no_cpu_baseline:
        import numpy as np
        from oracle import Oracle

        orc = Oracle()
        sample = min(w.frames, max(1, args.cpu_sample_frames))
        t0 = time.perf_counter()
        differing = 0
        for f in range(sample):
            k = orc.keep(w.boxes[f], w.scores[f], np.float32(w.theta))
            differing += int((k != keep_gpu[f]).sum())
        cpu_s = time.perf_counter() - t0
        sample_pairs = sample * (w.n * (w.n - 1) // 2)
        cpu_baseline = {
            "value": round(sample_pairs / cpu_s, 1),
            "unit": "pair-tests/s",
            "cores": 1,
            "kind": "oracle",
            "sample": f"first {sample} of {w.frames} frames of {w.name}, single thread, {cpu_s:.2f} s",
            "differing_keep_bits_vs_gpu": differing,
        }
        # the same oracle function, one frame per task, on all host cores the box gives this process
        from concurrent.futures import ThreadPoolExecutor

        threads = max(1, min(16, len(os.sched_getaffinity(0))))
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=threads) as pool:  # the C call releases the GIL
            list(pool.map(lambda f: orc.keep(w.boxes[f], w.scores[f], np.float32(w.theta)), range(sample)))
        par_s = time.perf_counter() - t0
        cpu_baseline["frames_parallel"] = {"value": round(sample_pairs / par_s, 1), "unit": "pair-tests/s",
                                           "cores": threads, "seconds": round(par_s, 2)}

    line = {
        "metric": "pair-tests/s (batched)",
        "value": round(value, 1),
        "unit": "pair-tests/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "frames": w.frames, "boxes_per_frame": w.n, "threshold": w.theta,
                   "path": f"{all_pairs_entry}: every pair of the ranked triangle evaluated (rank + fused pair-test/reduce "
                           "kernels); nms_run_batched's own route for this size is under extra.automatic_route"},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
