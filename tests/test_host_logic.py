"""The library's host-checkable logic without a GPU: the numbering of the map step's work
units (a float square root with an integer correction, swept for every unit a launch can
hold), the unit counts, the sort keys on every kind of score, the workspace layout against
nms_workspace_bytes, and the pair test compiled by a plain host compiler -- all built from
the same headers the kernels include, with g++ and with the sanitizers on."""
import os
import subprocess
from fractions import Fraction

import numpy as np
import pytest

from workloads import random_frame, scores_of_every_kind

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER_SOURCE = os.path.join(ROOT, "tests", "host", "host_logic_driver.cpp")
MAX_MAP_WORKGROUPS = 16777215   # NMS_MAX_MAP_WORKGROUPS of include/nms.h
MAP_WAVES = 4                   # wavefronts (work units) per workgroup of the map step


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = tmp_path_factory.mktemp("host") / "host_logic_driver"
    subprocess.run(["g++", "-std=c++17", "-O2", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-ffp-contract=off", DRIVER_SOURCE, "-o", str(exe)], check=True)
    return str(exe)


def run(driver, *args, stdin=None):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1")
    proc = subprocess.run([driver, *args], input=stdin, capture_output=True, text=True, env=env)
    assert proc.returncode == 0, proc.stderr[-2000:]
    assert "runtime error" not in proc.stderr and "AddressSanitizer" not in proc.stderr, proc.stderr[-2000:]
    return proc.stdout


def test_header_constants_match():
    text = open(os.path.join(ROOT, "include", "nms.h")).read()
    assert f"#define NMS_MAX_MAP_WORKGROUPS {MAX_MAP_WORKGROUPS}" in text
    assert "constexpr int kMapWaves = 4;" in open(os.path.join(ROOT, "paper_2502_00535_amd", "csrc", "kernels", "map.h")).read()


def test_unit_numbering_for_every_unit_a_launch_can_hold(driver):
    out = run(driver, "triangle", str(MAX_MAP_WORKGROUPS * MAP_WAVES)).split("\n")
    assert out[0] == "first_mismatch -1 -1 -1", out[0]
    assert out[1] == "unit_count_mismatches 0"
    assert out[2] == "last_unit_mismatches 0"


def test_small_frames_shares_fit_the_kernels(driver):
    """Every batch shape the one-launch sort-free kernels take (frames up to 4200 boxes, up to 70,000 frames): a
    workgroup's share of victims fits its tables, no workgroup is without a tile, and nms_route_for names the route."""
    out = run(driver, "shares").strip().split("\n")
    taken, bad = int(out[-1].split()[1]), int(out[-1].split()[3])
    assert bad == 0, out
    assert taken > 100000


def test_workspace_layout_matches_the_size_helper(driver):
    import paper_2502_00535_amd.binding as nms

    cases = [(1, 1), (63, 1), (64, 3), (65, 2), (1000, 7), (1024, 64), (4096, 256), (4097, 1), (5000, 3), (16384, 1),
             (16384, 40), (65536, 1), (65536, 9), (300, 65535)]
    text = "".join(f"{n} {f} 4096\n" for n, f in cases)
    rows = [list(map(int, line.split())) for line in run(driver, "layout", stdin=text).strip().split("\n")]
    for (n, f), (order, sorted5, ysc, ytile, tsc, keys, stage, end) in zip(cases, rows):
        n_pad = nms.nms_padded_n(n)
        assert end == nms.nms_workspace_bytes(n, f), (n, f)
        offsets = [order, sorted5, ysc, ytile, tsc, keys, stage, end]
        assert offsets == sorted(offsets) and all(o % 256 == 0 for o in offsets)
        # every part holds what is stored there
        assert sorted5 - order >= 4 * n * f and ysc - sorted5 >= 20 * n_pad * f
        assert ytile - ysc >= 16 * n_pad * f and tsc - ytile >= 4 * (n_pad // 64) * f and keys - tsc >= 4 * n_pad * f
        assert stage - keys == nms.nms_sort_workspace_bytes(n, f)
        assert end - stage == (0 if n <= 4096 else -(-(f * (n_pad // 64) * 32 * 8) // 256) * 256)


def real_key(score, index):
    s = float(score)
    if s == float("inf"):
        return (0, Fraction(0), index)
    if s == float("-inf"):
        return (2, Fraction(0), index)
    return (1, -Fraction(s), index)


@pytest.mark.parametrize("n,seed", [(9, 0), (700, 1), (5000, 2)])
def test_sort_keys_order_every_kind_of_score(driver, tmp_path, n, seed):
    scores = scores_of_every_kind(seed, n)
    path = tmp_path / "scores.bin"
    scores.tofile(path)
    keys = [int(line, 16) for line in run(driver, "keys", str(path)).split()]
    assert len(keys) == n and len(set(keys)) == n
    by_key = sorted(range(n), key=lambda t: keys[t])
    by_definition = sorted(range(n), key=lambda t: real_key(scores[t], t))
    assert by_key == by_definition
    assert all(k != 0xFFFFFFFFFFFFFFFF for k in keys)   # the padding sentinel of the rank step stays free


def test_pair_test_built_by_the_host_compiler(driver, tmp_path, oracle):
    """nms_pair.h through g++ alone: the literal form and the division-free form against the
    oracle's measure, thresholds on and next to overlaps that occur."""
    rng = np.random.default_rng(3)
    boxes, _ = random_frame(5, 120, extent=120, max_side=70, integer=False)
    records, want = [], []
    for _ in range(3000):
        i, j = rng.integers(0, 120, 2)
        q = oracle.overlap(boxes[i], boxes[j])
        theta = np.float32(rng.choice([0.3, 0.5, float(q), float(np.nextafter(q, np.float32(2))), float(np.nextafter(q, np.float32(-1)))]))
        if not (theta > 0):
            theta = np.float32(0.25)
        records.append(np.concatenate([boxes[i], boxes[j], [theta]]).astype(np.float32))
        want.append(0 if q < theta else 1)
    path = tmp_path / "pairs.bin"
    np.stack(records).tofile(path)
    got = [tuple(map(int, line.split())) for line in run(driver, "pairs", str(path)).strip().split("\n")]
    assert [g[0] for g in got] == want
    # the division-free form answers wherever its threshold range applies (-1 = outside: literal form only)
    assert all(g[1] in (-1, w) for g, w in zip(got, want))
    assert sum(1 for g in got if g[1] != -1) > 2500
