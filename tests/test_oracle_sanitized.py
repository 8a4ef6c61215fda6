"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only; no
GPU).  The oracle source is built into a small program with -fsanitize=address,undefined,
every exported function is run on seeded frames (empty, single, ragged sizes, ties, labels,
the square-box form with spare capacity), and the dump must be free of sanitizer reports and
equal, byte for byte, what the ordinary -O2 build returns."""
import os
import subprocess

import numpy as np
import pytest

from workloads import random_frame, scores_of_every_kind

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER_SOURCE = os.path.join(ROOT, "tests", "host", "oracle_sanitizer_driver.c")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = tmp_path_factory.mktemp("asan") / "oracle_sanitized"
    subprocess.run(["gcc", "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-ffp-contract=off", "-fno-fast-math", "-fexcess-precision=standard", "-msse2", "-mfpmath=sse",
                    DRIVER_SOURCE, "-o", str(exe)], check=True)
    return str(exe)


def parse(dump):
    out = {}
    for line in dump.strip().split("\n"):
        tag, size, *hexa = line.split(" ")
        out[tag] = bytes.fromhex(hexa[0]) if hexa and hexa[0] else b""
        assert len(out[tag]) == int(size)
    return out


@pytest.mark.parametrize("n,seed,kind", [(0, 0, "int"), (1, 1, "int"), (2, 2, "float"), (64, 3, "int"), (65, 4, "float"),
                                         (200, 5, "special_scores"), (333, 6, "float")])
def test_oracle_under_sanitizers(driver, oracle, tmp_path, n, seed, kind):
    rng = np.random.default_rng(seed)
    if n:
        boxes, scores = random_frame(seed, n, extent=150, max_side=60, integer=(kind == "int"), score_levels=max(2, n // 3))
        if kind == "special_scores":
            scores = scores_of_every_kind(seed, n)
    else:
        boxes, scores = np.zeros((0, 4), np.float32), np.zeros(0, np.float32)
    classes = rng.integers(0, 3, n).astype(np.int32)
    theta = np.float32(0.4)
    dmax, k = 64, 4
    m = min(n, 40)
    D = np.zeros((dmax, 4), np.float32)
    if m:
        side = rng.integers(3, 30, m).astype(np.float32)
        D[:m] = np.stack([np.floor(boxes[:m, 0]), np.floor(boxes[:m, 1]), side,
                          (rng.permutation(m) + 1).astype(np.float32) / np.float32(m + 1)], axis=1)
    path = tmp_path / "case.bin"
    with open(path, "wb") as fh:
        fh.write(np.array([n, dmax, k], np.int32).tobytes())
        fh.write(np.array([theta], np.float32).tobytes())
        fh.write(boxes.astype(np.float32).tobytes())
        fh.write(scores.astype(np.float32).tobytes())
        fh.write(classes.tobytes())
        fh.write(D.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    proc = subprocess.run([driver, str(path)], capture_output=True, text=True, env=env)
    assert proc.returncode == 0, proc.stderr[-3000:]
    assert "runtime error" not in proc.stderr and "Sanitizer" not in proc.stderr, proc.stderr[-3000:]
    got = parse(proc.stdout)

    # the ordinary build of the same source, through its ctypes front end
    assert got["keep"] == oracle.keep(boxes, scores, theta).tobytes()
    assert got["greedy"] == oracle.greedy_keep(boxes, scores, theta).tobytes()
    order = oracle.order(scores)
    assert got["order"] == order.tobytes()
    if n:
        B = oracle.map(boxes, scores, theta)
        assert got["map"] == B.tobytes() and got["reduce"] == oracle.reduce(B).tobytes()
        assert got["ranked"] == oracle.ranked_boxes(boxes, order).tobytes()
        assert got["elims"] == oracle.ranked_eliminations(boxes, order, theta).tobytes()
        assert got["words"] == oracle.ranked_elimination_words(boxes, order, theta).tobytes()
    for combo in range(64):
        want = oracle.keep_ex(boxes, scores, theta, rule="greedy" if combo & 1 else "paper",
                              measure="iou" if combo & 2 else "outranking_area", compare="gt" if combo & 4 else "ge",
                              ties="ignore" if combo & 8 else "index", pixel_offset=0.0 if combo & 16 else 1.0,
                              classes=classes if combo & 32 else None)
        assert got[f"ex{combo}"] == want.tobytes(), f"combination {combo}"
    Bs, Vs = oracle.alg12_square(D, theta, k)
    assert got["squareB"] == Bs.tobytes() and got["squareV"] == Vs.tobytes()
